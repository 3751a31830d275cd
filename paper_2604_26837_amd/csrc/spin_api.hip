// Context, sizing and status plumbing of the C ABI (host side).
#include <math.h>
#include <new>
#include <string.h>

#include "spin_common.h"

static inline int32_t cdiv32(int64_t a, int64_t b) { return (int32_t)((a + b - 1) / b); }

extern "C" int spin_create(const spin_config *c, spin_ctx **out) {
  if (!c || !out) return SPIN_ERR_INVALID;
  if (c->max_batch <= 0 || c->num_q_heads <= 0 || c->num_kv_heads <= 0 || c->max_context <= 0 ||
      c->topk < 0 || c->sink_pages < 0 || c->recent_pages < 0 || c->leaf_entries <= 0 ||
      c->lru_timestamps < 0 || c->decode_splits < 0)
    return SPIN_ERR_INVALID;
  if (c->num_q_heads % c->num_kv_heads != 0) return SPIN_ERR_INVALID;
  if (c->head_dim != SPIN_HEAD_DIM || c->page_tokens != SPIN_PAGE_TOKENS) return SPIN_ERR_UNSUPPORTED;
  const int32_t group = c->num_q_heads / c->num_kv_heads;
  if (group > 16) return SPIN_ERR_UNSUPPORTED;
  const int32_t tp = c->partition_tokens;
  if (tp <= 0) return SPIN_ERR_INVALID;
  if (!((tp < 16 && 16 % tp == 0) || (tp >= 16 && tp % 16 == 0))) return SPIN_ERR_UNSUPPORTED;
  if (c->lru_timestamps > 256) return SPIN_ERR_UNSUPPORTED;
  if (c->lru_policy != 0 && c->lru_policy != 1) return SPIN_ERR_INVALID;
  if (c->decode_depth != 0 && (c->decode_depth < 2 || c->decode_depth > 4)) return SPIN_ERR_INVALID;
  if (c->variable_partitions && tp < 16) return SPIN_ERR_UNSUPPORTED;
  // the key sketch is one row per token: every SKETCH kernel takes summary row == token
  if (c->score_kind == SPIN_SCORE_SKETCH && tp != 1) return SPIN_ERR_UNSUPPORTED;
  if (c->score_tiles_per_wg < 0 || (c->score_waves != 0 && c->score_waves != 1 && c->score_waves != 2 && c->score_waves != 4 && c->score_waves != 8))
    return SPIN_ERR_INVALID;

  spin_ctx *x = new (std::nothrow) spin_ctx;
  if (!x) return SPIN_ERR_INVALID;
  memset(x, 0, sizeof(*x));
  x->cfg = *c;
  x->group = group;
  x->max_rows = c->max_batch * c->num_kv_heads;
  x->max_pages = cdiv32(c->max_context, SPIN_PAGE_TOKENS);
  // with variable-length partitions max_context/16 bounds a row's pages and, since a
  // partition owns at least one page, its partitions too
  x->max_parts = c->variable_partitions ? cdiv32(c->max_context, SPIN_PAGE_TOKENS) : cdiv32(c->max_context, tp);
  x->k_token_major = tp < 16 ? 1 : 0;
  x->pages_per_part = tp >= 16 ? tp / 16 : 0;
  x->parts_per_page = tp < 16 ? 16 / tp : 0;

  switch (c->score_kind) {
    case SPIN_SCORE_MINMAX: x->kd = 256; x->rows_per_part = 1; break;
    case SPIN_SCORE_REPMAX:
      // 1 = one mean key per partition (a landmark / centroid), 2 or 4 = means of equal sub-ranges
      if ((c->reps_per_partition != 1 && c->reps_per_partition != 2 && c->reps_per_partition != 4) ||
          tp % c->reps_per_partition != 0) { delete x; return SPIN_ERR_UNSUPPORTED; }
      x->kd = 128; x->rows_per_part = c->reps_per_partition; break;
    case SPIN_SCORE_SKETCH:
      if (c->sketch_channels != 16) { delete x; return SPIN_ERR_UNSUPPORTED; }
      x->kd = 16; x->rows_per_part = 1; break;
    default: delete x; return SPIN_ERR_INVALID;
  }

  // upper bound of the partitions all of whose pages are forced
  int64_t forced_max;
  if (c->variable_partitions) {
    forced_max = c->sink_pages + c->recent_pages;   // partitions may be as small as one page
  } else if (tp >= 16) {
    const int32_t m = x->pages_per_part;
    forced_max = cdiv32(c->sink_pages, m) + cdiv32(c->recent_pages, m) + 1;
    if (c->sink_pages + c->recent_pages == 0) forced_max = 0;
  } else {
    forced_max = (int64_t)(c->sink_pages + c->recent_pages) * x->parts_per_page;
  }
  int64_t sel = c->topk_includes_forced ? (c->topk > forced_max ? c->topk : forced_max)
                                        : (int64_t)c->topk + forced_max;
  if (sel > x->max_parts) sel = x->max_parts;
  if (sel < 1) sel = 1;
  x->sel_stride = (int32_t)sel;
  // forced pages outside every selected partition exist only when a partition spans several pages
  int64_t pg = (tp > 16 || c->variable_partitions) ? sel * x->pages_per_part + c->sink_pages + c->recent_pages : sel;
  if (pg > x->max_pages) pg = x->max_pages;
  if (pg < 1) pg = 1;
  x->page_stride = (int32_t)pg;
  x->dir_stride = cdiv32(x->max_pages, c->leaf_entries);

  if (c->decode_waves != 0 && c->decode_waves != 2 && c->decode_waves != 4 && c->decode_waves != 8) {
    delete x;
    return SPIN_ERR_INVALID;
  }
  x->waves = c->decode_waves ? c->decode_waves : 8;
  // partitions smaller than a page: most pages are fetched in part (a few KiB), so a wavefront
  // keeps two pages in flight instead of one (measured: 53 -> 42 us on 64 rows x 65536 tokens)
  x->depth = c->decode_depth ? c->decode_depth : (tp < 16 ? 3 : 2);
  int32_t splits = c->decode_splits;
  if (splits == 0) {
    // about one 8-wave workgroup on each of the 256 compute units, all resident
    // at once, and at least four pages per wavefront (measured best on MI355X)
    splits = 256 / x->max_rows;
    int32_t cap = x->page_stride / (4 * x->waves);
    if (splits > cap) splits = cap;
    if (splits < 1) splits = 1;
  }
  if (splits > 64) splits = 64;
  x->splits = splits;
  x->scale = c->softmax_scale > 0.f ? c->softmax_scale : 1.0f / sqrtf((float)c->head_dim);
  // the always-attended pages beside stages 2+3: about 16 pages per side workgroup, at most one per split
  // (each leaves a partial that one split's first wavefront starts from)
  x->side_wgs = 0;
  const int32_t forced_pages = c->sink_pages + c->recent_pages;
  if (c->lru_timestamps == 0 && tp >= SPIN_PAGE_TOKENS && !c->variable_partitions && x->max_parts <= 4096 &&
      forced_pages >= 1 && forced_pages <= 1024) {
    int32_t s_wgs = (forced_pages + 15) / 16;
    x->side_wgs = s_wgs > splits ? splits : s_wgs;
  }
  x->pstride = splits + (x->side_wgs > 1 ? x->side_wgs : 1);

  size_t off = SPIN_WS_HEADER;
  x->ws_ticket_off = off;                       // one arrival counter per row, zero between launches
  off += (size_t)x->max_rows * sizeof(int32_t);
  off = (off + 255) & ~(size_t)255;
  // stage 2 of long rows: 4096 counters per row, zero between launches
  if (x->max_parts > 16384 && x->max_parts <= 131072 && !c->variable_partitions) {
    x->ws_hist_off = off;
    off += (size_t)x->max_rows * 4096 * sizeof(int32_t);
  }
  x->ws_zero_bytes = off;
  x->ws_skip_off = off;
  off += (size_t)x->max_rows * 2 * sizeof(int32_t);
  off = (off + 255) & ~(size_t)255;
  // workgroup partials of stage 4: one per split, plus those of the always-attended pages when the launch of
  // stages 2+3 attends them (at least one: the first of two passes over a page list leaves its result there)
  x->ws_ml_off = off;
  off += (size_t)x->max_rows * x->pstride * group * 2 * sizeof(float);
  off = (off + 255) & ~(size_t)255;
  x->ws_acc_off = off;
  off += (size_t)x->max_rows * x->pstride * group * SPIN_HEAD_DIM * sizeof(float);
  x->ws_bytes = (off + 255) & ~(size_t)255;
  // set-up for spin_sparse_decode_static on the device that is current now: its first call then asks the
  // runtime for nothing (a caller may be capturing by then).  Best effort: a context may be created with no
  // GPU present, and the entry point looks the address up itself on a device that was not prepared here.
  (void)spin_static_scratch_prepare();
  *out = x;
  return SPIN_OK;
}

static void prof_release(spin_ctx *ctx) {
  for (int k = 0; k < SPIN_KERNEL_IDS; ++k) {
    if (ctx->prof_ev[k]) {
      for (int i = 0; i < 2 * ctx->prof_cap; ++i)
        if (ctx->prof_ev[k][i]) (void)hipEventDestroy(ctx->prof_ev[k][i]);
      delete[] ctx->prof_ev[k];
      ctx->prof_ev[k] = nullptr;
    }
    ctx->prof_n[k] = 0;
  }
  ctx->prof_cap = 0;
}

extern "C" void spin_destroy(spin_ctx *ctx) {
  if (!ctx) return;
  prof_release(ctx);
  delete ctx;
}

extern "C" int spin_profile_enable(spin_ctx *ctx, int32_t capacity) {
  if (!ctx || capacity < 0 || capacity > (1 << 16)) return SPIN_ERR_INVALID;
  prof_release(ctx);
  if (capacity == 0) return SPIN_OK;
  for (int k = 0; k < SPIN_KERNEL_IDS; ++k) {
    ctx->prof_ev[k] = new (std::nothrow) hipEvent_t[2 * capacity];
    if (!ctx->prof_ev[k]) { prof_release(ctx); return SPIN_ERR_INVALID; }
    for (int i = 0; i < 2 * capacity; ++i) ctx->prof_ev[k][i] = nullptr;
  }
  ctx->prof_cap = capacity;
  for (int k = 0; k < SPIN_KERNEL_IDS; ++k)
    for (int i = 0; i < 2 * capacity; ++i)
      if (hipEventCreate(&ctx->prof_ev[k][i]) != hipSuccess) { prof_release(ctx); return SPIN_ERR_HIP; }
  return SPIN_OK;
}

extern "C" int spin_profile_read(spin_ctx *ctx, int32_t which, int32_t *count, float *mean_us, float *min_us) {
  if (!ctx || which < 0 || which >= SPIN_KERNEL_IDS || !count || !mean_us || !min_us) return SPIN_ERR_INVALID;
  *count = 0; *mean_us = 0.f; *min_us = 0.f;
  if (ctx->prof_cap == 0) return SPIN_OK;
  const int n = ctx->prof_n[which];
  double sum = 0.0; float mn = 3.4e38f;
  for (int i = 0; i < n; ++i) {
    float ms = 0.f;
    SPIN_HIP_CHECK(hipEventSynchronize(ctx->prof_ev[which][2 * i + 1]));
    SPIN_HIP_CHECK(hipEventElapsedTime(&ms, ctx->prof_ev[which][2 * i], ctx->prof_ev[which][2 * i + 1]));
    sum += ms; if (ms < mn) mn = ms;
  }
  ctx->prof_n[which] = 0;
  *count = n;
  if (n > 0) { *mean_us = (float)(sum / n * 1e3); *min_us = mn * 1e3f; }
  return SPIN_OK;
}

extern "C" const char *spin_status_string(int s) {
  switch (s) {
    case SPIN_OK: return "ok";
    case SPIN_ERR_INVALID: return "invalid argument";
    case SPIN_ERR_UNSUPPORTED: return "unsupported shape or mode";
    case SPIN_ERR_WORKSPACE: return "workspace missing";
    case SPIN_ERR_HIP: return "HIP runtime error";
    case SPIN_ERR_BUDGET: return "slot budget smaller than the step's selection";
    case SPIN_ERR_NOT_RESIDENT: return "selected page not resident";
    case SPIN_ERR_SLOT_RANGE: return "slot id outside the pool";
    case SPIN_ERR_LEAF_POOL: return "leaf segment pool exhausted";
    case SPIN_ERR_STATIC_LIMIT: return "shape needs more scratch than the library's static device array holds";
    default: return "unknown status";
  }
}

extern "C" int spin_set_partition_tables(spin_ctx *ctx, const int32_t *part_offsets, const int32_t *part_count,
                                         const int32_t *part_first_page, const int32_t *part_tokens) {
  if (!ctx) return SPIN_ERR_INVALID;
  if (!part_count && !part_first_page && !part_tokens) {   // back to uniform partitions
    ctx->var = spin_var{nullptr, nullptr, nullptr, nullptr};
    return SPIN_OK;
  }
  if (!part_offsets || !part_count || !part_first_page || !part_tokens) return SPIN_ERR_INVALID;
  const spin_config &c = ctx->cfg;
  // strides and the stage-2 path are sized for uniform partitions unless the context was created for tables
  if (!c.variable_partitions) return SPIN_ERR_UNSUPPORTED;
  // summaries that exist for partitions of any length: min / max keys, or one mean key (centroid)
  const bool kind_ok = c.score_kind == SPIN_SCORE_MINMAX ||
                       (c.score_kind == SPIN_SCORE_REPMAX && c.reps_per_partition == 1);
  if (c.partition_tokens < 16 || !kind_ok) return SPIN_ERR_UNSUPPORTED;
  ctx->var = spin_var{part_offsets, part_count, part_first_page, part_tokens};
  return SPIN_OK;
}

extern "C" size_t spin_workspace_bytes(const spin_ctx *c) { return c ? c->ws_bytes : 0; }
extern "C" int32_t spin_sel_stride(const spin_ctx *c) { return c ? c->sel_stride : 0; }
extern "C" int32_t spin_page_stride(const spin_ctx *c) { return c ? c->page_stride : 0; }
extern "C" int32_t spin_dir_stride(const spin_ctx *c) { return c ? c->dir_stride : 0; }
extern "C" int32_t spin_decode_splits(const spin_ctx *c) { return c ? c->splits : 0; }

extern "C" size_t spin_summary_bytes(const spin_ctx *c, int64_t padded_partitions) {
  if (!c || padded_partitions < 0) return 0;
  // one summary row = kd bf16; rows are padded per KV head to whole 16-row tiles
  return (size_t)padded_partitions * c->cfg.num_kv_heads * c->rows_per_part * c->kd * 2;
}

__global__ void spin_fill_i32_kernel(int32_t *p, int32_t v, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// Plain streaming read used as the bandwidth yardstick of a box: every lane
// fetches 16-byte units with a grid stride and folds them into one word.
__global__ __launch_bounds__(256) void spin_stream_read_kernel(const uint4 *__restrict__ p, size_t n_u4,
                                                               uint32_t *__restrict__ sink) {
  size_t i = (size_t)blockIdx.x * 256 * 8 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256 * 8;
  uint32_t acc = 0;
  for (; i < n_u4; i += stride) {
    uint4 v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = (i + 256 * k < n_u4) ? spin_nt_load(p + i + 256 * k) : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int k = 0; k < 8; ++k) acc ^= v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
  }
  if (acc == 0x9e3779b9u) *sink = acc;   // keeps the loads alive; practically never taken
}

extern "C" int spin_probe_stream_read(spin_ctx *ctx, const void *buf, size_t bytes, void *workspace, void *stream) {
  if (!ctx || !buf || bytes < 16) return SPIN_ERR_INVALID;
  if (!workspace) return SPIN_ERR_WORKSPACE;
  spin_launch(ctx, SPIN_K_PROBE, spin_stream_read_kernel, dim3(2048), dim3(256), 0, (hipStream_t)stream,
              (const uint4 *)buf, bytes / 16, (uint32_t *)workspace + 8);
  return spin_launch_status();
}

extern "C" int spin_workspace_init(spin_ctx *ctx, void *workspace, void *stream) {
  if (!ctx) return SPIN_ERR_INVALID;
  if (!workspace) return SPIN_ERR_WORKSPACE;
  const int n = (int)(ctx->ws_zero_bytes / 4);
  hipLaunchKernelGGL(spin_fill_i32_kernel, dim3((n + 255) / 256), dim3(256), 0, (hipStream_t)stream,
                     (int32_t *)workspace, 0, n);
  return spin_launch_status();
}

// step counter of a workspace (word 1 of its header), for launches recorded once and replayed
__global__ void spin_step_kernel(int32_t *ws, int32_t set_to) {
  if (threadIdx.x == 0 && blockIdx.x == 0) ws[1] = set_to >= 0 ? set_to : ws[1] + 1;
}

extern "C" int spin_set_step(spin_ctx *ctx, void *workspace, int32_t step, void *stream) {
  if (!ctx || step < 0) return SPIN_ERR_INVALID;
  if (!workspace) return SPIN_ERR_WORKSPACE;
  hipLaunchKernelGGL(spin_step_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, (int32_t *)workspace, step);
  return spin_launch_status();
}

extern "C" int spin_advance_step(spin_ctx *ctx, void *workspace, void *stream) {
  if (!ctx) return SPIN_ERR_INVALID;
  if (!workspace) return SPIN_ERR_WORKSPACE;
  hipLaunchKernelGGL(spin_step_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, (int32_t *)workspace, -1);
  return spin_launch_status();
}

extern "C" int spin_poll_status(spin_ctx *ctx, const void *workspace, void *stream) {
  if (!ctx) return SPIN_ERR_INVALID;
  if (!workspace) return SPIN_ERR_WORKSPACE;
  int32_t st = 0;
  SPIN_HIP_CHECK(hipMemcpyAsync(&st, workspace, sizeof(st), hipMemcpyDeviceToHost, (hipStream_t)stream));
  SPIN_HIP_CHECK(hipStreamSynchronize((hipStream_t)stream));
  return st;
}
