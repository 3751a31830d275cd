// Stages 2 and 3 in one launch (all-resident mode; rows of more than 16384
// partitions take the long-row kernels of stage 2, whose finishing launch resolves).  Both stages work on one row per workgroup, so the workgroup
// that selected a row resolves it straight away: the same device functions run
// as in the two stage calls, the results are the same bits, and one launch with
// its start-up latency chain is saved.
#include "spin_decode_dev.h"
#include "spin_resolve_dev.h"
#include "spin_select_dev.h"

template <int BLOCK, int KPT>
__global__ __launch_bounds__(BLOCK) void spin_select_resolve_kernel(
    const float *__restrict__ scores, const int32_t *__restrict__ part_offsets,
    const int32_t *__restrict__ seq_lens, int Hkv, int tp, int topk, int includes_forced, int sink_pages,
    int recent_pages, int sel_stride, int32_t *sel, int32_t *nsel, const int32_t *dir,
    const int32_t *__restrict__ leaf_pool, int64_t leaf_chunks, int page_stride, int dir_stride, int leaf_entries,
    int32_t *__restrict__ slots, int32_t *__restrict__ page_ids, uint16_t *__restrict__ valid_mask,
    int32_t *__restrict__ npages, int32_t *status, spin_var var) {
  const int row = blockIdx.x;
  const int take = select_reg_row<BLOCK, KPT>(scores, part_offsets, seq_lens, Hkv, tp, topk, includes_forced,
                                                     sink_pages, recent_pages, sel_stride, sel, nsel, row, var);
  __syncthreads();   // the selection was written by this workgroup: visible to all its threads from here
  resolve_row<BLOCK>(row, take, sel, seq_lens, dir, leaf_pool, leaf_chunks, Hkv, tp, sink_pages, recent_pages,
                     sel_stride, page_stride, dir_stride, leaf_entries, slots, page_ids, valid_mask, npages, status, var);
}

// ---------------------------------------------------------------------------
// The always-attended pages of a row (its first sink_pages and last recent_pages pages) do not
// depend on the selection, so they can be attended while stages 2+3 run: those are latency-bound
// on one workgroup per row and leave the rest of the chip and the memory system idle.  A second
// set of workgroups in the same launch (about one per 16 such pages of a row, at most one per
// split of stage 4) looks these pages up in the two-level table itself, attends them with stage
// 4's tile code and stores one partial (m, l, O) per query head behind the row's split partials;
// the first of them also records how many leading and trailing entries of the row's page list
// these pages are (stage 3 lists pages in ascending order and lists every such page, so the sink
// pages open the list and the recent pages close it, whatever the partition size).  Stage 4 then
// skips those entries, and the first wavefront of split j starts from the j-th partial instead of
// from the empty state.

// The always-attended pages of a row as one list: j < nlo is sink page j, the others are the recent
// pages from recent_begin on.  Looks entry j up for the calling lane (all lanes of the wavefront call;
// `active` says whether the lane has an entry): slot and token mask, or an empty mask when the page is
// not resident (stage 3 reports that).
__device__ inline void forced_lookup(bool active, int j, int nlo, int recent_begin, int N, int32_t mydir,
                                     bool dir_in_lanes, const int32_t *__restrict__ dir,
                                     const int32_t *__restrict__ leaf_pool, int64_t leaf_chunks, int row,
                                     int dir_stride, int leaf_entries, int64_t pool_slots, int &myslot,
                                     unsigned &mymask) {
  const int page = j < nlo ? j : recent_begin + (j - nlo);
  int32_t s = -1;
  if (dir_in_lanes) {
    const int ci = active ? page / leaf_entries : 0;
    const int32_t chunk = __shfl(mydir, ci < dir_stride ? ci : 0);   // every lane takes part in the exchange
    if (active && ci < dir_stride && chunk >= 0 && (int64_t)chunk < leaf_chunks)
      s = leaf_pool[(size_t)chunk * leaf_entries + (page - ci * leaf_entries)];
  } else if (active) {
    s = spin_walk(dir, leaf_pool, leaf_chunks, row, dir_stride, leaf_entries, page);
  }
  myslot = 0;
  mymask = 0;
  if (s >= 0 && (int64_t)s < pool_slots) {
    myslot = s;
    mymask = page_mask(page, N);
  }
}

struct forced_span {
  int nlo, nhi, recent_begin;
};
// the same rule as stages 2 and 3: a context no longer than the two windows is attended whole
__device__ inline forced_span forced_pages_of(int N, int sink_pages, int recent_pages) {
  const int pages = (N + 15) >> 4;
  int sink_end = min(sink_pages, pages);
  int recent_begin = max(pages - recent_pages, 0);
  if (sink_end >= recent_begin) { sink_end = pages; recent_begin = pages; }
  return forced_span{sink_end, pages - recent_begin, recent_begin};
}

template <int WAVES>
__device__ inline void attend_forced_row(
    int row, int side, int nside, const uint16_t *__restrict__ q, const uint4 *__restrict__ pool, int64_t pool_slots,
    const int32_t *__restrict__ seq_lens, const int32_t *__restrict__ dir, const int32_t *__restrict__ leaf_pool,
    int64_t leaf_chunks, int Hkv, int G, int Hq, int sink_pages, int recent_pages, int dir_stride, int leaf_entries,
    int nsplit, int pstride, float scale_log2e, float *part_ml, float *part_acc, int32_t *skip) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = lane & 15, c = lane >> 4;
  const int b = row / Hkv, h = row - b * Hkv;

  spin_bf16x8 qf[4];
  load_queries(qf, q, b, h, G, Hq, n, c);
  // the row's directory entries, one per lane, requested together with the context length, so that the leaf
  // entries are the only dependent table access (directories of more than 64 entries are walked page by page)
  const bool dir_in_lanes = dir_stride <= 64;
  int32_t mydir = -1;
  if (dir_in_lanes && lane < dir_stride) mydir = dir[(size_t)row * dir_stride + lane];
  const int N = seq_lens[b];
  const forced_span fs = forced_pages_of(N, sink_pages, recent_pages);
  const int nlo = fs.nlo, nhi = fs.nhi, recent_begin = fs.recent_begin;
  const int nf = nlo + nhi;
  if (threadIdx.x == 0 && side == 0) {
    skip[2 * row] = nlo;
    skip[2 * row + 1] = nhi;
  }
  // The list above is dealt round-robin to the row's `nside` workgroups and, inside one, to its wavefronts;
  // lane i looks up the i-th page of this wavefront (batches of 64).
  const int first = side + nside * wave, stride = nside * WAVES;
  const int cnt_all = nf > first ? (nf - first + stride - 1) / stride : 0;
  softmax_state st;
  softmax_reset(st);
  for (int base = 0; base < cnt_all; base += 64) {
    const int cnt = min(cnt_all - base, 64);
    int myslot = 0;
    unsigned mymask = 0;
    forced_lookup(lane < cnt, first + stride * (base + lane), nlo, recent_begin, N, mydir, dir_in_lanes, dir, leaf_pool,
                  leaf_chunks, row, dir_stride, leaf_entries, pool_slots, myslot, mymask);
    attend_lane_pages<2>(st, pool, myslot, mymask, cnt, lane, c, qf, scale_log2e);
  }
  decode_finish<WAVES, true>(st, row, side, b, h, lane, wave, n, c, G, Hq, nsplit, pstride, part_ml,
                       part_acc, nullptr, nullptr, nullptr);
}

struct spin_forced_args {
  const uint16_t *q;
  const uint4 *pool;
  int64_t pool_slots;
  int G, Hq, nsplit, pstride, nside;
  float scale_log2e;
  float *part_ml, *part_acc;
  int32_t *skip;
};

// workgroups [0, rows): stages 2+3 of a row, exactly as spin_select_resolve_kernel;
// workgroups [rows, rows + rows * nside): attention over the always-attended pages, nside workgroups per row
template <int KPT>
__global__ __launch_bounds__(512) void spin_select_resolve_forced_kernel(
    int rows, const float *__restrict__ scores, const int32_t *__restrict__ part_offsets,
    const int32_t *__restrict__ seq_lens, int Hkv, int tp, int topk, int includes_forced, int sink_pages,
    int recent_pages, int sel_stride, int32_t *sel, int32_t *nsel, const int32_t *dir,
    const int32_t *__restrict__ leaf_pool, int64_t leaf_chunks, int page_stride, int dir_stride, int leaf_entries,
    int32_t *__restrict__ slots, int32_t *__restrict__ page_ids, uint16_t *__restrict__ valid_mask,
    int32_t *__restrict__ npages, int32_t *status, spin_forced_args fa) {
  if ((int)blockIdx.x >= rows) {
    const int idx = (int)blockIdx.x - rows, srow = idx / fa.nside;
    attend_forced_row<8>(srow, idx - srow * fa.nside, fa.nside, fa.q, fa.pool, fa.pool_slots, seq_lens, dir, leaf_pool, leaf_chunks, Hkv,
                         fa.G, fa.Hq, sink_pages, recent_pages, dir_stride, leaf_entries, fa.nsplit, fa.pstride,
                         fa.scale_log2e, fa.part_ml, fa.part_acc, fa.skip);
    return;
  }
  const int row = blockIdx.x;
  const int take = select_reg_row<512, KPT>(scores, part_offsets, seq_lens, Hkv, tp, topk, includes_forced,
                                            sink_pages, recent_pages, sel_stride, sel, nsel, row, spin_var{});
  __syncthreads();   // the selection was written by this workgroup: visible to all its threads from here
  resolve_row<512>(row, take, sel, seq_lens, dir, leaf_pool, leaf_chunks, Hkv, tp, sink_pages, recent_pages,
                   sel_stride, page_stride, dir_stride, leaf_entries, slots, page_ids, valid_mask, npages, status,
                   spin_var{});
}

extern "C" int spin_select_resolve_forced(spin_ctx *ctx, int32_t batch, const float *scores,
                                          const int32_t *part_offsets, const int32_t *seq_lens, int32_t *sel,
                                          int32_t *nsel, const int32_t *dir, const int32_t *leaf_pool,
                                          int64_t leaf_chunks, int32_t *slots, int32_t *page_ids,
                                          uint16_t *valid_mask, int32_t *npages, const void *q, const void *kv_pool,
                                          int64_t pool_slots, void *workspace, void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch || leaf_chunks <= 0 || pool_slots <= 0) return SPIN_ERR_INVALID;
  if (!spin_forced_split_supported(ctx) || ctx->var.count) return SPIN_ERR_UNSUPPORTED;
  if (batch == 0) return SPIN_OK;
  if (!scores || !part_offsets || !seq_lens || !sel || !nsel || !dir || !leaf_pool || !slots || !page_ids ||
      !valid_mask || !npages || !q || !kv_pool)
    return SPIN_ERR_INVALID;
  if (!workspace) return SPIN_ERR_WORKSPACE;
  const spin_config &c = ctx->cfg;
  const int rows = batch * c.num_kv_heads;
  char *ws = (char *)workspace;
  const spin_forced_args fa = {(const uint16_t *)q, (const uint4 *)kv_pool, pool_slots, ctx->group, c.num_q_heads,
                               ctx->splits, ctx->pstride, ctx->side_wgs, ctx->scale * 1.4426950408889634f,
                               (float *)(ws + ctx->ws_ml_off), (float *)(ws + ctx->ws_acc_off),
                               (int32_t *)(ws + ctx->ws_skip_off)};
  // dynamic LDS: the merge buffers of the attention workgroups (8 wavefronts)
  const size_t lds = (size_t)8 * ctx->group * (SPIN_HEAD_DIM + 2) * sizeof(float);
#define SPIN_SRF_ARGS                                                                                         \
  dim3((unsigned)(rows * (1 + ctx->side_wgs))), dim3(512), lds, (hipStream_t)stream, rows, scores, part_offsets, seq_lens,      \
      c.num_kv_heads, c.partition_tokens, c.topk, c.topk_includes_forced, c.sink_pages, c.recent_pages,       \
      ctx->sel_stride, sel, nsel, dir, leaf_pool, leaf_chunks, ctx->page_stride, ctx->dir_stride,             \
      c.leaf_entries, slots, page_ids, valid_mask, npages, (int32_t *)workspace, fa
  if (ctx->max_parts <= 2048)
    spin_launch(ctx, SPIN_K_SELECT, spin_select_resolve_forced_kernel<4>, SPIN_SRF_ARGS);
  else
    spin_launch(ctx, SPIN_K_SELECT, spin_select_resolve_forced_kernel<8>, SPIN_SRF_ARGS);
#undef SPIN_SRF_ARGS
  return spin_launch_status();
}

// hist_ready: stage 1 of this step has filled the long-row histograms already
static int select_resolve_impl(spin_ctx *ctx, int32_t batch, const float *scores, const int32_t *part_offsets,
                               const int32_t *seq_lens, int32_t *sel, int32_t *nsel, const int32_t *dir,
                               const int32_t *leaf_pool, int64_t leaf_chunks, int32_t *slots, int32_t *page_ids,
                               uint16_t *valid_mask, int32_t *npages, void *workspace, void *stream,
                               bool hist_ready) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch || leaf_chunks <= 0) return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!scores || !part_offsets || !seq_lens || !sel || !nsel || !dir || !leaf_pool || !slots || !page_ids ||
      !valid_mask || !npages)
    return SPIN_ERR_INVALID;
  if (!workspace) return SPIN_ERR_WORKSPACE;
  const spin_config &c = ctx->cfg;
  if (c.lru_timestamps > 0) return SPIN_ERR_UNSUPPORTED;
  const int rows = batch * c.num_kv_heads;
  if (ctx->max_parts > 16384) {
    // long rows: the launch that finishes stage 2 resolves its row (refused where that path does not apply)
    const spin_resolve_args res{dir, leaf_pool, leaf_chunks, slots, page_ids, valid_mask, npages};
    return spin_select_impl(ctx, batch, scores, part_offsets, seq_lens, sel, nsel, workspace, stream, hist_ready, &res);
  }
#define SPIN_SR_ARGS                                                                                          \
  0, (hipStream_t)stream, scores, part_offsets, seq_lens, c.num_kv_heads, c.partition_tokens, c.topk,         \
      c.topk_includes_forced, c.sink_pages, c.recent_pages, ctx->sel_stride, sel, nsel, dir, leaf_pool,       \
      leaf_chunks, ctx->page_stride, ctx->dir_stride, c.leaf_entries, slots, page_ids, valid_mask, npages,    \
      (int32_t *)workspace, ctx->var
  if (ctx->max_parts <= 2048)
    spin_launch(ctx, SPIN_K_SELECT, spin_select_resolve_kernel<512, 4>, dim3((unsigned)rows), dim3(512), SPIN_SR_ARGS);
  else if (ctx->max_parts <= 4096)
    spin_launch(ctx, SPIN_K_SELECT, spin_select_resolve_kernel<512, 8>, dim3((unsigned)rows), dim3(512), SPIN_SR_ARGS);
  else
    spin_launch(ctx, SPIN_K_SELECT, spin_select_resolve_kernel<1024, 16>, dim3((unsigned)rows), dim3(1024),
                SPIN_SR_ARGS);
#undef SPIN_SR_ARGS
  return spin_launch_status();
}

extern "C" int spin_select_resolve(spin_ctx *ctx, int32_t batch, const float *scores, const int32_t *part_offsets,
                                   const int32_t *seq_lens, int32_t *sel, int32_t *nsel, const int32_t *dir,
                                   const int32_t *leaf_pool, int64_t leaf_chunks, int32_t *slots,
                                   int32_t *page_ids, uint16_t *valid_mask, int32_t *npages, void *workspace,
                                   void *stream) {
  return select_resolve_impl(ctx, batch, scores, part_offsets, seq_lens, sel, nsel, dir, leaf_pool, leaf_chunks, slots,
                             page_ids, valid_mask, npages, workspace, stream, false);
}

// Stages 1, 2 and 3 in two launches: spin_score_partitions (which, for rows of more than 16384 partitions, counts
// stage 2's first histogram as it goes) followed by spin_select_resolve.  Same results as the three stage calls.
extern "C" int spin_score_select_resolve(spin_ctx *ctx, int32_t batch, const void *q, const void *summaries,
                                         const int32_t *chan_idx, const int32_t *part_offsets,
                                         const int32_t *seq_lens, float *scores, int32_t *sel, int32_t *nsel,
                                         const int32_t *dir, const int32_t *leaf_pool, int64_t leaf_chunks,
                                         int32_t *slots, int32_t *page_ids, uint16_t *valid_mask, int32_t *npages,
                                         void *workspace, void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch || leaf_chunks <= 0) return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!sel || !nsel || !dir || !leaf_pool || !slots || !page_ids || !valid_mask || !npages) return SPIN_ERR_INVALID;
  if (!workspace) return SPIN_ERR_WORKSPACE;
  const spin_config &c = ctx->cfg;
  const int rows = batch * c.num_kv_heads;
  const bool long_rows = ctx->max_parts > 16384;
  // refuse before stage 1 is issued what the second launch would refuse
  if (c.lru_timestamps > 0 || (long_rows && !(ctx->ws_hist_off && rows <= 65535))) return SPIN_ERR_UNSUPPORTED;
  const bool fuse = long_rows;   // stage 1 of every score kind counts stage 2's first histogram for long rows
  int32_t *hist = fuse ? (int32_t *)((char *)workspace + ctx->ws_hist_off) : nullptr;
  const int st = spin_score_impl(ctx, batch, q, summaries, chan_idx, part_offsets, seq_lens, scores, workspace, stream,
                                 hist);
  if (st != SPIN_OK) return st;
  return select_resolve_impl(ctx, batch, scores, part_offsets, seq_lens, sel, nsel, dir, leaf_pool, leaf_chunks, slots,
                             page_ids, valid_mask, npages, workspace, stream, fuse);
}
