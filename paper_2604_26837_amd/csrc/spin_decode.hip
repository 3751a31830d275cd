// Stage 4: paged GQA decode attention over the resolved pages of each row
// (Section 4.1, Attention: standard attention restricted to the selected KV).
//
// One workgroup = one (row, split) pair; its wavefronts are dealt the split's
// pages round-robin.  Per page a wavefront issues eight contiguous 1 KiB loads
// (K tile then V tile of the slot), forms the 16 x 16 logit tile
// S[token][head] = K Q^T with four 16x16x32 bf16 matrix instructions (the
// group's G <= 16 query heads padded to 16 columns), runs the online softmax
// on its four logits per lane, and accumulates O[head][dim] += P V with eight
// 16x16x16 instructions; the logit tile's register layout is exactly the
// operand layout of P, so nothing moves between lanes except two max
// exchanges.  The loads of the next page are issued before the current page is
// consumed (two register buffers), and a wavefront fetches the slot ids and
// masks of all its pages with one load up front, so the only dependent memory
// round trips per wavefront are that one and the first page.
//
// Wavefront partials (m, l, O) are merged through LDS in wave order.  With
// more than one split the workgroup partials go to the workspace and the
// last workgroup of the row to arrive (a ticket counter in the workspace
// header) merges them in split order, so results are reproducible.
#include <mutex>

#include "spin_decode_dev.h"

#define SPIN_DECODE_FROM_PARTIAL 1   // the row's first wavefront starts from the partial at index nsplit
#define SPIN_DECODE_TO_PARTIAL 2     // the row's merged result goes there instead of to `out`

template <int WAVES, int DEPTH>
__global__ __launch_bounds__(WAVES * 64) void spin_decode_kernel(
    const uint16_t *__restrict__ q, const uint4 *__restrict__ pool, int64_t pool_slots,
    const int32_t *__restrict__ slots, const uint16_t *__restrict__ masks,
    const int32_t *__restrict__ npages, int page_stride, int G, int Hq, int Hkv, int nsplit, int pstride,
    const int32_t *__restrict__ skip, int mode, int nside, float scale_log2e, float *part_ml, float *part_acc, int32_t *tickets,
    uint16_t *__restrict__ out, float *__restrict__ lse, int32_t *status) {
  const int row = blockIdx.x / nsplit;
  const int split = blockIdx.x - row * nsplit;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int n = lane & 15;   // column: query head of the group (logits), channel-in-block (output)
  const int c = lane >> 4;   // token quad (logits) / head quad (output)
  const int b = row / Hkv;
  const int h = row - b * Hkv;

  // Pages are dealt round-robin: page p belongs to split p % nsplit and, inside
  // it, to wavefront (p / nsplit) % WAVES.  The addresses of this wavefront's
  // slot entries therefore do not depend on the row's page count, and their
  // load is issued together with it.
  const int32_t *rslots = slots + (size_t)row * page_stride;
  const uint16_t *rmask = masks + (size_t)row * page_stride;
  const int first = wave * nsplit + split, stride = WAVES * nsplit;
  int np = npages[row];
  np = np < 0 ? 0 : (np > page_stride ? page_stride : np);
  // list positions [0, skip_lo) and [np - skip_hi, np) were attended by an earlier launch (the row's
  // always-attended pages): they keep their place in the dealing but are not fetched or attended here
  int skip_lo = 0, skip_hi = 0;
  if (skip) {
    skip_lo = skip[2 * row];
    skip_hi = skip[2 * row + 1];
  }
  const int keep_end = np - (skip_hi > 0 ? skip_hi : 0);

  spin_bf16x8 qf[4];
  load_queries(qf, q, b, h, G, Hq, n, c);
  softmax_state st;
  softmax_reset(st);

  // The first wavefront of split s < nside starts from the s-th partial (m, l, O) an earlier launch left for
  // the row (its always-attended pages, or the first of two passes over the page list) instead of from the
  // empty state: that partial then is part of the ordinary merge.
  if ((mode & SPIN_DECODE_FROM_PARTIAL) && split < nside && wave == 0) {
    const size_t pf = ((size_t)row * pstride + nsplit + split) * G;
    if (n < G) {
      st.m = part_ml[(pf + n) * 2];
      if (c == 0) st.l = part_ml[(pf + n) * 2 + 1];   // the lanes' denominators are summed over c at the end
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (4 * c + i < G) {
#pragma unroll
        for (int jn = 0; jn < 8; ++jn) st.acc[jn][i] = part_acc[(pf + 4 * c + i) * SPIN_HEAD_DIM + 16 * jn + n];
      }
  }

  // this wavefront's pages: first + i * stride, i < nw
  const int nw_max = (page_stride - first + stride - 1) / stride;   // entries that exist in the buffer
  for (int base = 0; base < nw_max; base += 64) {
    int myslot = 0;
    unsigned mymask = 0;
    const int p = first + (base + lane) * stride;
    if (p < page_stride) {
      myslot = rslots[p];
      mymask = rmask[p];
    }
    const int nw = np > first ? (np - first + stride - 1) / stride : 0;
    if (base >= nw) break;
    const int cnt = (nw - base) < 64 ? (nw - base) : 64;
    if (lane < cnt) {
      if (p < skip_lo || p >= keep_end) {
        myslot = 0;   // attended elsewhere: nothing is fetched for an empty mask
        mymask = 0;
      } else if (myslot < 0 || (int64_t)myslot >= pool_slots) {
        spin_raise(status, SPIN_ERR_SLOT_RANGE);
        myslot = 0;   // read a valid slot, attend to none of it
        mymask = 0;
      }
    }
    attend_lane_pages<DEPTH>(st, pool, myslot, mymask, cnt, lane, c, qf, scale_log2e);
  }

  decode_finish<WAVES>(st, row, split, b, h, lane, wave, n, c, G, Hq, nsplit, pstride, part_ml, part_acc, tickets, out,
                       lse, (mode & SPIN_DECODE_TO_PARTIAL) != 0);
}

// ---------------------------------------------------------------------------
// Partitions smaller than a page (token-major slots): most attended pages hold one or two
// attended tokens, so a tile is not a physical page but 16 ATTENDED tokens gathered from
// wherever they live.  A wavefront expands the masks of its pages (dealt round-robin exactly as
// above) into a token list in LDS -- page order, then token order, so the accumulation order is
// fixed -- and then treats every 16 list entries as one tile: lane (n, c) fetches 64 contiguous
// bytes of the key of tile row n per load, and the values of tile rows 4c .. 4c+3 for its 8
// output channels with 2-byte loads that land in the operand layout of P V directly.  Per
// attended token that is the algorithmic 512 bytes (two cache lines of K, two of V) instead of
// the page's 8 KiB, and sixteen times fewer matrix tiles.  Logits, softmax and merge are the
// code of the page kernel.
#define TOK_LIST 1024   // list entries per wavefront and batch of 64 pages

struct tile_src {
  const uint4 *k;           // key row of tile row n (lane % 16), chunk c (lane / 16): + 4 j
  const uint16_t *v[4];     // value rows of tile rows 4c .. 4c+3 at channel n: + 16 jn
};

// Rows past the end of the list repeat its last entry: their loads stay inside attended data, their
// logits are masked and their probabilities are exactly zero.
__device__ inline tile_src tile_source(const uint4 *__restrict__ pool, const uint32_t *tok, int first, int count, int lane) {
  tile_src s;
  const int n = lane & 15, c = lane >> 4;
  const int last = count - 1 - first;                    // >= 0: the tile exists
  const uint32_t e = tok[first + min(n, last)];          // slot * 16 + token
  s.k = pool + (size_t)(e >> 4) * SPIN_SLOT_U4 + (e & 15u) * 16 + c;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t ev = tok[first + min(4 * c + i, last)];
    s.v[i] = (const uint16_t *)(pool + (size_t)(ev >> 4) * SPIN_SLOT_U4 + SPIN_KTILE_U4) + (ev & 15u) * SPIN_HEAD_DIM + n;
  }
  return s;
}

__device__ inline void load_tile(page_regs &r, const tile_src &s) {
#pragma unroll
  for (int j = 0; j < 4; ++j) r.k[j] = spin_nt_load(s.k + 4 * j);
  // operand layout of P V: r.v[jv] = {rows 4c,4c+1 | rows 4c+2,4c+3} for channel block 2jv, then 2jv+1.
  // Each 16-bit load lands in its half of an operand register, so nothing waits for the data
  // before the tile is consumed.
  typedef unsigned short us8 __attribute__((ext_vector_type(8)));
#pragma unroll
  for (int jv = 0; jv < 4; ++jv) {
    us8 w;
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
      for (int i = 0; i < 4; ++i) w[4 * blk + i] = s.v[i][16 * (2 * jv + blk)];
    r.v[jv] = __builtin_bit_cast(uint4, w);
  }
}

template <int WAVES>
__global__ __launch_bounds__(WAVES * 64) void spin_decode_tokens_kernel(
    const uint16_t *__restrict__ q, const uint4 *__restrict__ pool, int64_t pool_slots,
    const int32_t *__restrict__ slots, const uint16_t *__restrict__ masks,
    const int32_t *__restrict__ npages, int page_stride, int G, int Hq, int Hkv, int nsplit, int pstride,
    const int32_t *__restrict__ skip, float scale_log2e, float *part_ml, float *part_acc, int32_t *tickets,
    uint16_t *__restrict__ out, float *__restrict__ lse, int32_t *status) {
  extern __shared__ float smem[];
  // the token lists live behind the merge buffers of decode_finish
  uint32_t *tok = (uint32_t *)(smem + WAVES * G * (SPIN_HEAD_DIM + 2)) + (threadIdx.x >> 6) * TOK_LIST;

  const int row = blockIdx.x / nsplit;
  const int split = blockIdx.x - row * nsplit;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int n = lane & 15, c = lane >> 4;
  const int b = row / Hkv;
  const int h = row - b * Hkv;
  const int32_t *rslots = slots + (size_t)row * page_stride;
  const uint16_t *rmask = masks + (size_t)row * page_stride;
  const int first = wave * nsplit + split, stride = WAVES * nsplit;
  int np = npages[row];
  np = np < 0 ? 0 : (np > page_stride ? page_stride : np);

  spin_bf16x8 qf[4];
  {
    const uint4 *qrow = (const uint4 *)(q + ((size_t)(b * Hq + h * G + (n < G ? n : 0))) * SPIN_HEAD_DIM);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      uint4 v = qrow[j * 4 + c];
      if (n >= G) v = make_uint4(0, 0, 0, 0);
      qf[j] = __builtin_bit_cast(spin_bf16x8, v);
    }
  }
  softmax_state st;
  st.m = NEG_INF;
  st.l = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) st.acc[i] = (spin_f32x4){0.f, 0.f, 0.f, 0.f};

  const int nw_max = (page_stride - first + stride - 1) / stride;
  for (int base = 0; base < nw_max; base += 64) {
    int myslot = 0;
    unsigned mymask = 0;
    const int p = first + (base + lane) * stride;
    if (p < page_stride) {
      myslot = rslots[p];
      mymask = rmask[p];
    }
    const int nw = np > first ? (np - first + stride - 1) / stride : 0;
    if (base >= nw) break;
    const int cnt = (nw - base) < 64 ? (nw - base) : 64;
    if (lane >= cnt) mymask = 0;
    else if (myslot < 0 || (int64_t)myslot >= pool_slots) {
      spin_raise(status, SPIN_ERR_SLOT_RANGE);
      myslot = 0;
      mymask = 0;
    }
    // token list of this batch of pages: page order, then token order
    const int mine = __popc(mymask);
    const int incl = spin_wave_inclusive_scan(mine);
    const int total = __builtin_amdgcn_readlane(incl, 63);
    {
      int pos = incl - mine;
      unsigned m = mymask;
      while (m) {
        const int t = __ffs(m) - 1;
        m &= m - 1;
        tok[pos++] = ((uint32_t)myslot << 4) | (uint32_t)t;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the wavefront reads its own list: program order
    // two register buffers: the next tile's loads are issued before the current one is consumed
    page_regs r[2];
    const int ntiles = (total + 15) >> 4;
    if (ntiles > 0) load_tile(r[0], tile_source(pool, tok, 0, total, lane));
    for (int k = 0; k < ntiles; k += 2) {
      if (k + 1 < ntiles) load_tile(r[1], tile_source(pool, tok, 16 * (k + 1), total, lane));
      const int left0 = total - 16 * k;
      consume_page(st, r[0], qf, left0 >= 16 ? 0xffffu : ((1u << left0) - 1u), c, scale_log2e);
      if (k + 2 < ntiles) load_tile(r[0], tile_source(pool, tok, 16 * (k + 2), total, lane));
      if (k + 1 < ntiles) {
        const int left1 = total - 16 * (k + 1);
        consume_page(st, r[1], qf, left1 >= 16 ? 0xffffu : ((1u << left1) - 1u), c, scale_log2e);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // before the next batch overwrites the list
  }
  __syncthreads();   // the merge buffers are separate from the lists, but keep the phases apart
  decode_finish<WAVES>(st, row, split, b, h, lane, wave, n, c, G, Hq, nsplit, pstride, part_ml, part_acc, tickets, out,
                       lse);
}

// Host side of stage 4: checks, then the launch; the split-K scratch (row tickets, (m, l) pairs and
// accumulators of the workgroup partials) and the status word are handed in by the two entry points.
// skip != NULL: the row's always-attended pages were attended by the launch of stages 2+3, whose partial sits
// behind the splits' partials and whose list positions are named in skip[row][2].
static int decode_launch(spin_ctx *ctx, int32_t batch, const void *q, const void *kv_pool, int64_t pool_slots,
                         const int32_t *slots, const uint16_t *valid_mask, const int32_t *npages, void *out,
                         float *lse, float *part_ml, float *part_acc, int32_t *tickets, int32_t *status,
                         const int32_t *skip, int mode, int nside, void *stream) {
  const int rows = batch * ctx->cfg.num_kv_heads;
  const int G = ctx->group, nsplit = ctx->splits;
  const int pstride = ctx->pstride;
  const float scale_log2e = ctx->scale * 1.4426950408889634f;
  const int W = ctx->waves;
  const size_t lds = (size_t)W * G * (SPIN_HEAD_DIM + 2) * sizeof(float);
  if (ctx->k_token_major) {
    if (mode) return SPIN_ERR_UNSUPPORTED;   // the gathered-token kernel runs whole rows only
    // token-major slots: tiles of gathered tokens (always 8 wavefronts: the waves and depth knobs do not
    // apply, and the merge buffers are sized for 8 whatever the waves knob says)
    const size_t lds_tok = (size_t)8 * G * (SPIN_HEAD_DIM + 2) * sizeof(float) + (size_t)8 * TOK_LIST * sizeof(uint32_t);
    spin_launch(ctx, SPIN_K_DECODE, spin_decode_tokens_kernel<8>, dim3((unsigned)(rows * nsplit)), dim3(512), lds_tok,
                (hipStream_t)stream, (const uint16_t *)q, (const uint4 *)kv_pool, pool_slots, slots, valid_mask, npages,
                ctx->page_stride, G, ctx->cfg.num_q_heads, ctx->cfg.num_kv_heads, nsplit, pstride, skip, scale_log2e,
                part_ml, part_acc, tickets, (uint16_t *)out, lse, status);
    return spin_launch_status();
  }
#define SPIN_DECODE_LAUNCH2(WV, DP)                                                                              \
  spin_launch(ctx, SPIN_K_DECODE, spin_decode_kernel<WV, DP>, dim3((unsigned)(rows * nsplit)), dim3(WV * 64), lds, \
              (hipStream_t)stream, (const uint16_t *)q, (const uint4 *)kv_pool, pool_slots, slots, valid_mask,   \
              npages, ctx->page_stride, G, ctx->cfg.num_q_heads, ctx->cfg.num_kv_heads, nsplit, pstride, skip,   \
              mode, nside, scale_log2e, part_ml, part_acc, tickets, (uint16_t *)out, lse, status)
#define SPIN_DECODE_LAUNCH(WV)                          \
  do {                                                  \
    if (ctx->depth == 2) SPIN_DECODE_LAUNCH2(WV, 2);    \
    else if (ctx->depth == 4) SPIN_DECODE_LAUNCH2(WV, 4); \
    else SPIN_DECODE_LAUNCH2(WV, 3);                    \
  } while (0)
  if (W == 2) SPIN_DECODE_LAUNCH(2);
  else if (W == 8) SPIN_DECODE_LAUNCH(8);
  else SPIN_DECODE_LAUNCH(4);
#undef SPIN_DECODE_LAUNCH
#undef SPIN_DECODE_LAUNCH2
  return spin_launch_status();
}

extern "C" int spin_sparse_decode(spin_ctx *ctx, int32_t batch, const void *q, const void *kv_pool,
                                  int64_t pool_slots, const int32_t *slots, const uint16_t *valid_mask,
                                  const int32_t *npages, void *out, float *lse, void *workspace,
                                  void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch || pool_slots <= 0) return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!q || !kv_pool || !slots || !valid_mask || !npages || !out) return SPIN_ERR_INVALID;
  if (!workspace) return SPIN_ERR_WORKSPACE;
  char *ws = (char *)workspace;
  return decode_launch(ctx, batch, q, kv_pool, pool_slots, slots, valid_mask, npages, out, lse,
                       (float *)(ws + ctx->ws_ml_off), (float *)(ws + ctx->ws_acc_off),
                       (int32_t *)(ws + ctx->ws_ticket_off), (int32_t *)workspace, nullptr, 0, 0, stream);
}

// Attention in two passes over one page list: the first attends the tokens its masks name and leaves
// the row's merged partial (m, l, O) in the workspace, the second starts from it.
static int decode_two_pass(spin_ctx *ctx, int32_t batch, const void *q, const void *kv_pool, int64_t pool_slots,
                           const int32_t *slots, const uint16_t *valid_mask, const int32_t *npages, void *out,
                           float *lse, void *workspace, int mode, void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch || pool_slots <= 0) return SPIN_ERR_INVALID;
  if (ctx->k_token_major) return SPIN_ERR_UNSUPPORTED;
  if (batch == 0) return SPIN_OK;
  if (!q || !kv_pool || !slots || !valid_mask || !npages || (!out && !(mode & SPIN_DECODE_TO_PARTIAL)))
    return SPIN_ERR_INVALID;
  if (!workspace) return SPIN_ERR_WORKSPACE;
  char *ws = (char *)workspace;
  return decode_launch(ctx, batch, q, kv_pool, pool_slots, slots, valid_mask, npages, out, lse,
                       (float *)(ws + ctx->ws_ml_off), (float *)(ws + ctx->ws_acc_off),
                       (int32_t *)(ws + ctx->ws_ticket_off), (int32_t *)workspace, nullptr, mode, 1, stream);
}

extern "C" int spin_sparse_decode_begin(spin_ctx *ctx, int32_t batch, const void *q, const void *kv_pool,
                                        int64_t pool_slots, const int32_t *slots, const uint16_t *valid_mask,
                                        const int32_t *npages, void *workspace, void *stream) {
  return decode_two_pass(ctx, batch, q, kv_pool, pool_slots, slots, valid_mask, npages, nullptr, nullptr, workspace,
                         SPIN_DECODE_TO_PARTIAL, stream);
}

extern "C" int spin_sparse_decode_finish(spin_ctx *ctx, int32_t batch, const void *q, const void *kv_pool,
                                         int64_t pool_slots, const int32_t *slots, const uint16_t *valid_mask,
                                         const int32_t *npages, void *out, float *lse, void *workspace,
                                         void *stream) {
  return decode_two_pass(ctx, batch, q, kv_pool, pool_slots, slots, valid_mask, npages, out, lse, workspace,
                         SPIN_DECODE_FROM_PARTIAL, stream);
}

// Stage 4 over what spin_select_resolve_forced left: the pages other than the always-attended ones, merged
// with the partial that launch stored for them.
extern "C" int spin_sparse_decode_rest(spin_ctx *ctx, int32_t batch, const void *q, const void *kv_pool,
                                       int64_t pool_slots, const int32_t *slots, const uint16_t *valid_mask,
                                       const int32_t *npages, void *out, float *lse, void *workspace,
                                       void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch || pool_slots <= 0) return SPIN_ERR_INVALID;
  if (!spin_forced_split_supported(ctx)) return SPIN_ERR_UNSUPPORTED;
  if (batch == 0) return SPIN_OK;
  if (!q || !kv_pool || !slots || !valid_mask || !npages || !out) return SPIN_ERR_INVALID;
  if (!workspace) return SPIN_ERR_WORKSPACE;
  char *ws = (char *)workspace;
  return decode_launch(ctx, batch, q, kv_pool, pool_slots, slots, valid_mask, npages, out, lse,
                       (float *)(ws + ctx->ws_ml_off), (float *)(ws + ctx->ws_acc_off),
                       (int32_t *)(ws + ctx->ws_ticket_off), (int32_t *)workspace,
                       (const int32_t *)(ws + ctx->ws_skip_off), SPIN_DECODE_FROM_PARTIAL, ctx->side_wgs, stream);
}

// ---------------------------------------------------------------------------
// Stage 4 for callers that cannot hand over (or allocate) a workspace: the split-K scratch lives in
// a device array of the library itself.  Every GPU the library runs on holds its own copy of the
// array, at its own address, until the process ends.
#define SPIN_STATIC_SCRATCH_DEVICES 64
static __device__ __align__(256) unsigned char scratch[SPIN_STATIC_SCRATCH_BYTES];

// `scratch` above is only a host-side handle in host code: the device address is asked for once per
// device (with that device current) and kept; host code uses that address and never the symbol's name.
static void *g_scratch_ptr[SPIN_STATIC_SCRATCH_DEVICES];
static std::mutex g_scratch_mutex;

static int static_scratch(void **ptr) {
  int dev = -1;
  SPIN_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= SPIN_STATIC_SCRATCH_DEVICES) return SPIN_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    SPIN_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return SPIN_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return SPIN_OK;
}

int spin_static_scratch_prepare(void) {
  void *p = nullptr;
  return static_scratch(&p);
}

// clears the words that must be zero when the attention kernel starts (a kernel, not a memset, so
// that a caller may record the call into a HIP graph)
__global__ void spin_static_clear_kernel(int32_t *p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

extern "C" int spin_sparse_decode_static(spin_ctx *ctx, int32_t batch, const void *q, const void *kv_pool,
                                         int64_t pool_slots, const int32_t *slots, const uint16_t *valid_mask,
                                         const int32_t *npages, void *out, float *lse, int32_t *status,
                                         void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch || pool_slots <= 0) return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!q || !kv_pool || !slots || !valid_mask || !npages || !out) return SPIN_ERR_INVALID;
  // layout inside the array, sized for this call's rows: [status word, 256 B][tickets][(m, l)][accumulators]
  const size_t rows = (size_t)batch * ctx->cfg.num_kv_heads;
  const size_t partials = rows * ctx->pstride * ctx->group;   // the layout of the workspace (spare partials are not used here)
  const size_t ticket_off = SPIN_WS_HEADER;
  const size_t ml_off = (ticket_off + rows * sizeof(int32_t) + 255) & ~(size_t)255;
  const size_t acc_off = (ml_off + partials * 2 * sizeof(float) + 255) & ~(size_t)255;
  const size_t need = acc_off + partials * SPIN_HEAD_DIM * sizeof(float);
  if (need > SPIN_STATIC_SCRATCH_BYTES) return SPIN_ERR_STATIC_LIMIT;
  void *base = nullptr;
  const int rc = static_scratch(&base);
  if (rc != SPIN_OK) return rc;
  char *sc = (char *)base;
  // the array keeps the last call's contents: the status word and the row tickets start at zero
  const int nclear = (int)(ml_off / sizeof(int32_t));
  hipLaunchKernelGGL(spin_static_clear_kernel, dim3((nclear + 255) / 256), dim3(256), 0, (hipStream_t)stream,
                     (int32_t *)sc, nclear);
  if (hipGetLastError() != hipSuccess) return SPIN_ERR_HIP;
  return decode_launch(ctx, batch, q, kv_pool, pool_slots, slots, valid_mask, npages, out, lse,
                       (float *)(sc + ml_off), (float *)(sc + acc_off), (int32_t *)(sc + ticket_off),
                       status ? status : (int32_t *)sc, nullptr, 0, 0, stream);
}
