// Stage 1: score every partition of every row against the current query
// (Section 4.1, Select; Table 1, score(q, k_sums)).
//
// Each score kind is a contraction of a summary row with a query-derived
// vector, so a tile of 16 summary rows is one matrix-core tile
// S[head][row] = sum_k Q[head][k] * A[row][k]:
//   MINMAX  sum_d max(q*min, q*max) = sum_d ( max(q,0)*max_d + min(q,0)*min_d ),
//           i.e. the row [max | min] (256 elements) against [q+ | q-]; one of the
//           two products per channel is exactly zero, so nothing is added that
//           the definition does not add.  8 x (16x16x32) instructions.
//   REPMAX  representative . q over 128 channels, 4 x (16x16x32); then a
//           maximum over the partition's 4 rows.
//   SKETCH  16 sketched channels, 1 x (16x16x16).
// bf16 x bf16 products are exact in fp32; accumulation is fp32 inside the
// matrix core.  The queries are the first operand, so a lane holds one summary
// row's values for four heads and the maximum over the group's heads needs no
// exchange for groups of up to four heads (two otherwise).  Summary tiles are
// stored chunk-major so each load is a contiguous wavefront transaction.
#include "spin_score_dev.h"
#include "spin_select_dev.h"   // key order and forced-partition plan of stage 2, for the fused histogram

#define SCORE_WAVES 4

template <int NJ, bool MINMAX, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void spin_score_k32_kernel(
    const uint16_t *__restrict__ q, const uint4 *__restrict__ summ, const int32_t *__restrict__ part_offsets,
    int Hq, int Hkv, int G, int rows_per_part, int tiles_per_wg, int wgs_per_row, float *__restrict__ scores) {
  const int row = blockIdx.x / wgs_per_row, chunk = blockIdx.x - row * wgs_per_row;
  score_row_tiles<NJ, MINMAX, WAVES>(q, summ, part_offsets, Hq, Hkv, G, rows_per_part, tiles_per_wg, row, chunk,
                                            scores);
}

template <int NJ, bool MINMAX, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void spin_score_k32_single_kernel(
    const uint16_t *__restrict__ q, const uint4 *__restrict__ summ, const int32_t *__restrict__ part_offsets,
    int Hq, int Hkv, int G, int rows_per_part, int tiles_per_wg, int wgs_per_row, float *__restrict__ scores) {
  (void)tiles_per_wg;   // == WAVES
  const int row = blockIdx.x / wgs_per_row, chunk = blockIdx.x - row * wgs_per_row;
  score_row_single_tile<NJ, MINMAX, WAVES>(q, summ, part_offsets, Hq, Hkv, G, rows_per_part, row, chunk, scores);
}

// what stage 2 needs to know to tell candidates from forced partitions
struct score_hist_args {
  const int32_t *seq_lens;
  int32_t *hist;            // [rows][BIG_BINS]
  int tp, topk, includes_forced, sink_pages, recent_pages, sel_stride;
};

// MINMAX / REPMAX rows of more than 16384 partitions scored by stretches of `tiles_per_wg` tiles per workgroup,
// which also counts the leading 12 key bits of its candidates' scores: LDS bins, then one global add per bin the
// stretch touched.  That is the first launch of stage 2 for long rows; the score bits are those of the kernels above.
template <int NJ, bool MINMAX, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void spin_score_k32_hist_kernel(
    const uint16_t *__restrict__ q, const uint4 *__restrict__ summ, const int32_t *__restrict__ part_offsets,
    int Hq, int Hkv, int G, int rows_per_part, int tiles_per_wg, int wgs_per_row, float *__restrict__ scores,
    score_hist_args ha) {
  __shared__ int s_h[BIG_BINS];
  const int row = blockIdx.x / wgs_per_row, chunk = blockIdx.x - row * wgs_per_row;
  const int b = row / Hkv;
  const int PP = part_offsets[b + 1] - part_offsets[b];
  if (chunk * tiles_per_wg >= PP * rows_per_part / 16) return;   // the whole workgroup: nothing to score or count
  score_bins hb = {s_h, 0, 0};
  const sel_plan pl = select_plan(ha.seq_lens[b], PP, ha.tp, ha.topk, ha.includes_forced, ha.sink_pages,
                                  ha.recent_pages, ha.sel_stride);
  if (pl.kprime > 0) { hb.cand_lo = pl.nf_lo; hb.cand_hi = pl.first_hi; }
  for (int i = threadIdx.x; i < BIG_BINS; i += WAVES * 64) s_h[i] = 0;
  __syncthreads();
  score_row_tiles<NJ, MINMAX, WAVES, true>(q, summ, part_offsets, Hq, Hkv, G, rows_per_part, tiles_per_wg, row, chunk,
                                           scores, hb);
  __syncthreads();
  for (int i = threadIdx.x; i < BIG_BINS; i += WAVES * 64) {
    const int cnt = s_h[i];
    if (cnt) atomicAdd(&ha.hist[(size_t)row * BIG_BINS + i], cnt);
  }
}

// SKETCH: one 16x16x16 instruction per tile of 16 tokens (512 bytes).
// HIST: the workgroup also counts the leading 12 key bits of its candidates' scores (LDS, then one
// global add per bin it touched), which is the first launch of stage 2 for long rows.
template <bool HIST>
__global__ __launch_bounds__(SCORE_WAVES * 64) void spin_score_sketch_kernel(
    const uint16_t *__restrict__ q, const uint2 *__restrict__ summ, const int32_t *__restrict__ chan,
    const int32_t *__restrict__ part_offsets, int Hq, int Hkv, int G, int tiles_per_wg, int wgs_per_row,
    float *__restrict__ scores, score_hist_args ha) {
  __shared__ int s_h[HIST ? BIG_BINS : 1];
  const int row = blockIdx.x / wgs_per_row, chunk = blockIdx.x - row * wgs_per_row;
  const int b = row / Hkv, h = row - b * Hkv;
  const int PP = part_offsets[b + 1] - part_offsets[b];
  const int ntiles = PP / 16;
  const int t_begin = chunk * tiles_per_wg;
  if (t_begin >= ntiles) return;
  const int t_end = min(t_begin + tiles_per_wg, ntiles);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 15, c = lane >> 4;
  const size_t base = (size_t)Hkv * part_offsets[b] + (size_t)h * PP;

  const uint2 *tiles = summ + base * 4;   // 16 elements = 4 units of 8 bytes per row
  constexpr int U = 8;
  // the first batch of tiles is requested before the query gather below (two dependent loads)
  // has to be waited for
  int t0 = t_begin + wave * U;
  uint2 a[U];
#pragma unroll
  for (int u = 0; u < U; ++u) a[u] = (t0 + u < t_end) ? spin_nt_load2(tiles + (size_t)(t0 + u) * 64 + lane) : make_uint2(0, 0);

  int cand_lo = 0, cand_hi = 0;           // candidates of stage 2: partitions [cand_lo, cand_hi)
  if (HIST) {
    const sel_plan pl = select_plan(ha.seq_lens[b], PP, ha.tp, ha.topk, ha.includes_forced, ha.sink_pages,
                                    ha.recent_pages, ha.sel_stride);
    if (pl.kprime > 0) { cand_lo = pl.nf_lo; cand_hi = pl.first_hi; }
    for (int i = threadIdx.x; i < BIG_BINS; i += SCORE_WAVES * 64) s_h[i] = 0;
    __syncthreads();
  }
  // A operand: row n = head, k = sketched channels 4c..4c+3
  spin_s16x4 qf;
  {
    const uint16_t *qrow = q + ((size_t)(b * Hq + h * G + (n < G ? n : 0))) * SPIN_HEAD_DIM;
    uint16_t e[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) e[i] = n < G ? qrow[chan[h * 16 + 4 * c + i]] : (uint16_t)0;
    uint2 pk = make_uint2(e[0] | ((uint32_t)e[1] << 16), e[2] | ((uint32_t)e[3] << 16));
    qf = __builtin_bit_cast(spin_s16x4, pk);
  }
  for (; t0 < t_end; t0 += SCORE_WAVES * U) {
    // the next batch is in flight while this one is consumed
    uint2 nx[U];
    const int t1 = t0 + SCORE_WAVES * U;
#pragma unroll
    for (int u = 0; u < U; ++u) nx[u] = (t1 + u < t_end) ? spin_nt_load2(tiles + (size_t)(t1 + u) * 64 + lane) : make_uint2(0, 0);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (t0 + u >= t_end) break;
      spin_f32x4 s = {0.f, 0.f, 0.f, 0.f};
      s = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(qf, __builtin_bit_cast(spin_s16x4, a[u]), s, 0, 0, 0);
      const float m = spin_head_max(s, c, G);   // lane (n, c): heads 4c+i of token n
      if (c == 0) {
        const int p = (t0 + u) * 16 + n;
        scores[base + p] = m;
        if (HIST && p >= cand_lo && p < cand_hi) atomicAdd(&s_h[score_key(m) >> 20], 1);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) a[u] = nx[u];
  }
  if (HIST) {
    __syncthreads();
    for (int i = threadIdx.x; i < BIG_BINS; i += SCORE_WAVES * 64) {
      const int cnt = s_h[i];
      if (cnt) atomicAdd(&ha.hist[(size_t)row * BIG_BINS + i], cnt);
    }
  }
}

// SKETCH for groups of at most four query heads: four tiles of 16 tokens per pair of 16x16x32
// instructions.  The first operand's row 4j+g is head g against tile j: its 64 contraction
// elements are the head's 16 sketched query values in the 16 positions of tile j and zeros in the
// other three tiles' positions (exact zero products), the second operand stacks the four tiles'
// channels.  Lane (n, c) then holds the scores of token n of tile c for the four heads: the maximum
// stays in the lane, all 64 lanes store (one contiguous 256 bytes) and count, and the per-tile
// work of the one-tile kernel above is done once per four tiles.
template <bool HIST>
__global__ __launch_bounds__(SCORE_WAVES * 64) void spin_score_sketch4_kernel(
    const uint16_t *__restrict__ q, const uint2 *__restrict__ summ, const int32_t *__restrict__ chan,
    const int32_t *__restrict__ part_offsets, int Hq, int Hkv, int G, int tiles_per_wg, int wgs_per_row,
    float *__restrict__ scores, score_hist_args ha) {
  __shared__ int s_h[HIST ? BIG_BINS : 1];
  const int row = blockIdx.x / wgs_per_row, chunk = blockIdx.x - row * wgs_per_row;
  const int b = row / Hkv, h = row - b * Hkv;
  const int PP = part_offsets[b + 1] - part_offsets[b];
  const int ntiles = PP / 16;
  const int t_begin = chunk * tiles_per_wg;       // tiles_per_wg is a multiple of 4
  if (t_begin >= ntiles) return;
  const int t_end = min(t_begin + tiles_per_wg, ntiles);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 15, c = lane >> 4;
  const size_t base = (size_t)Hkv * part_offsets[b] + (size_t)h * PP;
  const uint2 *tiles = summ + base * 4;           // a tile: 64 units of 8 bytes, unit (channel quad cq, token) at cq*16 + token
  constexpr int U = 4;                            // groups of four tiles per wavefront and batch
  // lane (n, c) feeds instruction m with channels 8(c%2) .. +7 of token n of tile 2m + c/2:
  // the units (2(c%2), n) and (2(c%2) + 1, n) of that tile; tiles past the end are clamped
  const int unit = (2 * (c & 1)) * 16 + n;
  struct group4 { uint2 lo[2], hi[2]; };
  auto load_group = [&](group4 &g4, int t) {
#pragma unroll
    for (int m = 0; m < 2; ++m) {
      const int tile = min(t + 2 * m + (c >> 1), t_end - 1);
      const uint2 *src = tiles + (size_t)tile * 64 + unit;
      g4.lo[m] = spin_nt_load2(src);
      g4.hi[m] = spin_nt_load2(src + 16);
    }
  };
  int t0 = t_begin + wave * 4 * U;
  group4 cur[U];
#pragma unroll
  for (int u = 0; u < U; ++u)
    if (t0 + 4 * u < t_end) load_group(cur[u], t0 + 4 * u);

  int cand_lo = 0, cand_hi = 0;                   // candidates of stage 2: partitions [cand_lo, cand_hi)
  if (HIST) {
    const sel_plan pl = select_plan(ha.seq_lens[b], PP, ha.tp, ha.topk, ha.includes_forced, ha.sink_pages,
                                    ha.recent_pages, ha.sel_stride);
    if (pl.kprime > 0) { cand_lo = pl.nf_lo; cand_hi = pl.first_hi; }
    for (int i = threadIdx.x; i < BIG_BINS; i += SCORE_WAVES * 64) s_h[i] = 0;
    __syncthreads();
  }
  // first operand of instruction m: lane (r, c) supplies row r = 4j + g, contraction elements
  // 8c .. 8c+7 of the instruction's 32 = positions 8(c%2) .. +7 of tile 2m + c/2
  spin_bf16x8 qa[2];
  {
    const int j = n >> 2, g = n & 3;
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    if (g < G) {
      const uint16_t *qrow = q + ((size_t)(b * Hq + h * G + g)) * SPIN_HEAD_DIM;
#pragma unroll
      for (int e = 0; e < 8; e += 2)
        w[e >> 1] = (uint32_t)qrow[chan[h * 16 + 8 * (c & 1) + e]] | ((uint32_t)qrow[chan[h * 16 + 8 * (c & 1) + e + 1]] << 16);
    }
#pragma unroll
    for (int m = 0; m < 2; ++m) {
      const bool mine = j == 2 * m + (c >> 1);
      qa[m] = __builtin_bit_cast(spin_bf16x8, mine ? make_uint4(w[0], w[1], w[2], w[3]) : make_uint4(0u, 0u, 0u, 0u));
    }
  }
  for (; t0 < t_end; t0 += SCORE_WAVES * 4 * U) {
    // the next batch is in flight while this one is consumed
    group4 nxt[U];
    const int t1 = t0 + SCORE_WAVES * 4 * U;
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (t1 + 4 * u < t_end) load_group(nxt[u], t1 + 4 * u);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int t = t0 + 4 * u;
      if (t >= t_end) break;
      spin_f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int m = 0; m < 2; ++m) {
        const uint4 bm = make_uint4(cur[u].lo[m].x, cur[u].lo[m].y, cur[u].hi[m].x, cur[u].hi[m].y);
        s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa[m], __builtin_bit_cast(spin_bf16x8, bm), s, 0, 0, 0);
      }
      const float mx = spin_head_max(s, 0, G);    // lane (n, c): heads 0..3 of token n of tile t + c
      if (t + c < t_end) {
        const int p = (t + c) * 16 + n;           // = t*16 + lane: the wavefront stores 64 consecutive scores
        scores[base + p] = mx;
        if (HIST && p >= cand_lo && p < cand_hi) atomicAdd(&s_h[score_key(mx) >> 20], 1);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) cur[u] = nxt[u];
  }
  if (HIST) {
    __syncthreads();
    for (int i = threadIdx.x; i < BIG_BINS; i += SCORE_WAVES * 64) {
      const int cnt = s_h[i];
      if (cnt) atomicAdd(&ha.hist[(size_t)row * BIG_BINS + i], cnt);
    }
  }
}

int spin_score_impl(spin_ctx *ctx, int32_t batch, const void *q, const void *summaries, const int32_t *chan_idx,
                    const int32_t *part_offsets, const int32_t *seq_lens, float *scores, void *workspace,
                    void *stream, int32_t *hist) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch) return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!q || !summaries || !part_offsets || !seq_lens || !scores) return SPIN_ERR_INVALID;
  (void)workspace;
  const spin_config &c = ctx->cfg;
  const int rows = batch * c.num_kv_heads;
  const int max_pp = ((ctx->max_parts + 15) / 16) * 16;
  hipStream_t st = (hipStream_t)stream;
  const int W = c.score_waves ? c.score_waves : 4;
  const score_hist_args ha = {seq_lens, hist, c.partition_tokens, c.topk, c.topk_includes_forced, c.sink_pages,
                              c.recent_pages, ctx->sel_stride};
  if (hist && c.score_kind != SPIN_SCORE_SKETCH) {
    // long rows whose stage 2 starts from a histogram: stretches of 64 tiles, so that clearing and adding up the
    // 4096 LDS bins is small beside the 256 KiB or more of summaries a workgroup reads
    const bool mm = c.score_kind == SPIN_SCORE_MINMAX;
    const int R = mm ? 1 : c.reps_per_partition;
    const int tiles_per_wg = 64, max_tiles = max_pp * R / 16;
    const int wgs = (max_tiles + tiles_per_wg - 1) / tiles_per_wg;
    if (mm)
      spin_launch(ctx, SPIN_K_SCORE, spin_score_k32_hist_kernel<8, true, 4>, dim3((unsigned)rows * wgs), dim3(256), 0, st,
                  (const uint16_t *)q, (const uint4 *)summaries, part_offsets, c.num_q_heads, c.num_kv_heads, ctx->group,
                  R, tiles_per_wg, wgs, scores, ha);
    else
      spin_launch(ctx, SPIN_K_SCORE, spin_score_k32_hist_kernel<4, false, 4>, dim3((unsigned)rows * wgs), dim3(256), 0, st,
                  (const uint16_t *)q, (const uint4 *)summaries, part_offsets, c.num_q_heads, c.num_kv_heads, ctx->group,
                  R, tiles_per_wg, wgs, scores, ha);
    return spin_launch_status();
  }
  if (c.score_kind == SPIN_SCORE_MINMAX) {
    // one tile per wavefront measured best: the dispatcher streams the workgroups
    const int tiles_per_wg = c.score_tiles_per_wg ? c.score_tiles_per_wg : W, max_tiles = max_pp / 16;
    const int wgs = (max_tiles + tiles_per_wg - 1) / tiles_per_wg;
#define SPIN_SCORE_ARGS(RPP)                                                                                  \
  0, st, (const uint16_t *)q, (const uint4 *)summaries, part_offsets, c.num_q_heads, c.num_kv_heads, ctx->group, \
      RPP, tiles_per_wg, wgs, scores
    if (W == 2 && tiles_per_wg == 2)
      spin_launch(ctx, SPIN_K_SCORE, spin_score_k32_single_kernel<8, true, 2>, dim3((unsigned)rows * wgs), dim3(128),
                  SPIN_SCORE_ARGS(1));
    else if (W == 1 && tiles_per_wg == 1)
      spin_launch(ctx, SPIN_K_SCORE, spin_score_k32_single_kernel<8, true, 1>, dim3((unsigned)rows * wgs), dim3(64),
                  SPIN_SCORE_ARGS(1));
    else if (W == 8 && tiles_per_wg == 8)
      spin_launch(ctx, SPIN_K_SCORE, spin_score_k32_single_kernel<8, true, 8>, dim3((unsigned)rows * wgs), dim3(512),
                  SPIN_SCORE_ARGS(1));
    else if (W == 8)
      spin_launch(ctx, SPIN_K_SCORE, spin_score_k32_kernel<8, true, 8>, dim3((unsigned)rows * wgs), dim3(512),
                  SPIN_SCORE_ARGS(1));
    else if (tiles_per_wg == 4)
      spin_launch(ctx, SPIN_K_SCORE, spin_score_k32_single_kernel<8, true, 4>, dim3((unsigned)rows * wgs), dim3(256),
                  SPIN_SCORE_ARGS(1));
    else
      spin_launch(ctx, SPIN_K_SCORE, spin_score_k32_kernel<8, true, 4>, dim3((unsigned)rows * wgs), dim3(256),
                  SPIN_SCORE_ARGS(1));
  } else if (c.score_kind == SPIN_SCORE_REPMAX) {
    const int R = c.reps_per_partition;
    const int tiles_per_wg = c.score_tiles_per_wg ? c.score_tiles_per_wg : 2 * W, max_tiles = max_pp * R / 16;
    const int wgs = (max_tiles + tiles_per_wg - 1) / tiles_per_wg;
    if (W == 8)
      spin_launch(ctx, SPIN_K_SCORE, spin_score_k32_kernel<4, false, 8>, dim3((unsigned)rows * wgs), dim3(512),
                  SPIN_SCORE_ARGS(R));
    else
      spin_launch(ctx, SPIN_K_SCORE, spin_score_k32_kernel<4, false, 4>, dim3((unsigned)rows * wgs), dim3(256),
                  SPIN_SCORE_ARGS(R));
#undef SPIN_SCORE_ARGS
  } else {
    if (!chan_idx) return SPIN_ERR_INVALID;
    // groups of up to four heads: the four-tile kernel, 256 tiles per workgroup measured best (64 / 128 /
    // 256 / 512 / 1024: 34.0 / 30.6 / 28.4 / 29.8 / 35.3 us on 8 x 64K tokens with the histogram)
    const bool four = ctx->group <= 4 && (c.score_tiles_per_wg % 4) == 0;
    const int tiles_per_wg = c.score_tiles_per_wg ? c.score_tiles_per_wg : (four ? 256 : 128), max_tiles = max_pp / 16;
    const int wgs = (max_tiles + tiles_per_wg - 1) / tiles_per_wg;
#define SPIN_SKETCH_ARGS                                                                                         \
  dim3((unsigned)rows * wgs), dim3(SCORE_WAVES * 64), 0, st, (const uint16_t *)q, (const uint2 *)summaries, chan_idx, \
      part_offsets, c.num_q_heads, c.num_kv_heads, ctx->group, tiles_per_wg, wgs, scores, ha
    if (four) {
      if (hist) spin_launch(ctx, SPIN_K_SCORE, spin_score_sketch4_kernel<true>, SPIN_SKETCH_ARGS);
      else spin_launch(ctx, SPIN_K_SCORE, spin_score_sketch4_kernel<false>, SPIN_SKETCH_ARGS);
    } else if (hist) spin_launch(ctx, SPIN_K_SCORE, spin_score_sketch_kernel<true>, SPIN_SKETCH_ARGS);
    else spin_launch(ctx, SPIN_K_SCORE, spin_score_sketch_kernel<false>, SPIN_SKETCH_ARGS);
#undef SPIN_SKETCH_ARGS
  }
  return spin_launch_status();
}

extern "C" int spin_score_partitions(spin_ctx *ctx, int32_t batch, const void *q, const void *summaries,
                                     const int32_t *chan_idx, const int32_t *part_offsets,
                                     const int32_t *seq_lens, float *scores, void *workspace, void *stream) {
  return spin_score_impl(ctx, batch, q, summaries, chan_idx, part_offsets, seq_lens, scores, workspace, stream, nullptr);
}
