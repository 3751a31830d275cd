// Stage 1: score every partition of every row against the current query
// (Section 4.1, Select; Table 1, score(q, k_sums)).
//
// Each score kind is a contraction of a summary row with a query-derived
// vector, so a tile of 16 summary rows is one matrix-core tile
// S[row][head] = sum_k A[row][k] * B[k][head]:
//   MINMAX  sum_d max(q*min, q*max) = sum_d ( max(q,0)*max_d + min(q,0)*min_d ),
//           i.e. the row [max | min] (256 elements) against [q+ | q-]; one of the
//           two products per channel is exactly zero, so nothing is added that
//           the definition does not add.  8 x (16x16x32) instructions.
//   REPMAX  representative . q over 128 channels, 4 x (16x16x32); then a
//           maximum over the partition's 4 rows.
//   SKETCH  16 sketched channels, 1 x (16x16x16).
// bf16 x bf16 products are exact in fp32; accumulation is fp32 inside the
// matrix core.  The group's heads (columns) are reduced by a maximum with two
// to four DPP exchanges.  Summary tiles are stored chunk-major so each load is
// a contiguous wavefront transaction.
#include "spin_common.h"

#define SCORE_WAVES 4

__device__ inline uint32_t relu_pack(uint32_t w, bool pos) {
  // keep the halves whose sign matches: positive part (pos) or negative part
  const uint32_t lo = w & 0xffffu, hi = w >> 16;
  const bool lo_neg = lo & 0x8000u, hi_neg = hi & 0x8000u;
  const uint32_t l = (lo_neg != pos) ? lo : 0u, h = (hi_neg != pos) ? hi : 0u;
  return l | (h << 16);
}

// MINMAX and REPMAX: NJ instructions of 16x16x32 per tile (NJ = KD/32).  The
// workgroup's tiles are dealt round-robin to its wavefronts; the next tile's
// loads are issued before the current tile is consumed.
template <int NJ>
struct score_tile {
  uint4 a[NJ];
};

template <int NJ>
__device__ inline void load_tile(score_tile<NJ> &r, const uint4 *__restrict__ tp, int lane) {
#pragma unroll
  for (int j = 0; j < NJ; ++j) r.a[j] = spin_nt_load(tp + j * 64 + lane);
}

template <int NJ, bool MINMAX>
__device__ inline void consume_tile(const score_tile<NJ> &r, const spin_bf16x8 (&qf)[NJ], int n, int c, int G,
                                    float *__restrict__ scores, size_t base, int t) {
  spin_f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int j = 0; j < NJ; ++j)
    s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(spin_bf16x8, r.a[j]), qf[j], s, 0, 0, 0);
  // s[i] = value of summary row 4c+i for head n
  float v[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) v[i] = spin_row16_max(n < G ? s[i] : -__builtin_inff());
  if (MINMAX) {
    if (n == 0) *(float4 *)(scores + base + (size_t)t * 16 + 4 * c) = make_float4(v[0], v[1], v[2], v[3]);
  } else {
    // rows 4c..4c+3 are the four representatives of partition 4t + c
    const float m = fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3]));
    if (n == 0) scores[base + (size_t)t * 4 + c] = m;
  }
}

template <int NJ, bool MINMAX, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void spin_score_k32_kernel(
    const uint16_t *__restrict__ q, const uint4 *__restrict__ summ, const int32_t *__restrict__ part_offsets,
    int Hq, int Hkv, int G, int rows_per_part, int tiles_per_wg, int wgs_per_row, float *__restrict__ scores) {
  const int row = blockIdx.x / wgs_per_row, chunk = blockIdx.x - row * wgs_per_row;
  const int b = row / Hkv, h = row - b * Hkv;
  const int off_b = part_offsets[b];
  const int PP = part_offsets[b + 1] - off_b;
  const int ntiles = PP * rows_per_part / 16;
  const int t_begin = chunk * tiles_per_wg;
  if (t_begin >= ntiles) return;
  const int t_end = min(t_begin + tiles_per_wg, ntiles);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 15, c = lane >> 4;
  const size_t base = (size_t)Hkv * off_b + (size_t)h * PP;   // in partitions

  // B operand: column n = query head, k = elements 32j + 8c .. +8 of the query-side vector
  spin_bf16x8 qf[NJ];
  {
    const uint4 *qrow = (const uint4 *)(q + ((size_t)(b * Hq + h * G + (n < G ? n : 0))) * SPIN_HEAD_DIM);
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      uint4 v = qrow[(j & 3) * 4 + c];
      if (MINMAX) {
        const bool pos = j < 4;   // first 128 elements pair with max, the rest with min
        v = make_uint4(relu_pack(v.x, pos), relu_pack(v.y, pos), relu_pack(v.z, pos), relu_pack(v.w, pos));
      }
      if (n >= G) v = make_uint4(0, 0, 0, 0);
      qf[j] = __builtin_bit_cast(spin_bf16x8, v);
    }
  }

  const uint4 *tiles = summ + base * rows_per_part * (NJ * 4);   // NJ*32 elements = NJ*4 units per row
  int t = t_begin + wave;
  if (t >= t_end) return;
  score_tile<NJ> ra, rb;
  load_tile<NJ>(ra, tiles + (size_t)t * (NJ * 64), lane);
  for (; t < t_end; t += 2 * WAVES) {
    const int t1 = t + WAVES, t2 = t + 2 * WAVES;
    if (t1 < t_end) load_tile<NJ>(rb, tiles + (size_t)t1 * (NJ * 64), lane);
    consume_tile<NJ, MINMAX>(ra, qf, n, c, G, scores, base, t);
    if (t2 < t_end) load_tile<NJ>(ra, tiles + (size_t)t2 * (NJ * 64), lane);
    if (t1 < t_end) consume_tile<NJ, MINMAX>(rb, qf, n, c, G, scores, base, t1);
  }
}

// SKETCH: one 16x16x16 instruction per tile of 16 tokens (512 bytes).
__global__ __launch_bounds__(SCORE_WAVES * 64) void spin_score_sketch_kernel(
    const uint16_t *__restrict__ q, const uint2 *__restrict__ summ, const int32_t *__restrict__ chan,
    const int32_t *__restrict__ part_offsets, int Hq, int Hkv, int G, int tiles_per_wg, int wgs_per_row,
    float *__restrict__ scores) {
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

  // B operand: column n = head, k = sketched channels 4c..4c+3
  spin_s16x4 qf;
  {
    const uint16_t *qrow = q + ((size_t)(b * Hq + h * G + (n < G ? n : 0))) * SPIN_HEAD_DIM;
    uint16_t e[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) e[i] = n < G ? qrow[chan[h * 16 + 4 * c + i]] : (uint16_t)0;
    uint2 pk = make_uint2(e[0] | ((uint32_t)e[1] << 16), e[2] | ((uint32_t)e[3] << 16));
    qf = __builtin_bit_cast(spin_s16x4, pk);
  }
  const uint2 *tiles = summ + base * 4;   // 16 elements = 4 units of 8 bytes per row
  constexpr int U = 8;
  for (int t0 = t_begin + wave * U; t0 < t_end; t0 += SCORE_WAVES * U) {
    uint2 a[U];
#pragma unroll
    for (int u = 0; u < U; ++u) a[u] = (t0 + u < t_end) ? tiles[(size_t)(t0 + u) * 64 + lane] : make_uint2(0, 0);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (t0 + u >= t_end) break;
      spin_f32x4 s = {0.f, 0.f, 0.f, 0.f};
      s = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(spin_s16x4, a[u]), qf, s, 0, 0, 0);
      float v[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] = spin_row16_max(n < G ? s[i] : -__builtin_inff());
      if (n == 0)
        *(float4 *)(scores + base + (size_t)(t0 + u) * 16 + 4 * c) = make_float4(v[0], v[1], v[2], v[3]);
    }
  }
}

extern "C" int spin_score_partitions(spin_ctx *ctx, int32_t batch, const void *q, const void *summaries,
                                     const int32_t *chan_idx, const int32_t *part_offsets,
                                     const int32_t *seq_lens, float *scores, void *workspace, void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch) return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!q || !summaries || !part_offsets || !seq_lens || !scores) return SPIN_ERR_INVALID;
  (void)workspace;
  const spin_config &c = ctx->cfg;
  const int rows = batch * c.num_kv_heads;
  const int max_pp = ((ctx->max_parts + 15) / 16) * 16;
  hipStream_t st = (hipStream_t)stream;
  const int W = c.score_waves ? c.score_waves : 4;
  if (c.score_kind == SPIN_SCORE_MINMAX) {
    // one tile per wavefront measured best: the dispatcher streams the workgroups
    const int tiles_per_wg = c.score_tiles_per_wg ? c.score_tiles_per_wg : W, max_tiles = max_pp / 16;
    const int wgs = (max_tiles + tiles_per_wg - 1) / tiles_per_wg;
#define SPIN_SCORE_ARGS(RPP)                                                                                  \
  0, st, (const uint16_t *)q, (const uint4 *)summaries, part_offsets, c.num_q_heads, c.num_kv_heads, ctx->group, \
      RPP, tiles_per_wg, wgs, scores
    if (W == 8)
      spin_launch(ctx, SPIN_K_SCORE, spin_score_k32_kernel<8, true, 8>, dim3((unsigned)rows * wgs), dim3(512),
                  SPIN_SCORE_ARGS(1));
    else
      spin_launch(ctx, SPIN_K_SCORE, spin_score_k32_kernel<8, true, 4>, dim3((unsigned)rows * wgs), dim3(256),
                  SPIN_SCORE_ARGS(1));
  } else if (c.score_kind == SPIN_SCORE_REPMAX) {
    const int tiles_per_wg = c.score_tiles_per_wg ? c.score_tiles_per_wg : 2 * W, max_tiles = max_pp * 4 / 16;
    const int wgs = (max_tiles + tiles_per_wg - 1) / tiles_per_wg;
    if (W == 8)
      spin_launch(ctx, SPIN_K_SCORE, spin_score_k32_kernel<4, false, 8>, dim3((unsigned)rows * wgs), dim3(512),
                  SPIN_SCORE_ARGS(4));
    else
      spin_launch(ctx, SPIN_K_SCORE, spin_score_k32_kernel<4, false, 4>, dim3((unsigned)rows * wgs), dim3(256),
                  SPIN_SCORE_ARGS(4));
#undef SPIN_SCORE_ARGS
  } else {
    if (!chan_idx) return SPIN_ERR_INVALID;
    const int tiles_per_wg = 128, max_tiles = max_pp / 16;
    const int wgs = (max_tiles + tiles_per_wg - 1) / tiles_per_wg;
    spin_launch(ctx, SPIN_K_SCORE, spin_score_sketch_kernel, dim3((unsigned)rows * wgs), dim3(SCORE_WAVES * 64), 0, st,
                       (const uint16_t *)q, (const uint2 *)summaries, chan_idx, part_offsets, c.num_q_heads,
                       c.num_kv_heads, ctx->group, tiles_per_wg, wgs, scores);
  }
  return spin_launch_status();
}
