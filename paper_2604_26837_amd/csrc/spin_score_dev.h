// Device code of stage 1 shared by the stand-alone kernel and the fused launch.
#pragma once
#include "spin_common.h"

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

// maximum over the heads of the group of a 16 x 16 tile S[head][column] held as lane (n, c):
// S[4c+i][n]; the result is valid in every lane
__device__ inline float spin_head_max(const spin_f32x4 &s, int c, int G) {
  float m = -__builtin_inff();
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (4 * c + i < G) m = fmaxf(m, s[i]);
  if (G > 4) {
    m = fmaxf(m, __shfl_xor(m, 16));
    m = fmaxf(m, __shfl_xor(m, 32));
  }
  return m;
}

// what a workgroup that also counts stage 2's first histogram needs: the LDS bins and the row's candidate range
struct score_bins {
  int *bins;            // [BIG_BINS] in LDS
  int cand_lo, cand_hi; // partitions [cand_lo, cand_hi) are candidates of stage 2
};

template <int NJ, bool MINMAX, bool HIST = false>
__device__ inline void consume_tile(const score_tile<NJ> &r, const spin_bf16x8 (&qf)[NJ], int n, int c, int G,
                                    int rpp, float *__restrict__ scores, size_t base, int t,
                                    score_bins hb = score_bins{nullptr, 0, 0}) {
  // the queries are the A operand, the summary rows the B operand: lane (n, c) ends up with
  // S[head 4c+i][summary row n], so the maximum over the group's heads stays inside the lane
  // (plus two exchanges between the lane quarters when the group has more than 4 heads)
  spin_f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int j = 0; j < NJ; ++j)
    s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf[j], __builtin_bit_cast(spin_bf16x8, r.a[j]), s, 0, 0, 0);
  float m = spin_head_max(s, c, G);
  if (MINMAX) {
    if (c == 0) {
      scores[base + (size_t)t * 16 + n] = m;
      if (HIST) {
        const int p = t * 16 + n;
        if (p >= hb.cand_lo && p < hb.cand_hi) atomicAdd(&hb.bins[score_key(m) >> 20], 1);
      }
    }
  } else {
    // rows rpp*p .. rpp*p + rpp-1 (rpp = 1, 2 or 4) are the representatives of partition (16/rpp) t + p:
    // neighbouring lanes n
    if (rpp >= 2) m = fmaxf(m, spin_dpp<SPIN_DPP_XOR1>(m));
    if (rpp == 4) m = fmaxf(m, spin_dpp<SPIN_DPP_XOR2>(m));
    if (c == 0 && (n & (rpp - 1)) == 0) {
      scores[base + (size_t)t * (16 / rpp) + n / rpp] = m;
      if (HIST) {
        const int p = t * (16 / rpp) + n / rpp;
        if (p >= hb.cand_lo && p < hb.cand_hi) atomicAdd(&hb.bins[score_key(m) >> 20], 1);
      }
    }
  }
}

// Scores the tiles [chunk*tiles_per_wg, +tiles_per_wg) of one row with the calling
// workgroup (WAVES wavefronts).
template <int NJ, bool MINMAX, int WAVES, bool HIST = false>
__device__ inline void score_row_tiles(
    const uint16_t *__restrict__ q, const uint4 *__restrict__ summ, const int32_t *__restrict__ part_offsets,
    int Hq, int Hkv, int G, int rows_per_part, int tiles_per_wg, int row, int chunk, float *__restrict__ scores,
    score_bins hb = score_bins{nullptr, 0, 0}) {
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

  // A operand: row n = query head, k = elements 32j + 8c .. +8 of the query-side vector
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
    consume_tile<NJ, MINMAX, HIST>(ra, qf, n, c, G, rows_per_part, scores, base, t, hb);
    if (t2 < t_end) load_tile<NJ>(ra, tiles + (size_t)t2 * (NJ * 64), lane);
    if (t1 < t_end) consume_tile<NJ, MINMAX, HIST>(rb, qf, n, c, G, rows_per_part, scores, base, t1, hb);
  }
}

// One tile per wavefront (tiles_per_wg == WAVES, the default launch): no loop and no second
// tile buffer, which keeps the kernel at fewer registers and more wavefronts in flight per
// compute unit; the tile is requested before the query vectors are gathered.
template <int NJ, bool MINMAX, int WAVES>
__device__ inline void score_row_single_tile(
    const uint16_t *__restrict__ q, const uint4 *__restrict__ summ, const int32_t *__restrict__ part_offsets,
    int Hq, int Hkv, int G, int rows_per_part, int row, int chunk, float *__restrict__ scores) {
  const int b = row / Hkv, h = row - b * Hkv;
  const int off_b = part_offsets[b];
  const int PP = part_offsets[b + 1] - off_b;
  const int ntiles = PP * rows_per_part / 16;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t = chunk * WAVES + wave;
  if (t >= ntiles) return;
  const int n = lane & 15, c = lane >> 4;
  const size_t base = (size_t)Hkv * off_b + (size_t)h * PP;   // in partitions
  const uint4 *tiles = summ + base * rows_per_part * (NJ * 4);
  score_tile<NJ> r;
  load_tile<NJ>(r, tiles + (size_t)t * (NJ * 64), lane);
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
  consume_tile<NJ, MINMAX>(r, qf, n, c, G, rows_per_part, scores, base, t);
}

