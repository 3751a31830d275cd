// Index: per-partition summaries from the keys in the pool (Section 4.1, Index;
// Table 1: per-page pooling of keys).  Set-up work, not on the per-step path.
//
// Summary rows are written in tiles of 16 rows, chunk-major
// [KD/KC chunks][16 rows][KC elements], the operand image stage 1 loads:
//   MINMAX  row = partition, KD = 256 = [max(128) | min(128)], KC = 8
//   REPMAX  row = partition*4 + r,  KD = 128, KC = 8
//   SKETCH  row = token,            KD = 16,  KC = 4
#include "spin_common.h"

// Index of a 16-byte unit in a wavefront's regrouping buffer: one unit of padding after every 16, so
// that the regrouped reads (lane l reads unit 4 l + i, a 64-byte stride) spread over all LDS banks
// instead of hitting every fourth one.
__device__ inline int spin_lds_pad(int unit) { return unit + (unit >> 4); }

// Two bf16 values in one register <-> two 16-bit integers in the same order (the sign-magnitude
// pattern with the magnitude bits of negative values flipped; the map is its own inverse).  -0 orders
// just below +0; NaN patterns order beyond the infinities, so keys are expected to be finite.
typedef short spin_i16x2 __attribute__((ext_vector_type(2)));
__device__ inline spin_i16x2 spin_bf16x2_order_key(uint32_t w) {
  const spin_i16x2 x = __builtin_bit_cast(spin_i16x2, w);
  return x ^ ((x >> (spin_i16x2){15, 15}) & (spin_i16x2){0x7fff, 0x7fff});
}
__device__ inline uint32_t spin_bf16x2_from_order_key(spin_i16x2 k) {
  return __builtin_bit_cast(uint32_t, k ^ ((k >> (spin_i16x2){15, 15}) & (spin_i16x2){0x7fff, 0x7fff}));
}
template <int CTRL>
__device__ inline spin_i16x2 spin_dpp_i16x2(spin_i16x2 v) {
  const int x = __builtin_bit_cast(int, v);
  return __builtin_bit_cast(spin_i16x2, __builtin_amdgcn_update_dpp(x, x, CTRL, 0xf, 0xf, false));
}

// a double from the lane CTRL names, as two 32-bit exchanges
template <int CTRL>
__device__ inline double spin_dpp_f64(double v) {
  const unsigned long long u = (unsigned long long)__double_as_longlong(v);
  const int lo = (int)(uint32_t)u, hi = (int)(uint32_t)(u >> 32);
  const uint32_t rlo = (uint32_t)__builtin_amdgcn_update_dpp(lo, lo, CTRL, 0xf, 0xf, false);
  const uint32_t rhi = (uint32_t)__builtin_amdgcn_update_dpp(hi, hi, CTRL, 0xf, 0xf, false);
  return __longlong_as_double((long long)(((unsigned long long)rhi << 32) | rlo));
}

// element offset of (summary row R, element e)
__device__ inline size_t summ_off(size_t R, int e, int kd, int kc) {
  return (R >> 4) * (size_t)(16 * kd) + ((size_t)(e / kc) * 16 + (R & 15)) * kc + (e % kc);
}

// One workgroup per 16 partitions of a row: thread = (partition r = tid%16, 8-channel chunk ch = tid/16).
__global__ __launch_bounds__(256) void spin_index_minmax_kernel(
    const uint4 *__restrict__ pool, int64_t pool_slots, const int32_t *__restrict__ dir,
    const int32_t *__restrict__ leaf_pool, int64_t leaf_chunks, const int32_t *__restrict__ part_offsets,
    const int32_t *__restrict__ seq_lens, int Hkv, int tp, int dir_stride, int leaf_entries, int max_tiles,
    uint16_t *__restrict__ summ, int32_t *status, int k_token_major) {
  const int row = blockIdx.x / max_tiles, tile = blockIdx.x - row * max_tiles;
  const int b = row / Hkv, h = row - b * Hkv;
  const int PP = part_offsets[b + 1] - part_offsets[b];
  if (tile * 16 >= PP) return;
  const int N = seq_lens[b];
  const int P = (N + tp - 1) / tp;
  const size_t base = (size_t)Hkv * part_offsets[b] + (size_t)h * PP;
  const int r = threadIdx.x & 15, ch = threadIdx.x >> 4;
  const int p = tile * 16 + r;
  float mn[8], mx[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) { mn[i] = __builtin_inff(); mx[i] = -__builtin_inff(); }
  bool any = false;
  if (p < P) {
    const int t0 = p * tp, t1 = min(t0 + tp, N);
    for (int pg = t0 >> 4; pg <= (t1 - 1) >> 4; ++pg) {
      const int32_t slot = spin_walk(dir, leaf_pool, leaf_chunks, row, dir_stride, leaf_entries, pg);
      if (slot < 0 || (int64_t)slot >= pool_slots) { spin_raise(status, SPIN_ERR_NOT_RESIDENT); continue; }
      const uint4 *kt = pool + (size_t)slot * SPIN_SLOT_U4;
      const int a = max(t0 - pg * 16, 0), e = min(t1 - pg * 16, 16);
      for (int t = a; t < e; ++t) {
        const uint4 v = kt[spin_k_unit(k_token_major, t, ch)];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float lo = __uint_as_float(w[i] << 16), hi = __uint_as_float(w[i] & 0xffff0000u);
          mn[2 * i] = fminf(mn[2 * i], lo); mx[2 * i] = fmaxf(mx[2 * i], lo);
          mn[2 * i + 1] = fminf(mn[2 * i + 1], hi); mx[2 * i + 1] = fmaxf(mx[2 * i + 1], hi);
        }
        any = true;
      }
    }
  }
  uint32_t omx[4], omn[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    // values are bf16 to begin with: the upper halves are exact
    omx[i] = any ? ((__float_as_uint(mx[2 * i]) >> 16) | (__float_as_uint(mx[2 * i + 1]) & 0xffff0000u)) : 0u;
    omn[i] = any ? ((__float_as_uint(mn[2 * i]) >> 16) | (__float_as_uint(mn[2 * i + 1]) & 0xffff0000u)) : 0u;
  }
  const size_t R = base + p;
  uint4 *o = (uint4 *)summ;
  // 16-byte unit index of (row R, chunk): tile*(16*256/8) + chunk*16 + R%16
  const size_t tbase = (R >> 4) * (size_t)(16 * 256 / 8);
  o[tbase + (size_t)ch * 16 + (R & 15)] = make_uint4(omx[0], omx[1], omx[2], omx[3]);
  o[tbase + (size_t)(16 + ch) * 16 + (R & 15)] = make_uint4(omn[0], omn[1], omn[2], omn[3]);
}

// MINMAX for partitions made of whole pages (partition_tokens >= 16), the hot
// Index shape: one workgroup per tile of 16 partitions, each of its four
// wavefronts folds four partitions.  A page's K tile is fetched with four
// contiguous 1 KiB loads, passed through the wavefront's own 4 KiB of LDS to
// regroup it (lane = 8-channel chunk x token quad), folded over the lane's four
// tokens in registers and over the four token quads with two DPP exchanges.
__global__ __launch_bounds__(256) void spin_index_minmax_pages_kernel(
    const uint4 *__restrict__ pool, int64_t pool_slots, const int32_t *__restrict__ dir,
    const int32_t *__restrict__ leaf_pool, int64_t leaf_chunks, const int32_t *__restrict__ part_offsets,
    const int32_t *__restrict__ seq_lens, int Hkv, int tp, int dir_stride, int leaf_entries, int max_tiles,
    uint16_t *__restrict__ summ, int32_t *status, spin_var var) {
  __shared__ uint4 s_tile[4][SPIN_KTILE_U4 + SPIN_KTILE_U4 / 16];   // padded: see spin_lds_pad()
  __shared__ uint4 s_out[512];
  const int row = blockIdx.x / max_tiles, tile = blockIdx.x - row * max_tiles;
  const int b = row / Hkv, h = row - b * Hkv;
  const int PP = part_offsets[b + 1] - part_offsets[b];
  if (tile * 16 >= PP) return;
  const int N = seq_lens[b];
  const size_t base = (size_t)Hkv * part_offsets[b] + (size_t)h * PP;
  int P = var.count ? var.count[row] : (N + tp - 1) / tp;
  P = P < 0 ? 0 : (P > PP ? PP : P);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int ch = lane >> 2, tq = lane & 3;      // after regrouping: chunk of 8 channels, tokens 4tq..4tq+3
  uint4 *lds = s_tile[wave];
  uint4 *o = (uint4 *)summ;
  // uniform partitions: the wavefront's four partitions cover consecutive pages, whose slots are looked
  // up once, one page per lane (two dependent loads for the whole wavefront instead of per page)
  const int ppp = tp >> 4;
  const int pgA = (tile * 16 + wave * 4) * ppp;
  const bool pre = !var.count && 4 * ppp <= 64;
  int32_t myslot = -1;
  if (pre && lane < 4 * ppp && pgA + lane < ((N + 15) >> 4))
    myslot = spin_walk(dir, leaf_pool, leaf_chunks, row, dir_stride, leaf_entries, pgA + lane);
  // ... and the page after the one being folded is already on its way (the wavefront's pages are consecutive)
  const int pgEnd = pre ? min(pgA + 4 * ppp, (N + 15) >> 4) : 0;
  uint4 nv[4];
  bool nok = false;
  auto fetch = [&](int pg) {
    const int32_t slot = __builtin_amdgcn_readlane(myslot, pg - pgA);
    nok = slot >= 0 && (int64_t)slot < pool_slots;
    if (nok) {
      const uint4 *kt = pool + (size_t)slot * SPIN_SLOT_U4 + lane;
#pragma unroll
      for (int j = 0; j < 4; ++j) nv[j] = spin_nt_load(kt + j * 64);
    }
  };
  if (pgA < pgEnd) fetch(pgA);
  for (int k = 0; k < 4; ++k) {
    const int r = wave * 4 + k;                  // partition inside the tile
    const int p = tile * 16 + r;
    // Minimum and maximum are taken on order-preserving 16-bit integer images of the bf16 values, two per
    // register (packed 16-bit min / max): 2.5 instructions per value instead of the 8 or so the float
    // minimum / maximum with their NaN quieting cost, which made this kernel instruction-bound.
    spin_i16x2 mn[4], mx[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) { mn[i] = (spin_i16x2){32767, 32767}; mx[i] = (spin_i16x2){-32768, -32768}; }
    bool any = false;
    if (p < P) {
      // the partition's pages and the token position (in page units of 16) where it ends
      int pg0, t1;
      if (var.count) {
        pg0 = var.first_page[base + p];
        t1 = pg0 * 16 + var.tokens[base + p];
      } else {
        pg0 = (p * tp) >> 4;
        t1 = min(p * tp + tp, N);
      }
      for (int pg = pg0; pg <= (t1 - 1) >> 4; ++pg) {
        if (pre) {
          const bool ok = nok;
          if (ok) {
#pragma unroll
            for (int j = 0; j < 4; ++j) lds[spin_lds_pad(j * 64 + lane)] = nv[j];
          }
          nok = false;
          if (pg + 1 < pgEnd) fetch(pg + 1);
          if (!ok) {
            if (lane == 0) spin_raise(status, SPIN_ERR_NOT_RESIDENT);
            continue;
          }
        } else {
          const int32_t slot = spin_walk(dir, leaf_pool, leaf_chunks, row, dir_stride, leaf_entries, pg);
          if (slot < 0 || (int64_t)slot >= pool_slots) {
            if (lane == 0) spin_raise(status, SPIN_ERR_NOT_RESIDENT);
            continue;
          }
          const uint4 *kt = pool + (size_t)slot * SPIN_SLOT_U4 + lane;
          uint4 v[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] = spin_nt_load(kt + j * 64);
#pragma unroll
          for (int j = 0; j < 4; ++j) lds[spin_lds_pad(j * 64 + lane)] = v[j];
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // same wavefront writes and reads: program order
        const int nvalid = min(t1 - pg * 16, 16);                // tokens of this page inside the partition
        if (nvalid == 16) {                                      // a full page (wave-uniform): no per-token test
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const uint4 u = lds[spin_lds_pad(ch * 16 + 4 * tq + i)];
            const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const spin_i16x2 key = spin_bf16x2_order_key(w[e]);
              mn[e] = __builtin_elementwise_min(mn[e], key);
              mx[e] = __builtin_elementwise_max(mx[e], key);
            }
          }
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const uint4 u = lds[spin_lds_pad(ch * 16 + 4 * tq + i)];
            if (4 * tq + i < nvalid) {
              const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                const spin_i16x2 key = spin_bf16x2_order_key(w[e]);
                mn[e] = __builtin_elementwise_min(mn[e], key);
                mx[e] = __builtin_elementwise_max(mx[e], key);
              }
            }
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        any = true;
      }
    }
    // fold the four token quads (lanes 4ch .. 4ch+3)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      mn[i] = __builtin_elementwise_min(mn[i], spin_dpp_i16x2<SPIN_DPP_XOR1>(mn[i]));
      mn[i] = __builtin_elementwise_min(mn[i], spin_dpp_i16x2<SPIN_DPP_XOR2>(mn[i]));
      mx[i] = __builtin_elementwise_max(mx[i], spin_dpp_i16x2<SPIN_DPP_XOR1>(mx[i]));
      mx[i] = __builtin_elementwise_max(mx[i], spin_dpp_i16x2<SPIN_DPP_XOR2>(mx[i]));
    }
    if (tq == 0) {
      uint32_t omx[4], omn[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        omx[i] = any ? spin_bf16x2_from_order_key(mx[i]) : 0u;
        omn[i] = any ? spin_bf16x2_from_order_key(mn[i]) : 0u;
      }
      // the workgroup's 16 partitions are one 8 KiB summary tile: collected in LDS, written out whole
      s_out[ch * 16 + r] = make_uint4(omx[0], omx[1], omx[2], omx[3]);
      s_out[(16 + ch) * 16 + r] = make_uint4(omn[0], omn[1], omn[2], omn[3]);
    }
  }
  __syncthreads();
  const size_t tbase = ((base + (size_t)tile * 16) >> 4) * (size_t)(16 * 256 / 8);   // base is a multiple of 16
  o[tbase + threadIdx.x] = s_out[threadIdx.x];
  o[tbase + 256 + threadIdx.x] = s_out[256 + threadIdx.x];
}

// fp64 -> bf16 with a single rounding: truncate to fp32 with a sticky low bit
// (round to odd), then round the 16 dropped bits to nearest even.
__device__ inline uint16_t spin_f64_to_bf16(double x) {
  float f = __double2float_rz(x);
  uint32_t u = __float_as_uint(f);
  if ((double)f != x) u |= 1u;
  return spin_f32_to_bf16(__uint_as_float(u));
}

// One workgroup per tile of 16 summary rows (4 partitions x 4 representatives):
// thread = (summary row r = tid%16, 8-channel chunk ch = tid/16).  Sums run in
// fp64, where they are exact for bf16 addends, so the mean has one rounding.
__global__ __launch_bounds__(256) void spin_index_repmean_kernel(
    const uint4 *__restrict__ pool, int64_t pool_slots, const int32_t *__restrict__ dir,
    const int32_t *__restrict__ leaf_pool, int64_t leaf_chunks, const int32_t *__restrict__ part_offsets,
    const int32_t *__restrict__ seq_lens, int Hkv, int tp, int reps, int dir_stride, int leaf_entries,
    int max_tiles, uint16_t *__restrict__ summ, int32_t *status, int k_token_major) {
  const int row = blockIdx.x / max_tiles, tile = blockIdx.x - row * max_tiles;
  const int b = row / Hkv, h = row - b * Hkv;
  const int PP = part_offsets[b + 1] - part_offsets[b];
  if (tile * 16 >= PP * reps) return;
  const int N = seq_lens[b];
  const int P = (N + tp - 1) / tp;
  const size_t base = ((size_t)Hkv * part_offsets[b] + (size_t)h * PP) * reps;
  const int r = threadIdx.x & 15, ch = threadIdx.x >> 4;
  const int sr = tile * 16 + r;            // summary row inside this KV row
  const int p = sr / reps, rep = sr - p * reps;
  const int sub = tp / reps;
  uint32_t outw[4] = {0, 0, 0, 0};
  if (p < P) {
    // an empty sub-range repeats representative 0 of the partition
    int t0 = p * tp + rep * sub, t1 = min(t0 + sub, N);
    if (t1 <= t0) { t0 = p * tp; t1 = min(t0 + sub, N); }
    double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int pg = t0 >> 4; pg <= (t1 - 1) >> 4; ++pg) {
      const int32_t slot = spin_walk(dir, leaf_pool, leaf_chunks, row, dir_stride, leaf_entries, pg);
      if (slot < 0 || (int64_t)slot >= pool_slots) { spin_raise(status, SPIN_ERR_NOT_RESIDENT); continue; }
      const uint4 *kt = pool + (size_t)slot * SPIN_SLOT_U4;
      const int a = max(t0 - pg * 16, 0), e = min(t1 - pg * 16, 16);
      for (int t = a; t < e; ++t) {
        const uint4 v = kt[spin_k_unit(k_token_major, t, ch)];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          acc[2 * i] += (double)__uint_as_float(w[i] << 16);
          acc[2 * i + 1] += (double)__uint_as_float(w[i] & 0xffff0000u);
        }
      }
    }
    const double cnt = (double)(t1 - t0);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      outw[i] = (uint32_t)spin_f64_to_bf16(acc[2 * i] / cnt) | ((uint32_t)spin_f64_to_bf16(acc[2 * i + 1] / cnt) << 16);
  }
  const size_t R = base + sr;
  uint4 *o = (uint4 *)summ;
  const size_t tbase = (R >> 4) * (size_t)(16 * 128 / 8);
  o[tbase + (size_t)ch * 16 + (R & 15)] = make_uint4(outw[0], outw[1], outw[2], outw[3]);
}

// REPMAX when every representative covers whole pages (partition_tokens / reps a multiple of 16),
// the hot shape: one workgroup per tile of 16 summary rows, each of its four wavefronts builds
// four of them.  As in the MINMAX kernel above a page's K tile is fetched with four contiguous
// 1 KiB loads and regrouped through the wavefront's own 4 KiB of LDS (lane = 8-channel chunk x
// token quad); the lane adds its four tokens in fp64 (exact for bf16 addends), the four token
// quads are added with two exchanges, and the mean is rounded once.
__global__ __launch_bounds__(256) void spin_index_repmean_pages_kernel(
    const uint4 *__restrict__ pool, int64_t pool_slots, const int32_t *__restrict__ dir,
    const int32_t *__restrict__ leaf_pool, int64_t leaf_chunks, const int32_t *__restrict__ part_offsets,
    const int32_t *__restrict__ seq_lens, int Hkv, int tp, int reps, int dir_stride, int leaf_entries,
    int max_tiles, uint16_t *__restrict__ summ, int32_t *status, spin_var var) {
  __shared__ uint4 s_tile[4][SPIN_KTILE_U4 + SPIN_KTILE_U4 / 16];   // padded: see spin_lds_pad()
  const int row = blockIdx.x / max_tiles, tile = blockIdx.x - row * max_tiles;
  const int b = row / Hkv, h = row - b * Hkv;
  const int PP = part_offsets[b + 1] - part_offsets[b];
  if (tile * 16 >= PP * reps) return;
  const int N = seq_lens[b];
  // variable-length partitions (one representative each: the mean key of the partition's own tokens)
  int P = var.count ? var.count[row] : (N + tp - 1) / tp;
  P = P < 0 ? 0 : (P > PP ? PP : P);
  const size_t base = ((size_t)Hkv * part_offsets[b] + (size_t)h * PP) * reps;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int ch = lane >> 2, tq = lane & 3;      // after regrouping: chunk of 8 channels, tokens 4tq..4tq+3
  const int sub = tp / reps;
  uint4 *lds = s_tile[wave];
  uint4 *o = (uint4 *)summ;
  // uniform partitions with no empty sub-range among the wavefront's four summary rows: their pages are
  // consecutive, so the slots are looked up once (one page per lane) and the next page is requested
  // while the current one is added up
  const int ppr = sub >> 4;
  const int sr0 = tile * 16 + wave * 4;
  const int pgA = sr0 * ppr;
  const bool pre = !var.count && 4 * ppr <= 64 && (int64_t)(sr0 + 3) * sub < N;
  const int pgEnd = pre ? min(pgA + 4 * ppr, (N + 15) >> 4) : 0;
  int32_t myslot = -1;
  if (lane < 4 * ppr && pgA + lane < pgEnd)
    myslot = spin_walk(dir, leaf_pool, leaf_chunks, row, dir_stride, leaf_entries, pgA + lane);
  uint4 nv[4];
  bool nok = false;
  auto fetch = [&](int pg) {
    const int32_t slot = __builtin_amdgcn_readlane(myslot, pg - pgA);
    nok = slot >= 0 && (int64_t)slot < pool_slots;
    if (nok) {
      const uint4 *kt = pool + (size_t)slot * SPIN_SLOT_U4 + lane;
#pragma unroll
      for (int j = 0; j < 4; ++j) nv[j] = spin_nt_load(kt + j * 64);
    }
  };
  if (pgA < pgEnd) fetch(pgA);
  for (int k = 0; k < 4; ++k) {
    const int sr = sr0 + k;                      // summary row inside this KV row
    const int p = sr / reps, rep = sr - p * reps;
    uint32_t outw[4] = {0, 0, 0, 0};
    if (p < P) {
      // an empty sub-range repeats representative 0 of the partition
      int t0 = p * tp + rep * sub, t1 = min(t0 + sub, N);
      if (t1 <= t0) { t0 = p * tp; t1 = min(t0 + sub, N); }
      if (var.count) {                           // reps == 1: base indexes the tables as it does the rows
        t0 = var.first_page[base + p] * 16;
        t1 = t0 + var.tokens[base + p];
      }
      double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      for (int pg = t0 >> 4; pg <= (t1 - 1) >> 4; ++pg) {
        if (pre) {
          const bool ok = nok;
          if (ok) {
#pragma unroll
            for (int j = 0; j < 4; ++j) lds[spin_lds_pad(j * 64 + lane)] = nv[j];
          }
          nok = false;
          if (pg + 1 < pgEnd) fetch(pg + 1);
          if (!ok) {
            if (lane == 0) spin_raise(status, SPIN_ERR_NOT_RESIDENT);
            continue;
          }
        } else {
          const int32_t slot = spin_walk(dir, leaf_pool, leaf_chunks, row, dir_stride, leaf_entries, pg);
          if (slot < 0 || (int64_t)slot >= pool_slots) {
            if (lane == 0) spin_raise(status, SPIN_ERR_NOT_RESIDENT);
            continue;
          }
          const uint4 *kt = pool + (size_t)slot * SPIN_SLOT_U4 + lane;
          uint4 v[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] = spin_nt_load(kt + j * 64);
#pragma unroll
          for (int j = 0; j < 4; ++j) lds[spin_lds_pad(j * 64 + lane)] = v[j];
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // same wavefront writes and reads: program order
        const int nvalid = min(t1 - pg * 16, 16);                // the sub-range starts on a page boundary
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const uint4 u = lds[spin_lds_pad(ch * 16 + 4 * tq + i)];
          if (4 * tq + i < nvalid) {
            const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              acc[2 * e] += (double)__uint_as_float(w[e] << 16);
              acc[2 * e + 1] += (double)__uint_as_float(w[e] & 0xffff0000u);
            }
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      }
      // add the four token quads (lanes 4ch .. 4ch+3); exact sums, so the order does not matter
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        acc[i] += spin_dpp_f64<SPIN_DPP_XOR1>(acc[i]);
        acc[i] += spin_dpp_f64<SPIN_DPP_XOR2>(acc[i]);
      }
      // the mean: a token count that is a power of two (the usual case) divides exactly through its reciprocal
      const int n = t1 - t0;
      const double cnt = (double)n, inv = 1.0 / cnt;
      if ((n & (n - 1)) == 0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] *= inv;
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] /= cnt;
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
        outw[i] = (uint32_t)spin_f64_to_bf16(acc[2 * i]) | ((uint32_t)spin_f64_to_bf16(acc[2 * i + 1]) << 16);
    }
    if (tq == 0) {
      const size_t R = base + sr;
      const size_t tbase = (R >> 4) * (size_t)(16 * 128 / 8);
      o[tbase + (size_t)ch * 16 + (R & 15)] = make_uint4(outw[0], outw[1], outw[2], outw[3]);
    }
  }
}

// SKETCH (token partitions): the 16 sketched channels of every key.  One workgroup per 16 pages, four
// per wavefront: a page's K tile is fetched whole with four contiguous 1 KiB loads (picking 2-byte
// elements straight from HBM moved the same cache lines at 4 TB/s), the next page being requested
// while the current one is used; lane (channel quad, token) then picks its four elements from the
// wavefront's LDS copy, and the page's 512-byte summary tile leaves as one contiguous store.
__global__ __launch_bounds__(256) void spin_index_sketch_kernel(
    const uint4 *__restrict__ pool, int64_t pool_slots, const int32_t *__restrict__ dir,
    const int32_t *__restrict__ leaf_pool, int64_t leaf_chunks, const int32_t *__restrict__ part_offsets,
    const int32_t *__restrict__ seq_lens, const int32_t *__restrict__ chan, int Hkv, int dir_stride,
    int leaf_entries, int max_tiles, uint16_t *__restrict__ summ, int32_t *status, int k_token_major) {
  __shared__ uint4 s_tile[4][SPIN_KTILE_U4 + SPIN_KTILE_U4 / 16];   // padded: see spin_lds_pad()
  const int row = blockIdx.x / max_tiles, tile = blockIdx.x - row * max_tiles;
  const int b = row / Hkv, h = row - b * Hkv;
  const int PP = part_offsets[b + 1] - part_offsets[b];   // tokens of the padded row, a multiple of 16
  const int pages_pad = PP >> 4;
  if (tile * 16 >= pages_pad) return;
  const int N = seq_lens[b];
  const int pages = min((N + 15) >> 4, pages_pad);
  const size_t base = (size_t)Hkv * part_offsets[b] + (size_t)h * PP;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int cq = lane >> 4, r = lane & 15;       // channel quad, token of the page
  const uint16_t *lds = (const uint16_t *)s_tile[wave];
  uint4 *ldsw = s_tile[wave];
  int at[4];                                     // where the lane's four elements sit in the LDS copy
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int d = chan[h * 16 + cq * 4 + i] & (SPIN_HEAD_DIM - 1);   // a channel outside the head reads inside it
    at[i] = spin_lds_pad(spin_k_unit(k_token_major, r, d >> 3)) * 8 + (d & 7);
  }
  const int pgA = tile * 16 + wave * 4;
  const int pgEnd = min(pgA + 4, pages);
  int32_t myslot = -1;
  if (lane < 4 && pgA + lane < pgEnd)
    myslot = spin_walk(dir, leaf_pool, leaf_chunks, row, dir_stride, leaf_entries, pgA + lane);
  uint4 nv[4];
  bool nok = false;
  auto fetch = [&](int pg) {
    const int32_t slot = __builtin_amdgcn_readlane(myslot, pg - pgA);
    nok = slot >= 0 && (int64_t)slot < pool_slots;
    if (nok) {
      const uint4 *kt = pool + (size_t)slot * SPIN_SLOT_U4 + lane;
#pragma unroll
      for (int j = 0; j < 4; ++j) nv[j] = spin_nt_load(kt + j * 64);
    }
  };
  if (pgA < pgEnd) fetch(pgA);
  uint2 *o = (uint2 *)summ;
  for (int pg = pgA; pg < min(pgA + 4, pages_pad); ++pg) {
    uint2 out = make_uint2(0u, 0u);              // tokens past the context and pages that are not resident: zeros
    if (pg < pgEnd) {
      const bool ok = nok;
      if (ok) {
#pragma unroll
        for (int j = 0; j < 4; ++j) ldsw[spin_lds_pad(j * 64 + lane)] = nv[j];
      }
      nok = false;
      if (pg + 1 < pgEnd) fetch(pg + 1);
      if (!ok) {
        if (lane == 0) spin_raise(status, SPIN_ERR_NOT_RESIDENT);
      } else {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // same wavefront writes and reads: program order
        if (pg * 16 + r < N)
          out = make_uint2(lds[at[0]] | ((uint32_t)lds[at[1]] << 16), lds[at[2]] | ((uint32_t)lds[at[3]] << 16));
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      }
    }
    // the page's summary tile [4 channel quads][16 tokens][4 elements]: 64 x 8 bytes, lane by lane
    o[((base >> 4) + (size_t)pg) * 64 + lane] = out;
  }
}

extern "C" int spin_build_summaries(spin_ctx *ctx, int32_t batch, const void *kv_pool, int64_t pool_slots,
                                    const int32_t *dir, const int32_t *leaf_pool, int64_t leaf_chunks,
                                    const int32_t *part_offsets, const int32_t *seq_lens,
                                    const int32_t *chan_idx, void *summaries, void *workspace, void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch || pool_slots <= 0 || leaf_chunks <= 0) return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!kv_pool || !dir || !leaf_pool || !part_offsets || !seq_lens || !summaries) return SPIN_ERR_INVALID;
  if (!workspace) return SPIN_ERR_WORKSPACE;
  const spin_config &c = ctx->cfg;
  // variable-length partitions: min/max keys, or one mean key (centroid) per partition
  if (ctx->var.count && !(c.partition_tokens >= 16 &&
                          (c.score_kind == SPIN_SCORE_MINMAX ||
                           (c.score_kind == SPIN_SCORE_REPMAX && c.reps_per_partition == 1))))
    return SPIN_ERR_UNSUPPORTED;
  const int rows = batch * c.num_kv_heads;
  const int max_pp = ((ctx->max_parts + 15) / 16) * 16;
  hipStream_t st = (hipStream_t)stream;
  int32_t *status = (int32_t *)workspace;
  if (c.score_kind == SPIN_SCORE_MINMAX) {
    const int max_tiles = max_pp / 16;
    if (c.partition_tokens >= 16)
      spin_launch(ctx, SPIN_K_INDEX, spin_index_minmax_pages_kernel, dim3((unsigned)rows * max_tiles), dim3(256), 0, st,
                  (const uint4 *)kv_pool, pool_slots, dir, leaf_pool, leaf_chunks, part_offsets, seq_lens,
                  c.num_kv_heads, c.partition_tokens, ctx->dir_stride, c.leaf_entries, max_tiles,
                  (uint16_t *)summaries, status, ctx->var);
    else
      spin_launch(ctx, SPIN_K_INDEX, spin_index_minmax_kernel, dim3((unsigned)rows * max_tiles), dim3(256), 0, st,
                       (const uint4 *)kv_pool, pool_slots, dir, leaf_pool, leaf_chunks, part_offsets, seq_lens,
                       c.num_kv_heads, c.partition_tokens, ctx->dir_stride, c.leaf_entries, max_tiles,
                       (uint16_t *)summaries, status, ctx->k_token_major);
  } else if (c.score_kind == SPIN_SCORE_REPMAX) {
    const int max_tiles = max_pp * c.reps_per_partition / 16;
    if ((c.partition_tokens / c.reps_per_partition) % 16 == 0 || ctx->var.count)
      spin_launch(ctx, SPIN_K_INDEX, spin_index_repmean_pages_kernel, dim3((unsigned)rows * max_tiles), dim3(256), 0, st,
                  (const uint4 *)kv_pool, pool_slots, dir, leaf_pool, leaf_chunks, part_offsets, seq_lens,
                  c.num_kv_heads, c.partition_tokens, c.reps_per_partition, ctx->dir_stride, c.leaf_entries,
                  max_tiles, (uint16_t *)summaries, status, ctx->var);
    else
      spin_launch(ctx, SPIN_K_INDEX, spin_index_repmean_kernel, dim3((unsigned)rows * max_tiles), dim3(256), 0, st,
                  (const uint4 *)kv_pool, pool_slots, dir, leaf_pool, leaf_chunks, part_offsets, seq_lens,
                  c.num_kv_heads, c.partition_tokens, c.reps_per_partition, ctx->dir_stride, c.leaf_entries,
                  max_tiles, (uint16_t *)summaries, status, ctx->k_token_major);
  } else {
    if (!chan_idx) return SPIN_ERR_INVALID;
    if (c.partition_tokens != 1) return SPIN_ERR_UNSUPPORTED;
    const int max_tiles = (max_pp / 16 + 15) / 16;   // 16 pages per workgroup
    spin_launch(ctx, SPIN_K_INDEX, spin_index_sketch_kernel, dim3((unsigned)rows * max_tiles), dim3(256), 0, st,
                       (const uint4 *)kv_pool, pool_slots, dir, leaf_pool, leaf_chunks, part_offsets, seq_lens,
                       chan_idx, c.num_kv_heads, ctx->dir_stride, c.leaf_entries, max_tiles,
                       (uint16_t *)summaries, status, ctx->k_token_major);
  }
  return spin_launch_status();
}
