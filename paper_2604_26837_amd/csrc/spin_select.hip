// Stage 2: per row, forced partitions plus the k' best-scoring candidates
// (Table 1, "-> topk"; Section 4.2: the always-attended windows are filtered
// out of the candidates).
//
// One workgroup per row.  Scores become order-preserving 32-bit keys (NaN ->
// -inf, -0 -> +0); an MSB-first radix select (four 8-bit passes, LDS
// histogram, parallel suffix scan) finds the key T of the k'-th best
// candidate; then one index-ordered compaction emits every forced partition,
// every candidate with key > T and the lowest-index candidates with key == T
// that are still needed.  Because emission is in index order the output is
// ascending and ties go to the lower id without any sort.
#include "spin_resolve_dev.h"
#include "spin_select_dev.h"

#define SEL_BLOCK 512

// exclusive prefix sum of one int per thread over the workgroup, plus the total
template <int BLOCK>
__device__ inline int block_exclusive_scan(int v, int *s_wave, int &total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int inc = spin_wave_inclusive_scan(v);
  __syncthreads();  // s_wave may still be read from a previous scan
  if (lane == 63) s_wave[wave] = inc;
  __syncthreads();
  int off = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < BLOCK / 64; ++w) {
    const int x = s_wave[w];
    if (w < wave) off += x;
    tot += x;
  }
  total = tot;
  return off + inc - v;
}

// Rows of any length: every pass re-reads the row's scores.
template <int BLOCK>
__device__ inline void select_generic_row(
    const float *__restrict__ scores, const int32_t *__restrict__ part_offsets,
    const int32_t *__restrict__ seq_lens, int Hkv, int tp, int topk, int includes_forced, int sink_pages,
    int recent_pages, int sel_stride, int32_t *__restrict__ sel, int32_t *__restrict__ nsel, int row) {
  __shared__ int s_hist[256];
  __shared__ int s_wave[BLOCK / 64];
  __shared__ int s_digit, s_remaining;

  const int b = row / Hkv, h = row - b * Hkv;
  const int N = seq_lens[b];
  const int PP = part_offsets[b + 1] - part_offsets[b];
  const float *rs = scores + (size_t)Hkv * part_offsets[b] + (size_t)h * PP;
  int32_t *rsel = sel + (size_t)row * sel_stride;
  const int tid = threadIdx.x;
  int P = N > 0 ? (N + tp - 1) / tp : 0;
  if (P > PP) P = PP;

  // forced partitions: a prefix [0, nf_lo) and a suffix [first_hi, P)
  const int pages = (N + 15) >> 4;
  int sink_end = min(sink_pages, pages);
  int recent_begin = max(pages - recent_pages, 0);
  if (sink_end >= recent_begin) { sink_end = pages; recent_begin = pages; }
  int nf_lo = (N <= sink_end * 16) ? P : (sink_end * 16) / tp;
  int first_hi = min((recent_begin * 16 + tp - 1) / tp, P);
  if (first_hi <= nf_lo) { nf_lo = P; first_hi = P; }
  const int nforced = nf_lo + (P - first_hi);
  const int ncand = P - nforced;
  int kprime = includes_forced ? max(topk - nforced, 0) : topk;
  kprime = min(kprime, ncand);
  int take = nforced + kprime;
  if (take > sel_stride) {   // cannot happen for strides from spin_sel_stride(); keep stores in range
    kprime = max(sel_stride - nforced, 0);
    take = min(nforced + kprime, sel_stride);
  }

  // contiguous chunk of partitions per thread
  int chunk = (P + BLOCK - 1) / BLOCK;
  chunk = (chunk + 3) & ~3;
  const int c0 = min(tid * chunk, P), c1 = min(c0 + chunk, P);

  // ---- radix select of the kprime-th largest candidate key ----
  uint32_t prefix = 0;
  int remaining = kprime;   // rank (1-based) of the wanted key among keys matching the prefix
  if (kprime > 0) {
    for (int shift = 24; shift >= 0; shift -= 8) {
      if (tid < 256) s_hist[tid] = 0;
      __syncthreads();
      for (int p = c0; p < c1; ++p) {
        if (p < nf_lo || p >= first_hi) continue;
        const uint32_t k = score_key(rs[p]);
        if (shift == 24 || (k >> (shift + 8)) == prefix) atomicAdd(&s_hist[(k >> shift) & 255u], 1);
      }
      __syncthreads();
      // suffix sums over digits: thread t looks at digit 255 - t
      int cnt = tid < 256 ? s_hist[255 - tid] : 0, total;
      const int excl = block_exclusive_scan<BLOCK>(cnt, s_wave, total);
      if (tid < 256 && excl < remaining && excl + cnt >= remaining) {
        s_digit = 255 - tid;
        s_remaining = remaining - excl;
      }
      __syncthreads();
      prefix = (prefix << 8) | (uint32_t)s_digit;
      remaining = s_remaining;
      __syncthreads();
    }
  }
  const uint32_t T = prefix;
  const int need_eq = kprime > 0 ? remaining : 0;   // how many candidates with key == T to take

  // ---- index-ordered compaction ----
  int my_gt = 0, my_eq = 0;
  for (int p = c0; p < c1; ++p) {
    if (p < nf_lo || p >= first_hi) { ++my_gt; continue; }
    if (kprime == 0) continue;
    const uint32_t k = score_key(rs[p]);
    my_gt += k > T;
    my_eq += k == T;
  }
  int total_eq, total_sel;
  const int eq_before = block_exclusive_scan<BLOCK>(my_eq, s_wave, total_eq);
  int eq_quota = min(max(need_eq - eq_before, 0), my_eq);
  const int pos0 = block_exclusive_scan<BLOCK>(my_gt + eq_quota, s_wave, total_sel);
  int pos = pos0;
  for (int p = c0; p < c1; ++p) {
    bool pick;
    if (p < nf_lo || p >= first_hi) pick = true;
    else if (kprime == 0) pick = false;
    else {
      const uint32_t k = score_key(rs[p]);
      pick = k > T;
      if (k == T && eq_quota > 0) { pick = true; --eq_quota; }
    }
    if (pick && pos < sel_stride) rsel[pos++] = p;
  }
  for (int i = take + tid; i < sel_stride; i += BLOCK) rsel[i] = -1;
  if (tid == 0) nsel[row] = min(total_sel, sel_stride);
}

__global__ __launch_bounds__(SEL_BLOCK) void spin_select_kernel(
    const float *__restrict__ scores, const int32_t *__restrict__ part_offsets,
    const int32_t *__restrict__ seq_lens, int Hkv, int tp, int topk, int includes_forced, int sink_pages,
    int recent_pages, int sel_stride, int32_t *__restrict__ sel, int32_t *__restrict__ nsel) {
  select_generic_row<SEL_BLOCK>(scores, part_offsets, seq_lens, Hkv, tp, topk, includes_forced, sink_pages,
                                recent_pages, sel_stride, sel, nsel, (int)blockIdx.x);
}

template <int BLOCK, int KPT>
__global__ __launch_bounds__(BLOCK) void spin_select_reg_kernel(
    const float *__restrict__ scores, const int32_t *__restrict__ part_offsets,
    const int32_t *__restrict__ seq_lens, int Hkv, int tp, int topk, int includes_forced, int sink_pages,
    int recent_pages, int sel_stride, int32_t *__restrict__ sel, int32_t *__restrict__ nsel, spin_var var) {
  (void)select_reg_row<BLOCK, KPT>(scores, part_offsets, seq_lens, Hkv, tp, topk, includes_forced, sink_pages,
                                          recent_pages, sel_stride, sel, nsel, (int)blockIdx.x, var);
}

// ---------------------------------------------------------------------------
// Long rows (more than 16384 partitions, e.g. token partitions of a 64K context).
//
// A single workgroup spends most of its time walking a long row several times,
// so the first digit is settled by the whole chip instead: a first launch, many
// workgroups per row, histograms the top 12 key bits of the candidates into the
// workspace.  The second launch, one workgroup per row, finds the bin D of the
// k'-th candidate from it, walks the row ONCE (coalesced, order does not
// matter): partitions above bin D and forced partitions set their bit in an LDS
// bitmap, the few keys inside bin D go to an LDS list, where three short radix
// passes over the remaining 20 bits find the threshold key T.  List entries
// above T join the bitmap, entries equal to T a second bitmap; one ordered walk
// over both emits the indices ascending, taking the lowest-index ties first.
// A row whose bin D does not fit the list (heavy ties) falls back, inside the
// same launch, to the multi-pass algorithms above; the results are the same.
#define BIG_CHUNK 8192
#define BIG_BLOCK 1024
#define BIG_CAP 3072

__global__ __launch_bounds__(256) void spin_select_hist_kernel(
    const float *__restrict__ scores, const int32_t *__restrict__ part_offsets,
    const int32_t *__restrict__ seq_lens, int Hkv, int tp, int topk, int includes_forced, int sink_pages,
    int recent_pages, int sel_stride, int32_t *__restrict__ hist) {
  __shared__ int s_h[BIG_BINS];
  const int row = blockIdx.y, tid = threadIdx.x;
  const int b = row / Hkv, h = row - b * Hkv;
  const int PP = part_offsets[b + 1] - part_offsets[b];
  const float *rs = scores + (size_t)Hkv * part_offsets[b] + (size_t)h * PP;
  const sel_plan pl = select_plan(seq_lens[b], PP, tp, topk, includes_forced, sink_pages, recent_pages, sel_stride);
  const int lo = max((int)blockIdx.x * BIG_CHUNK, pl.nf_lo);
  const int hi = min(((int)blockIdx.x + 1) * BIG_CHUNK, pl.first_hi);
  if (lo >= hi || pl.kprime == 0) return;
  for (int i = tid; i < BIG_BINS; i += 256) s_h[i] = 0;
  __syncthreads();
  // the chunk's 8192 scores as 8 aligned 16-byte loads per thread, all issued before the first use
  // (rows are padded to a multiple of 16 partitions, so a load never leaves the row)
  float4 f[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int p4 = (int)blockIdx.x * BIG_CHUNK + (i * 256 + tid) * 4;
    f[i] = p4 < PP ? *(const float4 *)(rs + p4) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int p4 = (int)blockIdx.x * BIG_CHUNK + (i * 256 + tid) * 4;
    const float v[4] = {f[i].x, f[i].y, f[i].z, f[i].w};
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (p4 + e >= lo && p4 + e < hi) atomicAdd(&s_h[score_key(v[e]) >> 20], 1);
  }
  __syncthreads();
  for (int i = tid; i < BIG_BINS; i += 256) {
    const int c = s_h[i];
    if (c) atomicAdd(&hist[(size_t)row * BIG_BINS + i], c);
  }
}

// The smallest score whose key is at least K (keys as in score_key).  Bit patterns that are no
// ordered number: below -inf every real key of the bin is at least key(-inf), so `low_end` asks
// for -inf there; above +inf no key exists and the NaN returned fails every comparison.
__device__ inline float key_floor_score(uint32_t K, bool low_end) {
  const uint32_t u = (K & 0x80000000u) ? (K ^ 0x80000000u) : ~K;
  if ((u & 0x7fffffffu) > 0x7f800000u) return (low_end && (u & 0x80000000u)) ? -__builtin_inff() : __builtin_nanf("");
  return __uint_as_float(u);
}

// The multi-pass algorithms for a row the one-walk path cannot take.  Kept out of line: they keep
// up to 64 keys per thread in registers, which must not shape the register allocation of the
// common path (measured: 18.6 -> 18.0 us on 64 rows of 65536 tokens).
__device__ __attribute__((noinline)) void select_big_fallback(
    const float *__restrict__ scores, const int32_t *__restrict__ part_offsets,
    const int32_t *__restrict__ seq_lens, int Hkv, int tp, int topk, int includes_forced, int sink_pages,
    int recent_pages, int sel_stride, int32_t *__restrict__ sel, int32_t *__restrict__ nsel, int row, int P) {
  if (P <= BIG_BLOCK * 64) {
    spin_var none = {};
    (void)select_reg_row<BIG_BLOCK, 64>(scores, part_offsets, seq_lens, Hkv, tp, topk, includes_forced, sink_pages,
                                               recent_pages, sel_stride, sel, nsel, row, none);
  } else {
    select_generic_row<BIG_BLOCK>(scores, part_offsets, seq_lens, Hkv, tp, topk, includes_forced, sink_pages,
                                  recent_pages, sel_stride, sel, nsel, row);
  }
}

// RESOLVE: the workgroup goes on to stage 3 for its row (same device function as the stage call).
template <bool RESOLVE>
__global__ __launch_bounds__(BIG_BLOCK) void spin_select_big_kernel(
    const float *__restrict__ scores, const int32_t *__restrict__ part_offsets,
    const int32_t *__restrict__ seq_lens, int Hkv, int tp, int topk, int includes_forced, int sink_pages,
    int recent_pages, int sel_stride, int32_t *sel, int32_t *__restrict__ nsel, int32_t *hist,
    int words_max, spin_resolve_args ra, int page_stride, int dir_stride, int leaf_entries, int32_t *status) {
  extern __shared__ uint32_t s_dyn[];
  uint32_t *s_main = s_dyn;                              // [words_max] bit p: partition p is selected
  uint32_t *s_eq = s_dyn + words_max;                    // [words_max] bit p: candidate p has the threshold key
  uint2 *s_list = (uint2 *)(s_dyn + 2 * words_max);      // [BIG_CAP] {key, partition} of the keys in bin D
  __shared__ int s_wave[BIG_BLOCK / 64];
  __shared__ unsigned long long s_wtot[BIG_BLOCK / 64];
  __shared__ int s_h[256];
  __shared__ int s_D, s_r, s_cntD, s_n, s_digit, s_remaining;

  const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = row / Hkv, h = row - b * Hkv;
  const int PP = part_offsets[b + 1] - part_offsets[b];
  const float *rs = scores + (size_t)Hkv * part_offsets[b] + (size_t)h * PP;
  int32_t *rsel = sel + (size_t)row * sel_stride;
  const sel_plan pl = select_plan(seq_lens[b], PP, tp, topk, includes_forced, sink_pages, recent_pages, sel_stride);
  const int P = pl.P, kprime = pl.kprime;
  const int W = (P + 31) >> 5;

  // bin of the k'-th candidate: thread t owns bins 4095-4t .. 4092-4t, highest first
  int4 *rh4 = (int4 *)(hist + (size_t)row * BIG_BINS) + (BIG_BINS / 4 - 1 - tid);   // one 16-byte load and store
  const int4 h4 = *rh4;
  *rh4 = make_int4(0, 0, 0, 0);                            // ready for the next launch
  const int hv[4] = {h4.w, h4.z, h4.y, h4.x};
  const int local = h4.x + h4.y + h4.z + h4.w;
  if (tid == 0) { s_D = BIG_BINS; s_r = 0; s_cntD = 0; s_n = 0; }
  int total;
  int running = block_exclusive_scan<BIG_BLOCK>(local, s_wave, total);   // its barriers order the lines above
  if (kprime > 0) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (running < kprime && running + hv[j] >= kprime) {
        s_D = BIG_BINS - 1 - 4 * tid - j;
        s_r = kprime - running;
        s_cntD = hv[j];
      }
      running += hv[j];
    }
  }
  __syncthreads();
  const int D = s_D;
  // (bin 7 holds -inf and the NaN scores, which rank as -inf: the walk below compares scores as
  // floats and would not see the NaNs, so that bin goes the multi-pass way as well)
  if (kprime > 0 && (D == BIG_BINS || D == 7 || s_cntD > BIG_CAP || W > words_max)) {
    // heavy ties in the threshold bin (or a histogram that does not cover the row): multi-pass algorithms
    select_big_fallback(scores, part_offsets, seq_lens, Hkv, tp, topk, includes_forced, sink_pages, recent_pages,
                        sel_stride, sel, nsel, row, P);
    if (RESOLVE) {
      __syncthreads();   // the selection was written by this workgroup: visible to all its threads from here
      resolve_row<BIG_BLOCK>(row, pl.take, sel, seq_lens, ra.dir, ra.leaf_pool, ra.leaf_chunks, Hkv, tp, sink_pages,
                             recent_pages, sel_stride, page_stride, dir_stride, leaf_entries, ra.slots, ra.page_ids,
                             ra.valid_mask, ra.npages, status, spin_var{});
    }
    return;
  }

  // the bitmaps start with the forced partitions [0, nf_lo) and [first_hi, P) set
  for (int i = tid; i < W; i += BIG_BLOCK) {
    const int p0 = i * 32;
    uint32_t m = 0;
    if (p0 < pl.nf_lo) m |= pl.nf_lo - p0 >= 32 ? 0xffffffffu : (1u << (pl.nf_lo - p0)) - 1u;
    if (p0 + 32 > pl.first_hi) {
      const uint32_t from = p0 >= pl.first_hi ? 0xffffffffu : ~((1u << (pl.first_hi - p0)) - 1u);
      const uint32_t upto = P - p0 >= 32 ? 0xffffffffu : (1u << (P - p0)) - 1u;   // P > p0: i < W
      m |= from & upto;
    }
    s_main[i] = m;
    s_eq[i] = 0;
  }
  __syncthreads();

  // One walk over the row, 16-byte loads, eight per thread in flight.  Membership of a score in
  // bin D or above is decided on the float itself: the key is monotone in the score, so
  // key >= K  <=>  score >= (the score whose key is K); a NaN score fails every comparison, which is
  // right above the bin of -inf (the rank NaN has as a key).  The exact key is only formed for the
  // few scores that join the list.
  const float f_lo = key_floor_score((uint32_t)D << 20, true);
  const float f_hi = D + 1 < BIG_BINS ? key_floor_score(((uint32_t)D + 1u) << 20, false) : __builtin_nanf("");
  for (int base = 0; base < P && kprime > 0; base += BIG_BLOCK * 32) {
    float4 f[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int p4 = base + (i * BIG_BLOCK + tid) * 4;
      f[i] = p4 < PP ? *(const float4 *)(rs + p4) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    // non-candidates (forced partitions, the padding past P) become NaN, which fails every comparison;
    // only the loads that straddle an end of the candidate range have any
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int p4 = base + (i * BIG_BLOCK + tid) * 4;
      if (!(p4 >= pl.nf_lo && p4 + 4 <= pl.first_hi)) {
        if (p4 + 0 < pl.nf_lo || p4 + 0 >= pl.first_hi) f[i].x = __builtin_nanf("");
        if (p4 + 1 < pl.nf_lo || p4 + 1 >= pl.first_hi) f[i].y = __builtin_nanf("");
        if (p4 + 2 < pl.nf_lo || p4 + 2 >= pl.first_hi) f[i].z = __builtin_nanf("");
        if (p4 + 3 < pl.nf_lo || p4 + 3 >= pl.first_hi) f[i].w = __builtin_nanf("");
      }
    }
    // classify the thread's 32 scores: bit 4i+e of `above` / `in_d` = score e of load i lies above bin D /
    // in it.  One comparison per score; the rest only runs when some lane of the wavefront passes it.
    uint32_t above = 0, in_d = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float v[4] = {f[i].x, f[i].y, f[i].z, f[i].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool ge_lo = v[e] >= f_lo;
        if (__ballot(ge_lo) == 0ull) continue;
        const bool ge_hi = v[e] >= f_hi;
        above |= (ge_lo && ge_hi) ? 1u << (4 * i + e) : 0u;
        in_d |= (ge_lo && !ge_hi) ? 1u << (4 * i + e) : 0u;
      }
    }
    if (above) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int p4 = base + (i * BIG_BLOCK + tid) * 4;
        const uint32_t bits = (above >> (4 * i)) & 0xfu;
        if (bits) atomicOr(&s_main[p4 >> 5], bits << (p4 & 31));   // p4 is a multiple of 4: the bits stay in one word
      }
    }
    // the scores in bin D join the list: one counter update per wavefront and batch
    if (__ballot(in_d != 0u)) {
      const int mine = __popc(in_d);
      const int inc = spin_wave_inclusive_scan(mine);
      int first = 0;
      if (lane == 63) first = atomicAdd(&s_n, inc);
      int pos = __builtin_amdgcn_readlane(first, 63) + inc - mine;
      if (in_d) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float v[4] = {f[i].x, f[i].y, f[i].z, f[i].w};
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if ((in_d >> (4 * i + e)) & 1u) {
              if (pos < BIG_CAP) s_list[pos] = make_uint2(score_key(v[e]), (uint32_t)(base + (i * BIG_BLOCK + tid) * 4 + e));
              ++pos;
            }
        }
      }
    }
  }
  __syncthreads();
  const int n = min(s_n, BIG_CAP);

  // threshold key among the list: digits of 8, 8 and 4 bits below the 12 settled ones
  uint32_t low = 0;                 // settled bits below bit 20, right-aligned
  int remaining = s_r;
  if (kprime > 0) {
#pragma unroll
    for (int pass = 0; pass < 3; ++pass) {
      const int shift = pass == 0 ? 12 : (pass == 1 ? 4 : 0);
      const int width = pass == 2 ? 4 : 8;
      if (tid < 256) s_h[tid] = 0;
      __syncthreads();
      for (int i = tid; i < n; i += BIG_BLOCK) {
        const uint32_t k20 = s_list[i].x & 0xfffffu;
        if (pass == 0 || (k20 >> (shift + width)) == low) atomicAdd(&s_h[(k20 >> shift) & ((1u << width) - 1u)], 1);
      }
      __syncthreads();
      if (wave == 0) {
        int v4[4], loc = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) { v4[j] = s_h[255 - 4 * lane - j]; loc += v4[j]; }
        const int inc = spin_wave_inclusive_scan(loc);
        int run = inc - loc;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (run < remaining && run + v4[j] >= remaining) {
            s_digit = 255 - 4 * lane - j;
            s_remaining = remaining - run;
          }
          run += v4[j];
        }
      }
      __syncthreads();
      low = (low << width) | (uint32_t)s_digit;
      remaining = s_remaining;
    }
  }
  const uint32_t T = ((uint32_t)D << 20) | low;
  const unsigned need_eq = kprime > 0 ? (unsigned)remaining : 0u;
  for (int i = tid; i < n; i += BIG_BLOCK) {
    const uint2 e = s_list[i];
    if (e.x > T) atomicOr(&s_main[e.y >> 5], 1u << (e.y & 31));
    else if (e.x == T) atomicOr(&s_eq[e.y >> 5], 1u << (e.y & 31));
  }
  __syncthreads();

  // ordered emission: thread t owns the words [t * wpt, (t + 1) * wpt)
  const int wpt = (W + BIG_BLOCK - 1) / BIG_BLOCK;
  const int w0 = min(tid * wpt, W), w1 = min(w0 + wpt, W);
  unsigned long long mine = 0;
  for (int w = w0; w < w1; ++w) mine += (unsigned long long)__popc(s_main[w]) + ((unsigned long long)__popc(s_eq[w]) << 32);
  const unsigned long long inc = (unsigned long long)(uint32_t)spin_wave_inclusive_scan((int)(uint32_t)mine) |
                                 ((unsigned long long)(uint32_t)spin_wave_inclusive_scan((int)(mine >> 32)) << 32);
  if (lane == 63) s_wtot[wave] = inc;
  __syncthreads();
  unsigned long long before = inc - mine;
  for (int w = 0; w < wave; ++w) before += s_wtot[w];
  const unsigned main_before = (unsigned)(before & 0xffffffffull), eq_before = (unsigned)(before >> 32);
  unsigned eq_quota = need_eq > eq_before ? need_eq - eq_before : 0u;
  int pos = (int)(main_before + min(eq_before, need_eq));
  for (int w = w0; w < w1; ++w) {
    const uint32_t m = s_main[w], e = s_eq[w];
    uint32_t both = m | e;
    while (both) {
      const int bit = __ffs(both) - 1;
      both &= both - 1;
      bool pick = (m >> bit) & 1u;
      if (!pick && eq_quota > 0) { pick = true; --eq_quota; }
      if (pick && pos < sel_stride) rsel[pos++] = w * 32 + bit;
    }
  }
  for (int i = pl.take + tid; i < sel_stride; i += BIG_BLOCK) rsel[i] = -1;
  if (tid == 0) nsel[row] = pl.take;
  if (RESOLVE) {
    __syncthreads();
    resolve_row<BIG_BLOCK>(row, pl.take, sel, seq_lens, ra.dir, ra.leaf_pool, ra.leaf_chunks, Hkv, tp, sink_pages,
                           recent_pages, sel_stride, page_stride, dir_stride, leaf_entries, ra.slots, ra.page_ids,
                           ra.valid_mask, ra.npages, status, spin_var{});
  }
}

int spin_select_impl(spin_ctx *ctx, int32_t batch, const float *scores, const int32_t *part_offsets,
                     const int32_t *seq_lens, int32_t *sel, int32_t *nsel, void *workspace, void *stream,
                     bool hist_ready, const spin_resolve_args *res) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch) return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!scores || !part_offsets || !seq_lens || !sel || !nsel) return SPIN_ERR_INVALID;
  const spin_config &c = ctx->cfg;
  const int rows = batch * c.num_kv_heads;
  // stage 3 in the same launch exists for the long-row path below only
  if (res && !(ctx->max_parts > 16384 && ctx->ws_hist_off && workspace && rows <= 65535)) return SPIN_ERR_UNSUPPORTED;
#define SPIN_SELECT_ARGS                                                                                      \
  0, (hipStream_t)stream, scores, part_offsets, seq_lens, c.num_kv_heads, c.partition_tokens, c.topk,         \
      c.topk_includes_forced, c.sink_pages, c.recent_pages, ctx->sel_stride, sel, nsel
  if (ctx->max_parts <= 2048)
    spin_launch(ctx, SPIN_K_SELECT, spin_select_reg_kernel<512, 4>, dim3((unsigned)rows), dim3(512), SPIN_SELECT_ARGS, ctx->var);
  else if (ctx->max_parts <= 4096)
    spin_launch(ctx, SPIN_K_SELECT, spin_select_reg_kernel<512, 8>, dim3((unsigned)rows), dim3(512), SPIN_SELECT_ARGS, ctx->var);
  else if (ctx->max_parts <= 16384)
    spin_launch(ctx, SPIN_K_SELECT, spin_select_reg_kernel<1024, 16>, dim3((unsigned)rows), dim3(1024),
                SPIN_SELECT_ARGS, ctx->var);
  else if (ctx->ws_hist_off && workspace && rows <= 65535) {   // rows are the histogram grid's second dimension
    // two launches: histogram of the first 12 key bits by many workgroups per row, then one workgroup per row
    int32_t *hist = (int32_t *)((char *)workspace + ctx->ws_hist_off);
    const int words_max = ((ctx->max_parts + 63) / 64) * 2;
    const size_t lds = (size_t)words_max * 8 + (size_t)BIG_CAP * 8;
    // at most 56 KiB for rows of 131072 partitions; the kernel's static arrays (under 8 KiB) come on top
    if (lds + 8192 > 64 * 1024) return SPIN_ERR_UNSUPPORTED;
    if (!hist_ready)   // stage 1 may have counted the bins already while it produced the scores
      spin_launch(ctx, SPIN_K_SELECT_HIST, spin_select_hist_kernel,
                  dim3((unsigned)((ctx->max_parts + BIG_CHUNK - 1) / BIG_CHUNK), (unsigned)rows), dim3(256), 0,
                  (hipStream_t)stream, scores, part_offsets, seq_lens, c.num_kv_heads, c.partition_tokens, c.topk,
                  c.topk_includes_forced, c.sink_pages, c.recent_pages, ctx->sel_stride, hist);
#define SPIN_BIG_ARGS                                                                                         \
  dim3((unsigned)rows), dim3(BIG_BLOCK), lds, (hipStream_t)stream, scores, part_offsets, seq_lens, c.num_kv_heads, \
      c.partition_tokens, c.topk, c.topk_includes_forced, c.sink_pages, c.recent_pages, ctx->sel_stride, sel, nsel,  \
      hist, words_max
    if (res)
      spin_launch(ctx, SPIN_K_SELECT, spin_select_big_kernel<true>, SPIN_BIG_ARGS, *res, ctx->page_stride,
                  ctx->dir_stride, c.leaf_entries, (int32_t *)workspace);
    else
      spin_launch(ctx, SPIN_K_SELECT, spin_select_big_kernel<false>, SPIN_BIG_ARGS, spin_resolve_args{}, 0, 0, 0,
                  (int32_t *)nullptr);
#undef SPIN_BIG_ARGS
    return spin_launch_status();
  } else if (ctx->max_parts <= 65536)
    spin_launch(ctx, SPIN_K_SELECT, spin_select_reg_kernel<1024, 64>, dim3((unsigned)rows), dim3(1024),
                SPIN_SELECT_ARGS, ctx->var);
  else if (ctx->var.count)
    return SPIN_ERR_UNSUPPORTED;   // variable-length partitions: rows of at most 65536 partitions
  else
    spin_launch(ctx, SPIN_K_SELECT, spin_select_kernel, dim3((unsigned)rows), dim3(SEL_BLOCK), SPIN_SELECT_ARGS);
#undef SPIN_SELECT_ARGS
  return spin_launch_status();
}

extern "C" int spin_select_topk(spin_ctx *ctx, int32_t batch, const float *scores, const int32_t *part_offsets,
                                const int32_t *seq_lens, int32_t *sel, int32_t *nsel, void *workspace,
                                void *stream) {
  return spin_select_impl(ctx, batch, scores, part_offsets, seq_lens, sel, nsel, workspace, stream, false, nullptr);
}

// Stages 1 and 2 in one call.  Where stage 2 takes two launches and stage 1 can count the leading
// key bits of its scores as it produces them, the histogram launch is saved; otherwise the two
// stages are simply issued one after the other.  Same results as the two calls, bit for bit.
extern "C" int spin_score_select_topk(spin_ctx *ctx, int32_t batch, const void *q, const void *summaries,
                                      const int32_t *chan_idx, const int32_t *part_offsets,
                                      const int32_t *seq_lens, float *scores, int32_t *sel, int32_t *nsel,
                                      void *workspace, void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch) return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!sel || !nsel) return SPIN_ERR_INVALID;
  // (same condition as the two-launch path of stage 2: the histogram must be consumed by the launch that follows)
  const bool fuse = ctx->ws_hist_off && workspace && batch * ctx->cfg.num_kv_heads <= 65535;
  int32_t *hist = fuse ? (int32_t *)((char *)workspace + ctx->ws_hist_off) : nullptr;
  const int st = spin_score_impl(ctx, batch, q, summaries, chan_idx, part_offsets, seq_lens, scores, workspace, stream,
                                 hist);
  if (st != SPIN_OK) return st;
  return spin_select_impl(ctx, batch, scores, part_offsets, seq_lens, sel, nsel, workspace, stream, fuse, nullptr);
}
