// Device code of stage 2 (register-resident variant) shared by the stand-alone
// kernel and the fused launch.
#pragma once
#include "spin_common.h"

struct sel_plan {
  int P, nf_lo, first_hi, kprime, take;
};

// forced prefix / suffix and k' of a row of uniform partitions (same rules as select_reg_row)
__device__ inline sel_plan select_plan(int N, int PP, int tp, int topk, int includes_forced, int sink_pages,
                                       int recent_pages, int sel_stride) {
  sel_plan pl;
  int P = N > 0 ? (N + tp - 1) / tp : 0;
  if (P > PP) P = PP;
  const int pages = (N + 15) >> 4;
  int sink_end = min(sink_pages, pages);
  int recent_begin = max(pages - recent_pages, 0);
  if (sink_end >= recent_begin) { sink_end = pages; recent_begin = pages; }
  int nf_lo = (N <= sink_end * 16) ? P : min((sink_end * 16) / tp, P);
  int first_hi = min((recent_begin * 16 + tp - 1) / tp, P);
  if (first_hi <= nf_lo) { nf_lo = P; first_hi = P; }
  const int nforced = nf_lo + (P - first_hi);
  int kprime = includes_forced ? max(topk - nforced, 0) : topk;
  kprime = min(kprime, P - nforced);
  int take = nforced + kprime;
  if (take > sel_stride) {
    kprime = max(sel_stride - nforced, 0);
    take = min(nforced + kprime, sel_stride);
  }
  pl.P = P; pl.nf_lo = nf_lo; pl.first_hi = first_hi; pl.kprime = kprime; pl.take = take;
  return pl;
}

// Register-resident variant for rows of at most BLOCK * KPT partitions: every
// thread keeps KPT consecutive keys in registers, so scores are read once; each
// digit has its own LDS histogram, every wavefront does the 256-bin suffix scan
// for itself (one barrier per digit), and the two compaction prefix sums share
// one scan.
// Returns the number of selected partitions.
template <int BLOCK, int KPT>
__device__ inline int select_reg_row(
    const float *__restrict__ scores, const int32_t *__restrict__ part_offsets,
    const int32_t *__restrict__ seq_lens, int Hkv, int tp, int topk, int includes_forced, int sink_pages,
    int recent_pages, int sel_stride, int32_t *__restrict__ sel, int32_t *__restrict__ nsel, int row,
    spin_var var) {
  constexpr int NW = BLOCK / 64;
  __shared__ int s_hist[4][256];   // one histogram per digit: no buffer is cleared while others read it
  __shared__ unsigned long long s_wtot[NW];

  const int b = row / Hkv, h = row - b * Hkv;
  const int N = seq_lens[b];
  const int off_b = part_offsets[b];
  const int PP = part_offsets[b + 1] - off_b;
  const float *rs = scores + (size_t)Hkv * off_b + (size_t)h * PP;
  int32_t *rsel = sel + (size_t)row * sel_stride;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const size_t vbase = (size_t)Hkv * off_b + (size_t)h * PP;
  int P = var.count ? var.count[row] : (N > 0 ? (N + tp - 1) / tp : 0);
  if (P < 0) P = 0;
  if (P > PP) P = PP;
  if (P > BLOCK * KPT) P = BLOCK * KPT;   // the host picks a variant that fits; keep indexing in range

  // keys of partitions c0 .. c0+KPT-1
  const int c0 = tid * KPT;
  uint32_t key[KPT];
#pragma unroll
  for (int k4 = 0; k4 < KPT; k4 += 4) {
    float4 f = make_float4(0.f, 0.f, 0.f, 0.f);
    if (c0 + k4 < PP) f = *(const float4 *)(rs + c0 + k4);
    key[k4] = score_key(f.x); key[k4 + 1] = score_key(f.y); key[k4 + 2] = score_key(f.z); key[k4 + 3] = score_key(f.w);
  }

  // forced partitions: a prefix [0, nf_lo) and a suffix [first_hi, P)
  const int pages = var.count ? spin_var_row_pages(var, vbase, P) : ((N + 15) >> 4);
  int sink_end = min(sink_pages, pages);
  int recent_begin = max(pages - recent_pages, 0);
  if (sink_end >= recent_begin) { sink_end = pages; recent_begin = pages; }
  int nf_lo, first_hi;
  if (var.count) {
    nf_lo = spin_var_count_end_le(var, vbase, P, sink_end);
    first_hi = spin_var_lower_bound_start(var, vbase, P, recent_begin);
  } else {
    nf_lo = (N <= sink_end * 16) ? P : min((sink_end * 16) / tp, P);
    first_hi = min((recent_begin * 16 + tp - 1) / tp, P);
  }
  if (first_hi <= nf_lo) { nf_lo = P; first_hi = P; }
  const int nforced = nf_lo + (P - first_hi);
  const int ncand = P - nforced;
  int kprime = includes_forced ? max(topk - nforced, 0) : topk;
  kprime = min(kprime, ncand);
  int take = nforced + kprime;
  if (take > sel_stride) {
    kprime = max(sel_stride - nforced, 0);
    take = min(nforced + kprime, sel_stride);
  }
  // candidates of this thread form the index range [ca, cb)
  const int ca = max(c0, nf_lo), cb = min(c0 + KPT, first_hi);

  uint32_t prefix = 0;
  int remaining = kprime;
  // Radix select of the k'-th largest candidate key, most significant digit first.  The digits
  // start at the highest bit in which the row's candidate keys differ at all (one min/max
  // reduction): scores of one row usually share sign, exponent and leading mantissa bits, so
  // this saves a pass or two and, above all, spreads the first histogram over many bins
  // instead of piling every key onto one LDS counter.
  // Rows with many keys per thread: for the first digit every thread counts, in one packed
  // register, its keys in the 8 highest digit values at or below the row's largest one; the full
  // histogram is only built when the k'-th candidate lies below them.
  constexpr bool TOP8 = KPT >= 16 && KPT <= 255;
  __shared__ uint32_t s_wmax[NW], s_wmin[NW];
  if (kprime > 0) {
    for (int i = tid; i < 4 * 256; i += BLOCK) (&s_hist[0][0])[i] = 0;
    uint32_t kmx = 0u, kmn = 0xffffffffu;
#pragma unroll
    for (int k = 0; k < KPT; ++k) {
      const int p = c0 + k;
      if (p >= ca && p < cb) { kmx = max(kmx, key[k]); kmn = min(kmn, key[k]); }
    }
    kmx = spin_wave_max_u32(kmx);
    kmn = spin_wave_min_u32(kmn);
    if (lane == 0) { s_wmax[wave] = kmx; s_wmin[wave] = kmn; }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < NW; ++w) { kmx = max(kmx, s_wmax[w]); kmn = min(kmn, s_wmin[w]); }
    int hi = kmx == kmn ? 0 : 32 - __clz((int)(kmx ^ kmn));   // the low `hi` bits are the ones that vary
    prefix = hi < 32 ? kmx >> hi : 0u;
    // Suffix scan of the 256-bin histogram `buf`, done by every wavefront for itself: digit of the
    // remaining-th largest candidate (and how many are still wanted inside it), or -1 when the
    // histogram holds fewer.  The result is uniform over the workgroup.
    auto find_digit = [&](int buf, int &digit, int &in_digit) {
      __syncthreads();
      // lane handles digits 255-4*lane .. 252-4*lane, in descending order
      int hv[4], local = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) { hv[j] = s_hist[buf][255 - 4 * lane - j]; local += hv[j]; }
      int running = spin_wave_inclusive_scan(local) - local;
      int my_digit = -1, my_rem = 0, my_cnt = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (running < remaining && running + hv[j] >= remaining) {
          my_digit = 255 - 4 * lane - j;
          my_rem = remaining - running;
          my_cnt = hv[j];
        }
        running += hv[j];
      }
      const unsigned long long found = __ballot(my_digit >= 0);
      digit = -1;
      in_digit = 0;
      if (found) {
        const int src = __ffsll((long long)found) - 1;
        digit = __builtin_amdgcn_readlane(my_digit, src);
        remaining = __builtin_amdgcn_readlane(my_rem, src);
        in_digit = __builtin_amdgcn_readlane(my_cnt, src);
      }
    };
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
      if (hi <= 0) break;                                  // block-uniform
      const int lo = max(hi - 8, 0), width = hi - lo;
      const uint32_t dmask = (1u << width) - 1u;
      const uint32_t top_digit = (kmx >> lo) & dmask;      // pass 0: the largest digit present
      if (TOP8 && pass == 0) {
        unsigned long long acc = 0;                  // 8 counters of 8 bits: digit top_digit - j in byte j
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
          const int p = c0 + k;
          const uint32_t o = top_digit - ((key[k] >> lo) & dmask);
          if (p >= ca && p < cb && o < 8u) acc += 1ull << (8u * o);
        }
        // widen to 16-bit fields (a wavefront holds at most 64 * 255 keys of one digit) and add up
        unsigned long long even = acc & 0x00ff00ff00ff00ffull, odd = (acc >> 8) & 0x00ff00ff00ff00ffull;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
          even += __shfl_xor(even, d);
          odd += __shfl_xor(odd, d);
        }
        if (lane < 8) {
          const unsigned long long v = (lane & 1) ? odd : even;
          const int c = (int)((v >> (16 * (lane >> 1))) & 0xffffull);
          if (c && (uint32_t)lane <= top_digit) atomicAdd(&s_hist[0][top_digit - lane], c);
        }
      } else {
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
          const int p = c0 + k;
          if (p >= ca && p < cb && (pass == 0 || (key[k] >> hi) == prefix))
            atomicAdd(&s_hist[pass][(key[k] >> lo) & dmask], 1);
        }
      }
      int digit, in_digit;
      find_digit(pass, digit, in_digit);
      if (TOP8 && pass == 0 && digit < 0) {          // block-uniform: add the digits not counted yet
        __syncthreads();                             // every wavefront has scanned the partial histogram
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
          const int p = c0 + k;
          const uint32_t dg = (key[k] >> lo) & dmask;
          if (p >= ca && p < cb && top_digit - dg >= 8u) atomicAdd(&s_hist[0][dg], 1);
        }
        find_digit(0, digit, in_digit);
      }
      prefix = (prefix << width) | (uint32_t)digit;
      hi = lo;
      // every candidate that shares this prefix is wanted: the digits below cannot change the outcome.  The
      // threshold becomes the smallest key with the prefix, of which there may be several or none: all are
      // wanted, and `remaining` (the candidates with the prefix) covers them.
      if (in_digit == remaining && hi > 0) {         // block-uniform
        prefix <<= hi;
        break;
      }
    }
  }
  const uint32_t T = prefix;
  // (after the early exit above, keys above T that share the prefix are picked as `key > T` and keys equal to T
  // within the quota, which is as large as the whole prefix: the same set either way)
  const unsigned need_eq = kprime > 0 ? (unsigned)remaining : 0u;

  // counts of this thread: low half = forced or above threshold, high half = equal to it
  unsigned long long mine = 0;
#pragma unroll
  for (int k = 0; k < KPT; ++k) {
    const int p = c0 + k;
    if (p >= P) continue;
    if (p < nf_lo || p >= first_hi) { mine += 1ull; continue; }
    if (kprime == 0) continue;
    mine += (key[k] > T) ? 1ull : 0ull;
    mine += (key[k] == T) ? (1ull << 32) : 0ull;
  }
  // the two counts never carry into one another: scan the halves separately
  const unsigned long long inc = (unsigned long long)(uint32_t)spin_wave_inclusive_scan((int)(uint32_t)mine) |
                                 ((unsigned long long)(uint32_t)spin_wave_inclusive_scan((int)(mine >> 32)) << 32);
  if (lane == 63) s_wtot[wave] = inc;
  __syncthreads();
  unsigned long long before = inc - mine;
#pragma unroll
  for (int w = 0; w < NW; ++w)
    if (w < wave) before += s_wtot[w];
  const unsigned gt_before = (unsigned)(before & 0xffffffffull), eq_before = (unsigned)(before >> 32);
  unsigned eq_quota = need_eq > eq_before ? need_eq - eq_before : 0u;
  int pos = (int)(gt_before + min(eq_before, need_eq));
#pragma unroll
  for (int k = 0; k < KPT; ++k) {
    const int p = c0 + k;
    if (p >= P) continue;
    bool pick;
    if (p < nf_lo || p >= first_hi) pick = true;
    else if (kprime == 0) pick = false;
    else {
      pick = key[k] > T;
      if (key[k] == T && eq_quota > 0) { pick = true; --eq_quota; }
    }
    if (pick && pos < sel_stride) rsel[pos++] = p;
  }
  for (int i = take + tid; i < sel_stride; i += BLOCK) rsel[i] = -1;
  if (tid == 0) nsel[row] = take;
  return take;
}

