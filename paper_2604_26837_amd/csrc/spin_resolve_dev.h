// Device code of stage 3 (all-resident mode) shared by the stand-alone kernel
// and the fused launch.
#pragma once
#include "spin_common.h"

template <int RES_BLOCK>
__device__ inline int res_block_exclusive_scan(int v, int *s_wave, int &total) {
  constexpr int RES_WAVES = RES_BLOCK / 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int inc = spin_wave_inclusive_scan(v);
  __syncthreads();
  if (lane == 63) s_wave[wave] = inc;
  __syncthreads();
  int off = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < RES_WAVES; ++w) {
    const int x = s_wave[w];
    if (w < wave) off += x;
    tot += x;
  }
  total = tot;
  return off + inc - v;
}

__device__ inline uint32_t page_mask(int page, int N) {
  const int n = min(max(N - page * 16, 0), 16);
  return (1u << n) - 1u;
}

struct res_out {
  int32_t *slots, *page_ids;
  uint16_t *mask;
};

__device__ inline void res_put(const res_out &o, int pos, int32_t slot, int32_t page, uint32_t mask) {
  o.slots[pos] = slot;
  o.page_ids[pos] = page;
  o.mask[pos] = (uint16_t)mask;
}

#define RES_DIR_LDS 256

// `dir` points at the row's directory entries (a copy in LDS when it fits)
// LOOKUP = false: only the page list and the masks are wanted (budget mode decides the slots)
template <bool LOOKUP>
__device__ inline void emit_page(const res_out &o, int pos, int page_stride, int page, uint32_t mask,
                                 const int32_t *dir, const int32_t *leaf_pool, int64_t leaf_chunks, int row,
                                 int dir_stride, int leaf_entries, int32_t *status) {
  if (pos < 0 || pos >= page_stride) return;
  (void)row;
  int32_t slot = -1;
  if (LOOKUP) {
    slot = spin_walk(dir, leaf_pool, leaf_chunks, 0, dir_stride, leaf_entries, page);
    if (slot < 0) {
      spin_raise(status, SPIN_ERR_NOT_RESIDENT);
      slot = -1;
      mask = 0;
    }
  }
  res_put(o, pos, slot, page, mask);
}

// A selection entry outside the row: its output position holds no page (nothing of a previous
// step stays there for stage 4 to attend) and the fault is reported.
__device__ inline void emit_invalid(const res_out &o, int pos, int page_stride, int32_t *status) {
  spin_raise(status, SPIN_ERR_INVALID);
  if (pos < 0 || pos >= page_stride) return;
  res_put(o, pos, -1, -1, 0);
}

// Resolves one row with the calling workgroup of RES_BLOCK threads; `ns` = the
// row's selection count.
template <int RES_BLOCK, bool LOOKUP = true>
__device__ inline void resolve_row(
    int row, int ns, const int32_t *__restrict__ sel, const int32_t *__restrict__ seq_lens,
    const int32_t *dir, const int32_t *__restrict__ leaf_pool, int64_t leaf_chunks, int Hkv, int tp,
    int sink_pages, int recent_pages, int sel_stride, int page_stride, int dir_stride, int leaf_entries,
    int32_t *__restrict__ slots, int32_t *__restrict__ page_ids, uint16_t *__restrict__ valid_mask,
    int32_t *__restrict__ npages, int32_t *status, spin_var var) {
  constexpr int RES_WAVES = RES_BLOCK / 64;
  __shared__ int s_wave[RES_WAVES];
  __shared__ int s_flagA, s_flagB, s_cntB;
  __shared__ int32_t s_dir[RES_DIR_LDS];
  const int tid = threadIdx.x;
  const int b = row / Hkv;
  // the row's directory entries are fetched together with its selection, so the
  // leaf lookups below are the only dependent round trip
  const int32_t *gdir = dir + (size_t)row * dir_stride;
  const bool dir_in_lds = dir_stride <= RES_DIR_LDS;
  if (dir_in_lds)
    for (int i = tid; i < dir_stride; i += RES_BLOCK) s_dir[i] = gdir[i];
  dir = dir_in_lds ? s_dir : gdir;
  const int N = seq_lens[b];
  const int pages = (N + 15) >> 4;
  ns = ns < 0 ? 0 : (ns > sel_stride ? sel_stride : ns);
  const int32_t *rsel = sel + (size_t)row * sel_stride;
  res_out o = {slots + (size_t)row * page_stride, page_ids + (size_t)row * page_stride,
               valid_mask + (size_t)row * page_stride};

  if (dir_in_lds) __syncthreads();

  if (var.count) {
    // Variable-length partitions: the page list of partition p starts at
    // first_page[p] and holds ceil(tokens[p]/16) pages (Partition Offset and
    // Meta-partition tables).  Output positions come from a prefix sum of the
    // selected partitions' page counts.
    __shared__ int s_sumA, s_sumB;
    const size_t vb = spin_var_base(var, row, Hkv);
    int P = var.count[row];
    const int cap = var.part_offsets[b + 1] - var.part_offsets[b];
    P = P < 0 ? 0 : (P > cap ? cap : P);
    const int vpages = spin_var_row_pages(var, vb, P);
    int sink_end = min(sink_pages, vpages);
    int recent_begin = max(vpages - recent_pages, 0);
    if (sink_end >= recent_begin) { sink_end = vpages; recent_begin = vpages; }
    int A = -1, B = -1, a0 = 0, a1 = 0, b0 = 0, b1 = 0;
    if (sink_end > 0) {
      const int pa = spin_var_lower_bound_start(var, vb, P, sink_end) - 1;   // last partition starting before sink_end
      if (pa >= 0 && var.first_page[vb + pa] + spin_var_npages(var, vb, pa) > sink_end) {
        A = pa; a0 = var.first_page[vb + pa]; a1 = sink_end;
      }
    }
    if (recent_begin < vpages) {
      const int pb = spin_var_lower_bound_start(var, vb, P, recent_begin + 1) - 1;   // partition holding recent_begin
      if (pb >= 0 && var.first_page[vb + pb] < recent_begin) {
        B = pb; b0 = recent_begin; b1 = var.first_page[vb + pb] + spin_var_npages(var, vb, pb);
      }
    }
    if (tid == 0) { s_flagA = 0; s_flagB = 0; s_sumA = 0; s_sumB = 0; }
    __syncthreads();
    for (int i = tid; i < ns; i += RES_BLOCK) {
      const int s = rsel[i];
      if (s < 0 || s >= P) { spin_raise(status, SPIN_ERR_INVALID); continue; }   // takes no output position
      const int n = spin_var_npages(var, vb, s);
      if (s == A) s_flagA = 1;
      if (s == B) s_flagB = 1;
      if (A >= 0 && s < A) atomicAdd(&s_sumA, n);
      if (B >= 0 && s < B) atomicAdd(&s_sumB, n);
    }
    __syncthreads();
    const int extraA = (A >= 0 && !s_flagA) ? (a1 - a0) : 0;
    const int extraB = (B >= 0 && !s_flagB) ? (b1 - b0) : 0;
    int carry = 0;
    for (int i0 = 0; i0 < ns; i0 += RES_BLOCK) {
      const int i = i0 + tid;
      int s = -1, n = 0;
      if (i < ns) {
        s = rsel[i];
        if (s >= 0 && s < P) n = spin_var_npages(var, vb, s); else s = -1;
      }
      int tot;
      const int before = res_block_exclusive_scan<RES_BLOCK>(n, s_wave, tot);
      if (s >= 0) {
        int pos = carry + before + ((extraA && s > A) ? extraA : 0) + ((extraB && s > B) ? extraB : 0);
        const int fp = var.first_page[vb + s], tk = var.tokens[vb + s];
        for (int k = 0; k < n; ++k) {
          const int nv = min(max(tk - 16 * k, 0), 16);
          emit_page<LOOKUP>(o, pos + k, page_stride, fp + k, (1u << nv) - 1u, dir, leaf_pool, leaf_chunks, row, dir_stride,
                    leaf_entries, status);
        }
      }
      carry += tot;
    }
    for (int k = tid; k < extraA; k += RES_BLOCK) {
      const int nv = min(max(var.tokens[vb + A] - 16 * (a0 + k - var.first_page[vb + A]), 0), 16);
      emit_page<LOOKUP>(o, s_sumA + k, page_stride, a0 + k, (1u << nv) - 1u, dir, leaf_pool, leaf_chunks, row, dir_stride,
                leaf_entries, status);
    }
    for (int k = tid; k < extraB; k += RES_BLOCK) {
      const int nv = min(max(var.tokens[vb + B] - 16 * (b0 + k - var.first_page[vb + B]), 0), 16);
      emit_page<LOOKUP>(o, s_sumB + ((A >= 0 && A <= B) ? extraA : 0) + k, page_stride, b0 + k, (1u << nv) - 1u, dir, leaf_pool,
                leaf_chunks, row, dir_stride, leaf_entries, status);
    }
    const int total = min(carry + extraA + extraB, page_stride);
    for (int i = total + tid; i < page_stride; i += RES_BLOCK) res_put(o, i, -1, -1, 0);
    if (tid == 0) npages[row] = total;
  } else if (tp == 16) {
    // partition == page: the selection is the page list.  The entry is loaded
    // before the row's counts are known (the buffer is sel_stride wide), so the
    // leaf lookup is the only dependent round trip.
    for (int i0 = 0; i0 < sel_stride; i0 += RES_BLOCK) {
      const int i = i0 + tid;
      const int s = i < sel_stride ? rsel[i] : -1;
      if (i < ns) {
        if (s >= 0 && s < pages)
          emit_page<LOOKUP>(o, i, page_stride, s, page_mask(s, N), dir, leaf_pool, leaf_chunks, row, dir_stride,
                            leaf_entries, status);
        else
          emit_invalid(o, i, page_stride, status);   // an entry that names no page of the row
      }
      if (i0 + RES_BLOCK >= ns) break;
    }
    const int total = min(ns, page_stride);
    for (int i = total + tid; i < page_stride; i += RES_BLOCK) res_put(o, i, -1, -1, 0);
    if (tid == 0) npages[row] = total;
  } else if (tp > 16) {
    const int m = tp >> 4;
    int sink_end = min(sink_pages, pages);
    int recent_begin = max(pages - recent_pages, 0);
    if (sink_end >= recent_begin) { sink_end = pages; recent_begin = pages; }
    // partition partly covered by the sink pages / by the recent pages (or -1)
    int A = -1, B = -1, a0 = 0, a1 = 0, b0 = 0, b1 = 0;
    if (m > 1 && sink_end > 0) {
      const int pa = (sink_end - 1) / m;
      if (min((pa + 1) * m, pages) > sink_end) { A = pa; a0 = pa * m; a1 = sink_end; }
    }
    if (m > 1 && recent_begin < pages) {
      const int pb = recent_begin / m;
      if (pb * m < recent_begin) { B = pb; b0 = recent_begin; b1 = min((pb + 1) * m, pages); }
    }
    if (tid == 0) { s_flagA = 0; s_flagB = 0; s_cntB = 0; }
    __syncthreads();
    int below_b = 0;
    for (int i = tid; i < ns; i += RES_BLOCK) {
      const int s = rsel[i];
      if (s == A) s_flagA = 1;
      if (s == B) s_flagB = 1;
      below_b += (B >= 0 && s < B);
    }
    if (B >= 0 && below_b) atomicAdd(&s_cntB, below_b);
    __syncthreads();
    const int extraA = (A >= 0 && !s_flagA) ? (a1 - a0) : 0;   // standalone sink pages
    const int extraB = (B >= 0 && !s_flagB) ? (b1 - b0) : 0;   // standalone recent pages
    const int sel_below_b = s_cntB;
    // pages of the selected partitions
    for (int idx = tid; idx < ns * m; idx += RES_BLOCK) {
      const int i = idx / m, k = idx - i * m;
      const int s = rsel[i];
      const int pg = s * m + k;
      int pos = i * m + k;
      if (extraA && s > A) pos += extraA;
      if (extraB && s > B) pos += extraB;
      if (s < 0 || (int64_t)s * m >= pages) {        // an entry that names no partition of the row
        emit_invalid(o, pos, page_stride, status);
        continue;
      }
      if (pg >= pages) continue;                     // the ragged end of the context's last partition
      emit_page<LOOKUP>(o, pos, page_stride, pg, page_mask(pg, N), dir, leaf_pool, leaf_chunks, row, dir_stride,
                leaf_entries, status);
    }
    // standalone forced pages: partitions 0..A-1 are wholly forced, hence selected
    for (int k = tid; k < extraA; k += RES_BLOCK)
      emit_page<LOOKUP>(o, A * m + k, page_stride, a0 + k, page_mask(a0 + k, N), dir, leaf_pool, leaf_chunks, row,
                dir_stride, leaf_entries, status);
    for (int k = tid; k < extraB; k += RES_BLOCK)
      emit_page<LOOKUP>(o, sel_below_b * m + ((A >= 0 && A <= B) ? extraA : 0) + k, page_stride, b0 + k,
                page_mask(b0 + k, N), dir, leaf_pool, leaf_chunks, row, dir_stride, leaf_entries, status);
    // total: only the context's last partition can be short
    int total = ns * m + extraA + extraB;
    if (ns > 0) {
      const int last = rsel[ns - 1];
      total -= max((last + 1) * m - pages, 0);
    }
    total = min(total, page_stride);
    for (int i = total + tid; i < page_stride; i += RES_BLOCK) res_put(o, i, -1, -1, 0);
    if (tid == 0) npages[row] = total;
  } else {
    const int ppp = 16 / tp;   // partitions per page
    int carry = 0;
    for (int i0 = 0; i0 < ns; i0 += RES_BLOCK) {
      const int i = i0 + tid;
      int first = 0, pg = -1;
      if (i < ns) {
        pg = rsel[i] / ppp;
        first = (i == 0) || (rsel[i - 1] / ppp != pg);
      }
      int tot;
      const int before = res_block_exclusive_scan<RES_BLOCK>(first, s_wave, tot);
      if (first) {
        uint32_t mk = 0;
        for (int j = i; j < ns && j < i + ppp; ++j) {
          const int s = rsel[j];
          if (s / ppp != pg) break;
          const int t0 = s * tp, cnt = min(tp, N - t0);
          if (s < 0 || cnt <= 0) { spin_raise(status, SPIN_ERR_INVALID); continue; }   // names no token of the row
          mk |= ((1u << cnt) - 1u) << (t0 & 15);
        }
        emit_page<LOOKUP>(o, carry + before, page_stride, pg, mk, dir, leaf_pool, leaf_chunks, row, dir_stride,
                  leaf_entries, status);
      }
      carry += tot;
    }
    const int total = min(carry, page_stride);
    for (int i = total + tid; i < page_stride; i += RES_BLOCK) res_put(o, i, -1, -1, 0);
    if (tid == 0) npages[row] = total;
  }
}

