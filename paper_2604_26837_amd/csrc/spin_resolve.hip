// Stage 3: selected partitions -> logical pages -> HBM slots through the
// two-level table (Section 5.2, Retrieve steps 1-2; Section 5.4).
//
// One workgroup per row.  Partitions of at least a page expand to their
// consecutive pages; forced pages lying in a partition that was not selected
// (possible only when a partition spans several pages) are merged in at their
// ascending position, computed in closed form.  Partitions smaller than a page
// collapse onto pages with a token mask: the first entry of each run of equal
// pages owns the output entry and ORs the run's token ranges.
#include "spin_resolve_dev.h"

template <int RES_BLOCK>
__global__ __launch_bounds__(RES_BLOCK) void spin_resolve_kernel(
    const int32_t *__restrict__ sel, const int32_t *__restrict__ nsel, const int32_t *__restrict__ seq_lens,
    const int32_t *dir, const int32_t *__restrict__ leaf_pool, int64_t leaf_chunks, int Hkv, int tp,
    int sink_pages, int recent_pages, int sel_stride, int page_stride, int dir_stride, int leaf_entries,
    int32_t *__restrict__ slots, int32_t *__restrict__ page_ids, uint16_t *__restrict__ valid_mask,
    int32_t *__restrict__ npages, int32_t *status, spin_var var) {
  const int row = blockIdx.x;
  resolve_row<RES_BLOCK>(row, nsel[row], sel, seq_lens, dir, leaf_pool, leaf_chunks, Hkv, tp, sink_pages, recent_pages,
                         sel_stride, page_stride, dir_stride, leaf_entries, slots, page_ids, valid_mask, npages, status,
                         var);
}

// ---------------------------------------------------------------------------
// Budget mode: bucketed-LRU replacement (Section 5.3), page partitions.
//
// One workgroup per row.  The row owns the S = slot_range[row][1] pool slots
// starting at slot_range[row][0]; rev_table[slot] = {resident logical page or -1, timestamp}; the leaf
// entries are the forward map page -> slot.  The four steps run in the paper's
// order: (1) classify the selected pages by a leaf lookup, (2)+(3) one scan of
// the row's slots updates timestamps and builds the per-timestamp histogram in
// LDS, a single wavefront finds the smallest threshold x whose cumulative
// count covers the net demand, and the pages at or below x are evicted,
// (4) the misses (ascending page id) take the free slots (ascending slot id),
// found with one prefix sum over the slots.
#define LRU_BLOCK 512
#define LRU_WAVES (LRU_BLOCK / 64)
#define LRU_MAX_TS 256
#define LRU_LDS_LIMIT (64 * 1024)   // LDS a workgroup may use without raising the kernel's limit
#define LRU_LDS_STATIC 4096         // reserve for the static arrays of the budget-mode kernels

__device__ inline int lru_scan(int v, int *s_wave, int &total) {   // exclusive prefix sum over the workgroup
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int inc = spin_wave_inclusive_scan(v);
  __syncthreads();
  if (lane == 63) s_wave[wave] = inc;
  __syncthreads();
  int off = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < LRU_WAVES; ++w) {
    const int x = s_wave[w];
    if (w < wave) off += x;
    tot += x;
  }
  total = tot;
  return off + inc - v;
}

// Partitions other than one page each (blocks, tokens, variable-length): the replacement policies
// work on pages, so the workgroup first expands the row's selection to its ascending page list
// with masks -- stage 3's own code, without the slot lookup -- and then runs the policy on that
// list (EXPAND).
struct lru_expand {
  int tp, sink_pages, recent_pages;
  spin_var var;
};

// the page list of the row as the policy's input; returns its length
template <bool EXPAND>
__device__ inline int lru_input(int row, const int32_t *__restrict__ sel, const int32_t *__restrict__ nsel,
                                const int32_t *__restrict__ seq_lens, const int32_t *dir, const int32_t *leaf_pool,
                                int64_t leaf_chunks, int Hkv, int sel_stride, int page_stride, int dir_stride,
                                int leaf_entries, int32_t *slots, int32_t *page_ids, uint16_t *valid_mask,
                                int32_t *npages, int32_t *status, const lru_expand &ex, const int32_t *&list) {
  if (!EXPAND) {
    list = sel + (size_t)row * sel_stride;
    return nsel[row];
  }
  resolve_row<LRU_BLOCK, false>(row, nsel[row], sel, seq_lens, dir, leaf_pool, leaf_chunks, Hkv, ex.tp, ex.sink_pages,
                                ex.recent_pages, sel_stride, page_stride, dir_stride, leaf_entries, slots, page_ids,
                                valid_mask, npages, status, ex.var);
  __syncthreads();   // the list was written by this workgroup: visible to all its threads from here
  list = page_ids + (size_t)row * page_stride;
  return npages[row];
}

// pages of the row's context (bound of a valid page id)
__device__ inline int lru_row_pages(const lru_expand &ex, int row, int Hkv, int N) {
  if (!ex.var.count) return (N + 15) >> 4;
  const size_t vb = spin_var_base(ex.var, row, Hkv);
  const int b = row / Hkv;
  const int cap = ex.var.part_offsets[b + 1] - ex.var.part_offsets[b];
  int P = ex.var.count[row];
  P = P < 0 ? 0 : (P > cap ? cap : P);
  return spin_var_row_pages(ex.var, vb, P);
}

template <bool EXPAND>
__global__ __launch_bounds__(LRU_BLOCK) void spin_resolve_lru_kernel(
    const int32_t *__restrict__ sel, const int32_t *__restrict__ nsel, const int32_t *__restrict__ seq_lens,
    const int32_t *__restrict__ dir, int32_t *leaf_pool, int64_t leaf_chunks, int32_t *rev,
    const int32_t *__restrict__ slot_base, int Hkv, int sel_stride, int page_stride, int dir_stride,
    int leaf_entries, int step_arg, int n_ts, int evict_exact, int max_slots_lds, int32_t *slots,
    int32_t *page_ids, uint16_t *valid_mask, int32_t *npages,
    int32_t *__restrict__ miss_pages, int32_t *__restrict__ miss_slots, int32_t *__restrict__ nmiss,
    int32_t *status, lru_expand ex) {
  extern __shared__ int32_t lds[];
  // a negative step asks for the workspace's own step counter (word 1 of its header): a captured
  // launch then follows the counter from replay to replay
  const int step = step_arg >= 0 ? step_arg : max(status[1], 0);
  int32_t *s_loc = lds;                                  // [page_stride]  leaf entry address (as chunk*LE+idx) per selected page
  int32_t *s_free = lds + page_stride;                   // [page_stride]  free slot (local) by rank
  uint8_t *s_flag = (uint8_t *)(lds + 2 * page_stride);  // [S] 1 = holds a selected page
  __shared__ int s_hist[LRU_MAX_TS];
  __shared__ int s_wave[LRU_WAVES];
  __shared__ int s_x, s_need_x, s_err;

  const int row = blockIdx.x, tid = threadIdx.x;
  const int b = row / Hkv;
  const int N = seq_lens[b];
  const int pages = lru_row_pages(ex, row, Hkv, N);
  const int32_t *rsel;
  int ns = lru_input<EXPAND>(row, sel, nsel, seq_lens, dir, leaf_pool, leaf_chunks, Hkv, sel_stride, page_stride,
                             dir_stride, leaf_entries, slots, page_ids, valid_mask, npages, status, ex, rsel);
  ns = ns < 0 ? 0 : ((!EXPAND && ns > sel_stride) ? sel_stride : ns);
  if (ns > page_stride) ns = page_stride;
  int32_t *o_slots = slots + (size_t)row * page_stride;
  int32_t *o_pages = page_ids + (size_t)row * page_stride;
  uint16_t *o_mask = valid_mask + (size_t)row * page_stride;
  int32_t *o_mpages = miss_pages + (size_t)row * page_stride;
  int32_t *o_mslots = miss_slots + (size_t)row * page_stride;
  const int sb = slot_base[2 * row];
  const int S = slot_base[2 * row + 1];
  const int32_t *gdir = dir + (size_t)row * dir_stride;

  if (tid == 0) s_err = 0;
  for (int i = tid; i < n_ts; i += LRU_BLOCK) s_hist[i] = 0;
  for (int j = tid; j < S && j < max_slots_lds; j += LRU_BLOCK) s_flag[j] = 0;
  __syncthreads();
  if (ns > S || S > max_slots_lds || S < 0) {
    if (tid == 0) { spin_raise(status, SPIN_ERR_BUDGET); npages[row] = 0; nmiss[row] = 0; }
    for (int i = tid; i < page_stride; i += LRU_BLOCK) { o_slots[i] = -1; o_pages[i] = -1; o_mask[i] = 0; }
    return;
  }
  const int ts_star = min(step, n_ts - 1);

  // (1) classification: hit when the leaf holds a slot of this row
  int my_miss = 0;
  for (int i = tid; i < ns; i += LRU_BLOCK) {
    const int pg = rsel[i];
    int loc = -1, slot = -1;
    if (pg >= 0 && pg < pages) {
      const int ci = pg / leaf_entries;
      const int32_t chunk = ci < dir_stride ? gdir[ci] : -1;
      if (chunk >= 0 && (int64_t)chunk < leaf_chunks) {
        loc = chunk * leaf_entries + (pg - ci * leaf_entries);
        slot = leaf_pool[loc];
      }
    }
    if (loc < 0) s_err = 1;                       // no leaf for a selected page
    if (slot >= sb && slot < sb + S) s_flag[slot - sb] = 1;
    else slot = -1;
    s_loc[i] = loc;
    o_slots[i] = slot;                            // hits are final, misses are filled in step (4)
    if (!EXPAND) {                                // (the expanded list already holds ids and masks)
      o_pages[i] = pg;
      o_mask[i] = (uint16_t)page_mask(pg, N);
    }
  }
  __syncthreads();
  if (s_err) {
    if (tid == 0) { spin_raise(status, SPIN_ERR_NOT_RESIDENT); npages[row] = 0; nmiss[row] = 0; }
    for (int i = tid; i < page_stride; i += LRU_BLOCK) { o_slots[i] = -1; o_pages[i] = -1; o_mask[i] = 0; }
    return;
  }

  // (2)+(3a) one scan over the row's slots: timestamps, histogram of evictable pages, empty count
  const int chunk = (S + LRU_BLOCK - 1) / LRU_BLOCK;
  const int j0 = min(tid * chunk, S), j1 = min(j0 + chunk, S);
  int my_free = 0;
  for (int j = j0; j < j1; ++j) {
    int2 e = *(const int2 *)(rev + 2 * (size_t)(sb + j));
    if (e.x < 0) { ++my_free; continue; }
    int ts = e.y;
    if (s_flag[j]) ts = ts_star;
    else {
      if (step > n_ts - 1) ts = max(ts - 1, 0);
      ts = min(max(ts, 0), n_ts - 1);
      atomicAdd(&s_hist[ts], 1);
    }
    if (ts != e.y) rev[2 * (size_t)(sb + j) + 1] = ts;
  }
  // miss ranks in page order (index order of the ascending selection)
  for (int i = tid; i < ns; i += LRU_BLOCK) my_miss += (o_slots[i] < 0);
  int demand, nfree;
  // ranks need the misses of lower indices: selection entries are dealt round-robin
  // above, so rank them with a second, contiguous pass
  (void)lru_scan(my_miss, s_wave, demand);
  (void)lru_scan(my_free, s_wave, nfree);
  const int net = max(0, demand - nfree);

  // (3b) threshold search, oldest bucket first
  if (tid == 0) { s_x = -1; s_need_x = 0; }
  __syncthreads();
  if (net > 0 && tid < 64) {
    // each lane owns a contiguous run of buckets
    const int per = (n_ts + 63) / 64;
    const int t0 = min(tid * per, n_ts), t1 = min(t0 + per, n_ts);
    int local = 0;
    for (int t = t0; t < t1; ++t) local += s_hist[t];
    const int inc = spin_wave_inclusive_scan(local);
    int running = inc - local;
    for (int t = t0; t < t1; ++t) {
      if (running < net && running + s_hist[t] >= net) { s_x = t; s_need_x = net - running; }
      running += s_hist[t];
    }
  }
  __syncthreads();
  const int x = s_x;
  if (net > 0 && x < 0) {   // cannot happen when ns <= S; keep the state untouched
    if (tid == 0) { spin_raise(status, SPIN_ERR_BUDGET); npages[row] = 0; nmiss[row] = 0; }
    return;
  }

  // (3c) eviction and free-slot ranking in one pass over the slots
  int my_eq = 0;
  if (net > 0 && evict_exact)
    for (int j = j0; j < j1; ++j) {
      const int2 e = *(const int2 *)(rev + 2 * (size_t)(sb + j));
      my_eq += (e.x >= 0 && !s_flag[j] && e.y == x);
    }
  int tot_eq = 0, eq_before = 0;
  if (evict_exact) eq_before = lru_scan(my_eq, s_wave, tot_eq);   // uniform branch: evict_exact is a kernel argument
  int eq_quota = max(min(s_need_x - eq_before, my_eq), 0);
  int my_newfree = 0;
  for (int j = j0; j < j1; ++j) {
    const int2 e = *(const int2 *)(rev + 2 * (size_t)(sb + j));
    bool is_free = e.x < 0;
    if (!is_free && net > 0 && !s_flag[j]) {
      bool ev = e.y < x || (e.y == x && !evict_exact);
      if (e.y == x && evict_exact && eq_quota > 0) { ev = true; --eq_quota; }
      if (ev) {
        // clear the forward entry of the evicted page and the slot
        const int pg = e.x, ci = pg / leaf_entries;
        const int32_t ch = ci < dir_stride ? gdir[ci] : -1;
        if (ch >= 0 && (int64_t)ch < leaf_chunks) leaf_pool[(size_t)ch * leaf_entries + (pg - ci * leaf_entries)] = -1;
        *(int2 *)(rev + 2 * (size_t)(sb + j)) = make_int2(-1, 0);
        is_free = true;
      }
    }
    my_newfree += is_free;
  }
  int tot_free;
  int frank = lru_scan(my_newfree, s_wave, tot_free);
  for (int j = j0; j < j1; ++j) {
    const int2 e = *(const int2 *)(rev + 2 * (size_t)(sb + j));
    if (e.x < 0) {
      if (frank < page_stride) s_free[frank] = j;
      ++frank;
    }
  }
  __syncthreads();

  // (4) admission: misses in ascending page order take free slots in ascending slot order
  const int pchunk = (ns + LRU_BLOCK - 1) / LRU_BLOCK;
  const int i0 = min(tid * pchunk, ns), i1 = min(i0 + pchunk, ns);
  int cnt = 0;
  for (int i = i0; i < i1; ++i) cnt += (o_slots[i] < 0);
  int tot_miss;
  int mrank = lru_scan(cnt, s_wave, tot_miss);
  for (int i = i0; i < i1; ++i) {
    if (o_slots[i] >= 0) continue;
    if (mrank >= tot_free || mrank >= page_stride) {   // cannot happen when ns <= S; never index past the free list
      spin_raise(status, SPIN_ERR_BUDGET);
      o_mask[i] = 0;
      ++mrank;
      continue;
    }
    const int j = s_free[mrank];
    const int pg = o_pages[i];
    *(int2 *)(rev + 2 * (size_t)(sb + j)) = make_int2(pg, ts_star);
    leaf_pool[s_loc[i]] = sb + j;
    o_slots[i] = sb + j;
    o_mpages[mrank] = pg;
    o_mslots[mrank] = sb + j;
    ++mrank;
  }
  for (int i = ns + tid; i < page_stride; i += LRU_BLOCK) { o_slots[i] = -1; o_pages[i] = -1; o_mask[i] = 0; }
  for (int i = tot_miss + tid; i < page_stride; i += LRU_BLOCK) { o_mpages[i] = -1; o_mslots[i] = -1; }
  if (tid == 0) { npages[row] = ns; nmiss[row] = tot_miss; }
}

// ---------------------------------------------------------------------------
// Budget mode, second policy: set-associative placement (lru_policy = 1).
//
// The row's S slots form S / 8 sets of 8 consecutive slots; the home set of a
// page is mix32(row, page) mod sets.  Lookups still go through the leaf entries,
// only placement is constrained.  Misses are placed as if one at a time in
// ascending page id: from the home set on, sets whose 8 ways all hold pages
// selected in this step are skipped (circularly); in the set reached the lowest
// empty way is taken, else the not-selected way with the smallest timestamp
// (lowest way on ties).  Because an admitted page counts as selected, the i-th
// miss to reach a set takes the i-th way of that set's order (empty ways by
// index, then not-selected ways by timestamp and index), whatever the other
// sets do: the kernel ranks the misses per set in parallel and falls back to
// one lane walking the miss list only when some set receives more misses than
// it has ways left.  Timestamps follow step 2 of the bucketed policy.
__device__ inline uint32_t sa_mix32(uint32_t row, uint32_t page) {
  uint32_t x = row * 0x9E3779B1u + page;
  x ^= x >> 16;
  x *= 0x85EBCA6Bu;
  x ^= x >> 13;
  x *= 0xC2B2AE35u;
  x ^= x >> 16;
  return x;
}

#define SA_WAYS 8

template <bool EXPAND>
__global__ __launch_bounds__(LRU_BLOCK) void spin_resolve_sa_kernel(
    const int32_t *__restrict__ sel, const int32_t *__restrict__ nsel, const int32_t *__restrict__ seq_lens,
    const int32_t *__restrict__ dir, int32_t *leaf_pool, int64_t leaf_chunks, int32_t *rev,
    const int32_t *__restrict__ slot_base, int Hkv, int sel_stride, int page_stride, int dir_stride,
    int leaf_entries, int step_arg, int n_ts, int max_slots_lds, int32_t *slots,
    int32_t *page_ids, uint16_t *valid_mask, int32_t *npages,
    int32_t *__restrict__ miss_pages, int32_t *__restrict__ miss_slots, int32_t *__restrict__ nmiss,
    int32_t *status, lru_expand ex) {
  extern __shared__ int32_t lds[];
  // a negative step asks for the workspace's own step counter (word 1 of its header): a captured
  // launch then follows the counter from replay to replay
  const int step = step_arg >= 0 ? step_arg : max(status[1], 0);
  int32_t *s_loc = lds;                                   // [page_stride] leaf entry address per selected page
  int32_t *s_mi = lds + page_stride;                      // [page_stride] selection index of the m-th miss
  int32_t *s_set = lds + 2 * page_stride;                 // [page_stride] home set, then set reached, then victim slot
  int32_t *s_rank = lds + 3 * page_stride;                // [page_stride] arrival rank of the miss in its set
  int32_t *s_cnt = lds + 4 * page_stride;                 // [max_sets] misses homed in the set / ways handed out
  uint8_t *s_cap = (uint8_t *)(s_cnt + max_slots_lds / SA_WAYS);   // [max_sets] ways not holding a selected page
  uint8_t *s_flag = s_cap + max_slots_lds / SA_WAYS;      // [S] 1 = holds a page selected in this step
  __shared__ int s_wave[LRU_WAVES];
  __shared__ int s_err;

  const int row = blockIdx.x, tid = threadIdx.x;
  const int b = row / Hkv;
  const int N = seq_lens[b];
  const int pages = lru_row_pages(ex, row, Hkv, N);
  const int32_t *rsel;
  int ns = lru_input<EXPAND>(row, sel, nsel, seq_lens, dir, leaf_pool, leaf_chunks, Hkv, sel_stride, page_stride,
                             dir_stride, leaf_entries, slots, page_ids, valid_mask, npages, status, ex, rsel);
  ns = ns < 0 ? 0 : ((!EXPAND && ns > sel_stride) ? sel_stride : ns);
  if (ns > page_stride) ns = page_stride;
  int32_t *o_slots = slots + (size_t)row * page_stride;
  int32_t *o_pages = page_ids + (size_t)row * page_stride;
  uint16_t *o_mask = valid_mask + (size_t)row * page_stride;
  int32_t *o_mpages = miss_pages + (size_t)row * page_stride;
  int32_t *o_mslots = miss_slots + (size_t)row * page_stride;
  const int sb = slot_base[2 * row];
  const int S = slot_base[2 * row + 1];
  const int sets = S > 0 ? S / SA_WAYS : 0;
  const int SU = sets * SA_WAYS;                          // slots in whole sets; the rest is never used
  const int32_t *gdir = dir + (size_t)row * dir_stride;

  if (tid == 0) s_err = 0;
  if (S <= max_slots_lds) {
    for (int j = tid; j < SU; j += LRU_BLOCK) s_flag[j] = 0;
    for (int j = tid; j < sets; j += LRU_BLOCK) s_cnt[j] = 0;
  }
  __syncthreads();
  if (S > max_slots_lds || sets < 1 || ns > SU) {
    if (tid == 0) { spin_raise(status, SPIN_ERR_BUDGET); npages[row] = 0; nmiss[row] = 0; }
    for (int i = tid; i < page_stride; i += LRU_BLOCK) { o_slots[i] = -1; o_pages[i] = -1; o_mask[i] = 0; }
    return;
  }
  const int ts_star = min(step, n_ts - 1);

  // (1) classification: hit when the leaf holds a slot of this row
  for (int i = tid; i < ns; i += LRU_BLOCK) {
    const int pg = rsel[i];
    int loc = -1, slot = -1;
    if (pg >= 0 && pg < pages) {
      const int ci = pg / leaf_entries;
      const int32_t chunk = ci < dir_stride ? gdir[ci] : -1;
      if (chunk >= 0 && (int64_t)chunk < leaf_chunks) {
        loc = chunk * leaf_entries + (pg - ci * leaf_entries);
        slot = leaf_pool[loc];
      }
    }
    if (loc < 0) s_err = 1;
    if (slot >= sb && slot < sb + S) {            // resident (a slot past the last whole set can only hold a
      if (slot < sb + SU) s_flag[slot - sb] = 1;  // page admitted before the row's slot count changed)
    } else slot = -1;
    s_loc[i] = loc;
    o_slots[i] = slot;
    if (!EXPAND) {
      o_pages[i] = pg;
      o_mask[i] = (uint16_t)page_mask(pg, N);
    }
  }
  __syncthreads();
  if (s_err) {
    if (tid == 0) { spin_raise(status, SPIN_ERR_NOT_RESIDENT); npages[row] = 0; nmiss[row] = 0; }
    for (int i = tid; i < page_stride; i += LRU_BLOCK) { o_slots[i] = -1; o_pages[i] = -1; o_mask[i] = 0; }
    return;
  }

  // (2) timestamps of the resident pages; ways left per set
  for (int j = tid; j < SU; j += LRU_BLOCK) {
    const int2 e = *(const int2 *)(rev + 2 * (size_t)(sb + j));
    if (e.x < 0) continue;
    int ts = e.y;
    if (s_flag[j]) ts = ts_star;
    else {
      if (step > n_ts - 1) ts = max(ts - 1, 0);
      ts = min(max(ts, 0), n_ts - 1);
    }
    if (ts != e.y) rev[2 * (size_t)(sb + j) + 1] = ts;
  }
  for (int st = tid; st < sets; st += LRU_BLOCK) {
    int c = 0;
#pragma unroll
    for (int w = 0; w < SA_WAYS; ++w) c += s_flag[st * SA_WAYS + w];
    s_cap[st] = (uint8_t)(SA_WAYS - c);
  }

  // (3) the misses in ascending page order (= selection order) and their home sets
  const int pchunk = (ns + LRU_BLOCK - 1) / LRU_BLOCK;
  const int i0 = min(tid * pchunk, ns), i1 = min(i0 + pchunk, ns);
  int cnt = 0;
  for (int i = i0; i < i1; ++i) cnt += (o_slots[i] < 0);
  int tot_miss;
  int mrank = lru_scan(cnt, s_wave, tot_miss);
  for (int i = i0; i < i1; ++i) {
    if (o_slots[i] >= 0) continue;
    const int home = (int)(sa_mix32((uint32_t)row, (uint32_t)o_pages[i]) % (uint32_t)sets);
    s_mi[mrank] = i;
    s_set[mrank] = home;
    atomicAdd(&s_cnt[home], 1);
    ++mrank;
  }
  __syncthreads();
  int over = 0;
  for (int st = tid; st < sets; st += LRU_BLOCK) over |= (s_cnt[st] > (int)s_cap[st]);
  over = __syncthreads_or(over);

  if (!over) {
    // every miss stays in its home set; rank = earlier misses with the same home
    for (int m = tid; m < tot_miss; m += LRU_BLOCK) {
      const int home = s_set[m];
      int r = 0;
      for (int k = 0; k < m; ++k) r += (s_set[k] == home);
      s_rank[m] = r;
    }
  } else {
    for (int st = tid; st < sets; st += LRU_BLOCK) s_cnt[st] = 0;
    __syncthreads();
    if (tid == 0) {
      for (int m = 0; m < tot_miss; ++m) {
        int st = s_set[m], hops = 0;
        while (s_cnt[st] >= (int)s_cap[st] && hops < sets) { st = st + 1 == sets ? 0 : st + 1; ++hops; }
        if (hops >= sets) { s_err = 1; st = -1; }     // cannot happen when ns <= 8 * sets
        else s_rank[m] = s_cnt[st]++;
        s_set[m] = st;
      }
    }
  }
  __syncthreads();
  if (s_err) {   // keep the tables as they are
    if (tid == 0) { spin_raise(status, SPIN_ERR_BUDGET); npages[row] = 0; nmiss[row] = 0; }
    return;
  }

  // (4a) victim of every miss: the way whose position in its set's order equals the rank
  for (int m = tid; m < tot_miss; m += LRU_BLOCK) {
    const int st = s_set[m], r = s_rank[m];
    int key[SA_WAYS], page[SA_WAYS];
#pragma unroll
    for (int w = 0; w < SA_WAYS; ++w) {
      const int j = st * SA_WAYS + w;
      const int2 e = *(const int2 *)(rev + 2 * (size_t)(sb + j));
      page[w] = e.x;
      key[w] = s_flag[j] ? 0x7fffffff : (e.x < 0 ? w : SA_WAYS * (1 + e.y) + w);
    }
    int vw = -1;
#pragma unroll
    for (int w = 0; w < SA_WAYS; ++w) {
      int before = 0;
#pragma unroll
      for (int v = 0; v < SA_WAYS; ++v) before += (key[v] < key[w]);
      if (key[w] != 0x7fffffff && before == r) vw = w;
    }
    int evicted = -1;
#pragma unroll
    for (int w = 0; w < SA_WAYS; ++w)
      if (w == vw) evicted = page[w];
    s_rank[m] = evicted;
    s_set[m] = vw < 0 ? -1 : st * SA_WAYS + vw;
  }
  __syncthreads();

  // (4b) eviction and admission
  for (int m = tid; m < tot_miss; m += LRU_BLOCK) {
    const int i = s_mi[m], j = s_set[m], old = s_rank[m];
    if (j < 0) {                                        // cannot happen: rank < ways left in the set
      spin_raise(status, SPIN_ERR_BUDGET);
      o_mask[i] = 0;
      o_mpages[m] = -1;
      o_mslots[m] = -1;
      continue;
    }
    if (old >= 0) {
      const int ci = old / leaf_entries;
      const int32_t ch = ci < dir_stride ? gdir[ci] : -1;
      if (ch >= 0 && (int64_t)ch < leaf_chunks) leaf_pool[(size_t)ch * leaf_entries + (old - ci * leaf_entries)] = -1;
    }
    const int pg = o_pages[i];
    *(int2 *)(rev + 2 * (size_t)(sb + j)) = make_int2(pg, ts_star);
    leaf_pool[s_loc[i]] = sb + j;
    o_slots[i] = sb + j;
    o_mpages[m] = pg;
    o_mslots[m] = sb + j;
  }
  for (int i = ns + tid; i < page_stride; i += LRU_BLOCK) { o_slots[i] = -1; o_pages[i] = -1; o_mask[i] = 0; }
  for (int i = tot_miss + tid; i < page_stride; i += LRU_BLOCK) { o_mpages[i] = -1; o_mslots[i] = -1; }
  if (tid == 0) { npages[row] = ns; nmiss[row] = tot_miss; }
}

extern "C" int spin_resolve_slots(spin_ctx *ctx, int32_t batch, int32_t step, const int32_t *sel,
                                  const int32_t *nsel, const int32_t *seq_lens, const int32_t *dir,
                                  int32_t *leaf_pool, int64_t leaf_chunks, int32_t *rev_table,
                                  const int32_t *slot_base, int32_t *slots, int32_t *page_ids,
                                  uint16_t *valid_mask, int32_t *npages, int32_t *miss_pages,
                                  int32_t *miss_slots, int32_t *nmiss, void *workspace, void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch || step < SPIN_STEP_FROM_WORKSPACE || leaf_chunks <= 0)
    return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!sel || !nsel || !seq_lens || !dir || !leaf_pool || !slots || !page_ids || !valid_mask || !npages)
    return SPIN_ERR_INVALID;
  if (!workspace) return SPIN_ERR_WORKSPACE;
  const spin_config &c = ctx->cfg;
  const int rows = batch * c.num_kv_heads;
  if (c.lru_timestamps > 0) {
    if (!rev_table || !slot_base || !miss_pages || !miss_slots || !nmiss) return SPIN_ERR_INVALID;
    if (c.lru_timestamps > LRU_MAX_TS) return SPIN_ERR_UNSUPPORTED;
    const bool expand = c.partition_tokens != 16 || ctx->var.count;
    const lru_expand ex = {c.partition_tokens, c.sink_pages, c.recent_pages, ctx->var};
    if (c.lru_policy == 1) {
      // LDS: four int32 per output entry; per set a counter and a byte; one flag byte per slot of the row.
      // The kernels' own static arrays (histogram, directory copy, scan cells: under 3 KiB) come on top of
      // the dynamic part, so the slot capacity is what is left of 64 KiB after a 4 KiB reserve.
      const int64_t avail_sa = LRU_LDS_LIMIT - LRU_LDS_STATIC - (int64_t)ctx->page_stride * 16;
      int64_t cap_sa = avail_sa > 0 ? (avail_sa * 8 / 13) & ~(int64_t)63 : 0;
      if (cap_sa > 32 * 1024) cap_sa = 32 * 1024;
      if (cap_sa < ctx->page_stride || cap_sa < SA_WAYS) return SPIN_ERR_UNSUPPORTED;
      const int max_slots_lds = (int)cap_sa;
      const size_t lds = (size_t)ctx->page_stride * 16 + (size_t)(max_slots_lds / SA_WAYS) * 5 + max_slots_lds;
#define SPIN_SA_ARGS                                                                                            \
  dim3((unsigned)rows), dim3(LRU_BLOCK), lds, (hipStream_t)stream, sel, nsel, seq_lens, dir, leaf_pool, leaf_chunks, \
      rev_table, slot_base, c.num_kv_heads, ctx->sel_stride, ctx->page_stride, ctx->dir_stride, c.leaf_entries,   \
      step, c.lru_timestamps, max_slots_lds, slots, page_ids, valid_mask, npages, miss_pages, miss_slots, nmiss,  \
      (int32_t *)workspace, ex
      if (expand) spin_launch(ctx, SPIN_K_RESOLVE, spin_resolve_sa_kernel<true>, SPIN_SA_ARGS);
      else spin_launch(ctx, SPIN_K_RESOLVE, spin_resolve_sa_kernel<false>, SPIN_SA_ARGS);
#undef SPIN_SA_ARGS
      return spin_launch_status();
    }
    // LDS: two int32 per output entry plus one flag byte per slot of the row (static arrays: see above)
    int64_t cap = (LRU_LDS_LIMIT - LRU_LDS_STATIC - (int64_t)ctx->page_stride * 8) & ~(int64_t)63;
    if (cap > 48 * 1024) cap = 48 * 1024;
    if (cap < ctx->page_stride) return SPIN_ERR_UNSUPPORTED;
    const int max_slots_lds = (int)cap;
    const size_t lds = (size_t)ctx->page_stride * 8 + max_slots_lds;
#define SPIN_LRU_ARGS                                                                                           \
  dim3((unsigned)rows), dim3(LRU_BLOCK), lds, (hipStream_t)stream, sel, nsel, seq_lens, dir, leaf_pool, leaf_chunks, \
      rev_table, slot_base, c.num_kv_heads, ctx->sel_stride, ctx->page_stride, ctx->dir_stride, c.leaf_entries,   \
      step, c.lru_timestamps, c.lru_evict_exact, max_slots_lds, slots, page_ids, valid_mask, npages, miss_pages,  \
      miss_slots, nmiss, (int32_t *)workspace, ex
    if (expand) spin_launch(ctx, SPIN_K_RESOLVE, spin_resolve_lru_kernel<true>, SPIN_LRU_ARGS);
    else spin_launch(ctx, SPIN_K_RESOLVE, spin_resolve_lru_kernel<false>, SPIN_LRU_ARGS);
#undef SPIN_LRU_ARGS
    return spin_launch_status();
  }
  // long selections (token partitions) get a workgroup that covers them in one sweep
#define SPIN_RESOLVE_ARGS                                                                                       \
  0, (hipStream_t)stream, sel, nsel, seq_lens, dir, leaf_pool, leaf_chunks, c.num_kv_heads, c.partition_tokens, \
      c.sink_pages, c.recent_pages, ctx->sel_stride, ctx->page_stride, ctx->dir_stride, c.leaf_entries, slots,  \
      page_ids, valid_mask, npages, (int32_t *)workspace, ctx->var
  if (ctx->sel_stride > 512)
    spin_launch(ctx, SPIN_K_RESOLVE, spin_resolve_kernel<1024>, dim3((unsigned)rows), dim3(1024), SPIN_RESOLVE_ARGS);
  else
    spin_launch(ctx, SPIN_K_RESOLVE, spin_resolve_kernel<256>, dim3((unsigned)rows), dim3(256), SPIN_RESOLVE_ARGS);
#undef SPIN_RESOLVE_ARGS
  return spin_launch_status();
}
