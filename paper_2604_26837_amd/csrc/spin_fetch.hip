// Retrieve steps 3-4 (Section 5.2): bring the missed pages from pinned host
// memory into the slots stage 3b assigned to them.
//
// Two copiers.  The host-driven one issues one 8 KiB hipMemcpyAsync per miss on
// a side stream (needs the miss list on the host).  The device-driven one is
// the paper's copy kernel (Section 5.5): one wavefront copies one page with
// 16-byte lane transactions straight out of pinned host memory; a fixed, small number of
// workgroups walks the (row, chunk of misses) pairs with a grid stride, so pages are spread over
// the wavefronts whatever row owns them, and the miss list never leaves the device.  The same
// kernel run the other way is Offload's copy (slot -> host page).
#include "spin_common.h"

extern "C" int spin_copy_misses_host(spin_ctx *ctx, int32_t batch, const void *host_kv,
                                     const int64_t *host_row_base, const int32_t *nmiss,
                                     const int32_t *miss_pages, const int32_t *miss_slots, void *kv_pool,
                                     int64_t pool_slots, void *copy_stream, int64_t *pages_copied) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch || pool_slots <= 0) return SPIN_ERR_INVALID;
  if (pages_copied) *pages_copied = 0;
  if (batch == 0) return SPIN_OK;
  if (!host_kv || !host_row_base || !nmiss || !miss_pages || !miss_slots || !kv_pool) return SPIN_ERR_INVALID;
  const int rows = batch * ctx->cfg.num_kv_heads;
  const int stride = ctx->page_stride;
  int64_t total = 0;
  for (int r = 0; r < rows; ++r) {
    const int n = nmiss[r];
    if (n < 0 || n > stride) return SPIN_ERR_INVALID;
    for (int i = 0; i < n; ++i) {
      const int32_t pg = miss_pages[(size_t)r * stride + i], slot = miss_slots[(size_t)r * stride + i];
      if (pg < 0 || slot < 0 || (int64_t)slot >= pool_slots) return SPIN_ERR_INVALID;
      int64_t hp = host_row_base[r] + pg;
      if (ctx->cpu_table) {                 // pinned host memory: readable from here as well
        if (hp < 0 || hp >= ctx->cpu_table_entries) return SPIN_ERR_INVALID;
        hp = ctx->cpu_table[hp];
      }
      // the host pool's size, when one was registered (with or without a table), bounds the page
      if (hp < 0 || (ctx->cpu_pages > 0 && hp >= ctx->cpu_pages)) return SPIN_ERR_INVALID;
      const char *src = (const char *)host_kv + (size_t)hp * SPIN_SLOT_BYTES;
      char *dst = (char *)kv_pool + (size_t)slot * SPIN_SLOT_BYTES;
      SPIN_HIP_CHECK(hipMemcpyAsync(dst, src, SPIN_SLOT_BYTES, hipMemcpyHostToDevice, (hipStream_t)copy_stream));
      ++total;
    }
  }
  if (pages_copied) *pages_copied = total;
  return SPIN_OK;
}

#define GATHER_WAVES 4
#define GATHER_PAGES_PER_WG 16
// Workgroups of a copy launch.  The host link is the limit (about 54 GB/s), and it takes about 64 compute units
// to saturate it (measured per step of the budget workload, 6.4 K pages: 8 / 16 / 32 / 64 / 128 / 512 / 2048
// workgroups -> 2605 / 1489 / 1092 / 1001 / 1000 / 1032 / 1032 us); more only crowd the units that other
// launches could use meanwhile.
#define GATHER_MAX_WGS 64

struct host_map {
  const int32_t *table;     // NULL: identity
  int64_t entries, pages;
};

// TO_HOST = false: host page -> slot (Retrieve).  TO_HOST = true: slot -> host page (Offload's copy,
// Table 1: copy(gpu_kv, cpu_kv, map)); the lists have the same shape in both directions.
template <bool TO_HOST>
__global__ __launch_bounds__(GATHER_WAVES * 64) void spin_gather_kernel(
    uint4 *__restrict__ host_kv, const int64_t *__restrict__ row_base, const int32_t *__restrict__ nmiss,
    const int32_t *__restrict__ miss_pages, const int32_t *__restrict__ miss_slots, uint4 *__restrict__ pool,
    int64_t pool_slots, int page_stride, int chunks_per_row, int total_items, int32_t *status, host_map hm) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // (row, chunk of the row's list) pairs are dealt to the workgroups with a grid stride: the link needs few
  // pages in flight, so the launch stays small and leaves the compute units to whatever runs beside it
  for (int item = blockIdx.x; item < total_items; item += gridDim.x) {
  const int row = item / chunks_per_row, chunk = item - row * chunks_per_row;
  int n = nmiss[row];
  n = n < 0 ? 0 : (n > page_stride ? page_stride : n);
  const int begin = chunk * GATHER_PAGES_PER_WG;
  const int end = min(begin + GATHER_PAGES_PER_WG, n);
  const int64_t rb = row_base[row];
  for (int i = begin + wave; i < end; i += GATHER_WAVES) {
    const int32_t pg = miss_pages[(size_t)row * page_stride + i];
    const int32_t slot = miss_slots[(size_t)row * page_stride + i];
    if (pg < 0 || slot < 0 || (int64_t)slot >= pool_slots) {
      if (lane == 0) spin_raise(status, SPIN_ERR_SLOT_RANGE);
      continue;
    }
    int64_t hpage = rb + pg;
    if (hm.table) {                         // CPU page table: offset of the page in the row's list -> physical host page
      const bool in_table = hpage >= 0 && hpage < hm.entries;
      hpage = in_table ? hm.table[hpage] : -1;
    }
    // the host pool's size, when one was registered (with or without a table), bounds the page
    if (hpage < 0 || (hm.pages > 0 && hpage >= hm.pages)) {
      if (lane == 0) spin_raise(status, SPIN_ERR_SLOT_RANGE);
      continue;
    }
    uint4 *hp = host_kv + (size_t)hpage * SPIN_SLOT_U4 + lane;
    uint4 *dp = pool + (size_t)slot * SPIN_SLOT_U4 + lane;
    const uint4 *src = TO_HOST ? dp : hp;
    uint4 *dst = TO_HOST ? hp : dp;
    uint4 v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = src[k * 64];
#pragma unroll
    for (int k = 0; k < 8; ++k) dst[k * 64] = v[k];
  }
  }
}

extern "C" int spin_gather_misses(spin_ctx *ctx, int32_t batch, const void *host_kv, const int64_t *row_base,
                                  const int32_t *nmiss, const int32_t *miss_pages, const int32_t *miss_slots,
                                  void *kv_pool, int64_t pool_slots, void *workspace, void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch || pool_slots <= 0) return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!host_kv || !row_base || !nmiss || !miss_pages || !miss_slots || !kv_pool) return SPIN_ERR_INVALID;
  if (!workspace) return SPIN_ERR_WORKSPACE;
  const int rows = batch * ctx->cfg.num_kv_heads;
  const int chunks = (ctx->page_stride + GATHER_PAGES_PER_WG - 1) / GATHER_PAGES_PER_WG;
  spin_launch(ctx, SPIN_K_GATHER, spin_gather_kernel<false>, dim3((unsigned)min(rows * chunks, GATHER_MAX_WGS)), dim3(GATHER_WAVES * 64), 0,
              (hipStream_t)stream, (uint4 *)const_cast<void *>(host_kv), row_base, nmiss, miss_pages, miss_slots,
              (uint4 *)kv_pool, pool_slots, ctx->page_stride, chunks, rows * chunks, (int32_t *)workspace,
              host_map{ctx->cpu_table, ctx->cpu_table_entries, ctx->cpu_pages});
  return spin_launch_status();
}

extern "C" int spin_offload_pages(spin_ctx *ctx, int32_t batch, const void *kv_pool, int64_t pool_slots, void *host_kv,
                                  const int64_t *row_base, const int32_t *count, const int32_t *pages,
                                  const int32_t *slots, void *workspace, void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch || pool_slots <= 0) return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!host_kv || !row_base || !count || !pages || !slots || !kv_pool) return SPIN_ERR_INVALID;
  if (!workspace) return SPIN_ERR_WORKSPACE;
  const int rows = batch * ctx->cfg.num_kv_heads;
  const int chunks = (ctx->page_stride + GATHER_PAGES_PER_WG - 1) / GATHER_PAGES_PER_WG;
  spin_launch(ctx, SPIN_K_OFFLOAD, spin_gather_kernel<true>, dim3((unsigned)min(rows * chunks, GATHER_MAX_WGS)), dim3(GATHER_WAVES * 64), 0,
              (hipStream_t)stream, (uint4 *)host_kv, row_base, count, pages, slots,
              (uint4 *)const_cast<void *>(kv_pool), pool_slots, ctx->page_stride, chunks, rows * chunks, (int32_t *)workspace,
              host_map{ctx->cpu_table, ctx->cpu_table_entries, ctx->cpu_pages});
  return spin_launch_status();
}

extern "C" int spin_set_host_page_table(spin_ctx *ctx, const int32_t *cpu_pages, int64_t entries, int64_t host_pages) {
  if (!ctx) return SPIN_ERR_INVALID;
  if (!cpu_pages) {   // identity mapping; host_pages > 0 still bounds the pages the copiers touch
    if (host_pages < 0) return SPIN_ERR_INVALID;
    ctx->cpu_table = nullptr; ctx->cpu_table_entries = 0; ctx->cpu_pages = host_pages;
    return SPIN_OK;
  }
  if (entries <= 0 || host_pages <= 0) return SPIN_ERR_INVALID;
  ctx->cpu_table = cpu_pages; ctx->cpu_table_entries = entries; ctx->cpu_pages = host_pages;
  return SPIN_OK;
}

// Splits a row's token masks by whether the page had to be fetched: while the copy of the missed pages is under
// way, attention can already run over the pages that hit (Section 5.2, Retrieve: only the misses travel).  Both
// lists ascend by page id, so a page is a miss iff a binary search finds it in the row's miss list.
__global__ __launch_bounds__(256) void spin_split_kernel(const int32_t *__restrict__ page_ids,
                                                         const uint16_t *__restrict__ mask,
                                                         const int32_t *__restrict__ npages,
                                                         const int32_t *__restrict__ miss_pages,
                                                         const int32_t *__restrict__ nmiss, int page_stride,
                                                         uint16_t *__restrict__ mask_hits,
                                                         uint16_t *__restrict__ mask_misses) {
  const int row = blockIdx.x;
  int np = npages[row], nm = nmiss[row];
  np = np < 0 ? 0 : (np > page_stride ? page_stride : np);
  nm = nm < 0 ? 0 : (nm > page_stride ? page_stride : nm);
  const int32_t *mp = miss_pages + (size_t)row * page_stride;
  for (int i = threadIdx.x; i < page_stride; i += blockDim.x) {
    uint16_t hit = 0, miss = 0;
    if (i < np) {
      const int32_t pg = page_ids[(size_t)row * page_stride + i];
      int lo = 0, hi = nm;
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (mp[mid] < pg) lo = mid + 1; else hi = mid;
      }
      const bool is_miss = lo < nm && mp[lo] == pg;
      const uint16_t m = mask[(size_t)row * page_stride + i];
      hit = is_miss ? 0 : m;
      miss = is_miss ? m : 0;
    }
    mask_hits[(size_t)row * page_stride + i] = hit;
    mask_misses[(size_t)row * page_stride + i] = miss;
  }
}

extern "C" int spin_split_hits_misses(spin_ctx *ctx, int32_t batch, const int32_t *page_ids, const uint16_t *valid_mask,
                                      const int32_t *npages, const int32_t *miss_pages, const int32_t *nmiss,
                                      uint16_t *mask_hits, uint16_t *mask_misses, void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch) return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!page_ids || !valid_mask || !npages || !miss_pages || !nmiss || !mask_hits || !mask_misses) return SPIN_ERR_INVALID;
  const int rows = batch * ctx->cfg.num_kv_heads;
  spin_launch(ctx, SPIN_K_META, spin_split_kernel, dim3((unsigned)rows), dim3(256), 0, (hipStream_t)stream, page_ids,
              valid_mask, npages, miss_pages, nmiss, ctx->page_stride, mask_hits, mask_misses);
  return spin_launch_status();
}
