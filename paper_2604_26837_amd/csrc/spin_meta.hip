// Metadata mechanisms around budget-mode stage 3: reclaiming slots from the
// tail of a row's slot table (Section 5.3, buffer elasticity) and allocating
// second-level table segments on demand from a bitmap-managed pool (Section 5.4).
#include "spin_common.h"

#define META_BLOCK 256
#define META_DIR_LDS 256

__global__ __launch_bounds__(META_BLOCK) void spin_reclaim_kernel(int32_t *slot_range, const int32_t *__restrict__ new_count,
                                                                  const int32_t *__restrict__ dir, int32_t *leaf_pool,
                                                                  int64_t leaf_chunks, int32_t *rev, int dir_stride,
                                                                  int leaf_entries, int32_t *status) {
  const int row = blockIdx.x;
  const int sb = slot_range[2 * row], S = slot_range[2 * row + 1];
  int keep = new_count[row];
  if (keep < 0) keep = 0;
  for (int j = keep + (int)threadIdx.x; j < S; j += META_BLOCK) {
    const int2 e = *(const int2 *)(rev + 2 * (size_t)(sb + j));
    if (e.x < 0) continue;
    const int ci = e.x / leaf_entries;
    const int32_t ch = ci < dir_stride ? dir[(size_t)row * dir_stride + ci] : -1;
    if (ch >= 0 && (int64_t)ch < leaf_chunks) leaf_pool[(size_t)ch * leaf_entries + (e.x - ci * leaf_entries)] = -1;
    else spin_raise(status, SPIN_ERR_NOT_RESIDENT);
    *(int2 *)(rev + 2 * (size_t)(sb + j)) = make_int2(-1, 0);
  }
  __syncthreads();
  if (threadIdx.x == 0) slot_range[2 * row + 1] = keep;
}

// take one free chunk: set a clear bit, looking from bit `start` of the bitmap onwards (circularly).
// Requests that start at different bits do not meet as long as the pool has room near them.
__device__ inline int32_t bitmap_take(uint32_t *bitmap, int64_t chunks, int64_t start) {
  const int nwords = (int)((chunks + 31) / 32);
  const int w0 = (int)(start >> 5) % nwords, sb = (int)(start & 31);
  for (int k = 0; k < nwords; ++k) {
    const int w = (w0 + k) % nwords;
    const int rot = k == 0 ? sb : 0;                 // the first word is searched from the start bit, circularly
    uint32_t word = __hip_atomic_load(&bitmap[w], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (;;) {
      uint32_t freeb = ~word;
      if ((int64_t)w * 32 + 32 > chunks) freeb &= (1u << (int)(chunks - (int64_t)w * 32)) - 1u;   // padding bits
      if (!freeb) break;
      const uint32_t r = rot ? ((freeb >> rot) | (freeb << (32 - rot))) : freeb;
      const int bit = (__builtin_ctz(r) + rot) & 31;
      const uint32_t old = atomicOr(&bitmap[w], 1u << bit);
      if (!(old & (1u << bit))) return (int32_t)((int64_t)w * 32 + bit);
      word = old | (1u << bit);
    }
  }
  return -1;
}

__global__ __launch_bounds__(META_BLOCK) void spin_alloc_leaves_kernel(
    const int32_t *__restrict__ sel, const int32_t *__restrict__ nsel, const int32_t *__restrict__ seq_lens,
    int32_t *dir, int32_t *leaf_pool, int64_t leaf_chunks, uint32_t *bitmap, int Hkv, int tp, int sink_pages,
    int recent_pages, int sel_stride, int dir_stride, int leaf_entries, int32_t *status) {
  __shared__ int s_need[META_DIR_LDS];
  __shared__ int s_new[META_DIR_LDS];
  const int row = blockIdx.x, tid = threadIdx.x;
  const int b = row / Hkv;
  const int N = seq_lens[b];
  const int pages = (N + 15) >> 4;
  int ns = nsel[row];
  ns = ns < 0 ? 0 : (ns > sel_stride ? sel_stride : ns);
  int32_t *rdir = dir + (size_t)row * dir_stride;
  for (int i = tid; i < dir_stride; i += META_BLOCK) { s_need[i] = 0; s_new[i] = -1; }
  __syncthreads();
  // ranges touched by the selected partitions and by the forced pages
  for (int i = tid; i < ns; i += META_BLOCK) {
    const int s = sel[(size_t)row * sel_stride + i];
    if (s < 0) continue;
    const int t0 = s * tp, t1 = min(t0 + tp, N);
    if (t1 <= t0) continue;
    for (int ci = (t0 >> 4) / leaf_entries; ci <= ((t1 - 1) >> 4) / leaf_entries && ci < dir_stride; ++ci) s_need[ci] = 1;
  }
  for (int pg = tid; pg < min(sink_pages, pages); pg += META_BLOCK) s_need[pg / leaf_entries] = 1;
  for (int pg = max(pages - recent_pages, 0) + tid; pg < pages; pg += META_BLOCK)
    if (pg / leaf_entries < dir_stride) s_need[pg / leaf_entries] = 1;
  __syncthreads();
  for (int ci = tid; ci < dir_stride; ci += META_BLOCK) {
    if (!s_need[ci] || rdir[ci] >= 0) continue;
    // requests spread over the pool in proportion to (row, range): no two meet while the pool has room
    const int64_t want = (int64_t)row * dir_stride + ci, all = (int64_t)gridDim.x * dir_stride;
    const int32_t ch = bitmap_take(bitmap, leaf_chunks, want * leaf_chunks / all);
    if (ch < 0) { spin_raise(status, SPIN_ERR_LEAF_POOL); continue; }
    s_new[ci] = ch;
  }
  __syncthreads();
  // fill the new leaves with "not resident", then publish them in the directory
  for (int ci = 0; ci < dir_stride; ++ci) {
    const int32_t ch = s_new[ci];
    if (ch < 0) continue;
    for (int i = tid; i < leaf_entries; i += META_BLOCK) leaf_pool[(size_t)ch * leaf_entries + i] = -1;
  }
  __syncthreads();
  for (int ci = tid; ci < dir_stride; ci += META_BLOCK)
    if (s_new[ci] >= 0) rdir[ci] = s_new[ci];
}

__global__ __launch_bounds__(META_BLOCK) void spin_free_leaves_kernel(int32_t *dir, int64_t leaf_chunks, uint32_t *bitmap,
                                                                      int dir_stride) {
  const int row = blockIdx.x;
  int32_t *rdir = dir + (size_t)row * dir_stride;
  for (int ci = threadIdx.x; ci < dir_stride; ci += META_BLOCK) {
    const int32_t ch = rdir[ci];
    if (ch >= 0 && (int64_t)ch < leaf_chunks) atomicAnd(&bitmap[ch >> 5], ~(1u << (ch & 31)));
    rdir[ci] = -1;
  }
}

extern "C" int spin_reclaim_tail(spin_ctx *ctx, int32_t batch, int32_t *slot_range, const int32_t *new_count,
                                 const int32_t *dir, int32_t *leaf_pool, int64_t leaf_chunks, int32_t *rev_table,
                                 void *workspace, void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch || leaf_chunks <= 0) return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!slot_range || !new_count || !dir || !leaf_pool || !rev_table) return SPIN_ERR_INVALID;
  if (!workspace) return SPIN_ERR_WORKSPACE;
  const int rows = batch * ctx->cfg.num_kv_heads;
  spin_launch(ctx, SPIN_K_META, spin_reclaim_kernel, dim3((unsigned)rows), dim3(META_BLOCK), 0, (hipStream_t)stream, slot_range,
                     new_count, dir, leaf_pool, leaf_chunks, rev_table, ctx->dir_stride, ctx->cfg.leaf_entries,
                     (int32_t *)workspace);
  return spin_launch_status();
}

extern "C" int spin_alloc_leaves(spin_ctx *ctx, int32_t batch, const int32_t *sel, const int32_t *nsel,
                                 const int32_t *seq_lens, int32_t *dir, int32_t *leaf_pool, int64_t leaf_chunks,
                                 uint32_t *leaf_bitmap, void *workspace, void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch || leaf_chunks <= 0) return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!sel || !nsel || !seq_lens || !dir || !leaf_pool || !leaf_bitmap) return SPIN_ERR_INVALID;
  if (!workspace) return SPIN_ERR_WORKSPACE;
  if (ctx->dir_stride > META_DIR_LDS) return SPIN_ERR_UNSUPPORTED;
  // the kernel takes a partition's page range from its id alone: not with registered partition tables
  if (ctx->var.count) return SPIN_ERR_UNSUPPORTED;
  const spin_config &c = ctx->cfg;
  const int rows = batch * c.num_kv_heads;
  spin_launch(ctx, SPIN_K_META, spin_alloc_leaves_kernel, dim3((unsigned)rows), dim3(META_BLOCK), 0, (hipStream_t)stream, sel, nsel,
                     seq_lens, dir, leaf_pool, leaf_chunks, leaf_bitmap, c.num_kv_heads, c.partition_tokens,
                     c.sink_pages, c.recent_pages, ctx->sel_stride, ctx->dir_stride, c.leaf_entries,
                     (int32_t *)workspace);
  return spin_launch_status();
}

extern "C" int spin_free_leaves(spin_ctx *ctx, int32_t batch, int32_t *dir, int64_t leaf_chunks, uint32_t *leaf_bitmap,
                                void *workspace, void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch || leaf_chunks <= 0) return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!dir || !leaf_bitmap) return SPIN_ERR_INVALID;
  (void)workspace;
  const int rows = batch * ctx->cfg.num_kv_heads;
  spin_launch(ctx, SPIN_K_META, spin_free_leaves_kernel, dim3((unsigned)rows), dim3(META_BLOCK), 0, (hipStream_t)stream, dir,
                     leaf_chunks, leaf_bitmap, ctx->dir_stride);
  return spin_launch_status();
}
