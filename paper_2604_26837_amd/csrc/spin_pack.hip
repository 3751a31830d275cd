// Offload, layout half: token-major pages -> matrix-operand slot layout.
//
// A slot stores its K tile as [dim/8 chunk (16)][token (16)][8 dims] and its V
// tile as [dim/32 (4)][token/4 (4)][dim%16 (16)][(dim/16)%2 (2)][token%4 (4)],
// the register images of the matrix-core operands spin_sparse_decode feeds, so
// each of its loads is one contiguous 1 KiB wavefront transaction.  When
// partitions are smaller than a page both tiles stay token-major,
// [token (16)][dim (128)]: attention then gathers single tokens (spin_k_unit).
#include "spin_common.h"

__global__ __launch_bounds__(256) void spin_pack_kernel(const uint16_t *__restrict__ src_k,
                                                        const uint16_t *__restrict__ src_v,
                                                        const int32_t *__restrict__ slots,
                                                        uint4 *__restrict__ pool, int64_t pool_slots,
                                                        int64_t n_pages, int k_token_major) {
  const int64_t page = blockIdx.x;
  if (page >= n_pages) return;
  const int32_t slot = slots[page];
  if (slot < 0 || (int64_t)slot >= pool_slots) return;  // a slot outside the pool: the page is skipped (this call
                                                        // has no workspace, hence no status word to raise)
  const int u = threadIdx.x;                             // 16-byte unit of the tile
  const int j = u >> 6, c = (u >> 4) & 3, x = u & 15;
  // K unit: token x, dims 32j + 8c .. +8 (contiguous in the source)
  const uint4 *ks = (const uint4 *)(src_k + (page * SPIN_PAGE_TOKENS + x) * SPIN_HEAD_DIM + 32 * j + 8 * c);
  uint4 *dst = pool + (int64_t)slot * SPIN_SLOT_U4;
  dst[spin_k_unit(k_token_major, x, 4 * j + c)] = *ks;
  if (k_token_major) {   // partitions smaller than a page: the V tile stays token-major as well
    dst[SPIN_KTILE_U4 + x * 16 + 4 * j + c] =
        *(const uint4 *)(src_v + (page * SPIN_PAGE_TOKENS + x) * SPIN_HEAD_DIM + 32 * j + 8 * c);
    return;
  }
  // V unit: dim-in-block x, tokens 4c..4c+3 for dim blocks 2j and 2j+1
  const uint16_t *vs = src_v + page * SPIN_PAGE_TOKENS * SPIN_HEAD_DIM;
  uint16_t e[8];
#pragma unroll
  for (int blk = 0; blk < 2; ++blk)
#pragma unroll
    for (int i = 0; i < 4; ++i) e[blk * 4 + i] = vs[(4 * c + i) * SPIN_HEAD_DIM + 32 * j + 16 * blk + x];
  uint4 v;
  v.x = e[0] | ((uint32_t)e[1] << 16);
  v.y = e[2] | ((uint32_t)e[3] << 16);
  v.z = e[4] | ((uint32_t)e[5] << 16);
  v.w = e[6] | ((uint32_t)e[7] << 16);
  dst[SPIN_KTILE_U4 + u] = v;
}

extern "C" int spin_pack_kv_pages(spin_ctx *ctx, int64_t n_pages, const void *src_k, const void *src_v,
                                  const int32_t *slots, void *kv_pool, int64_t pool_slots, void *stream) {
  if (!ctx || n_pages < 0 || pool_slots <= 0) return SPIN_ERR_INVALID;
  if (n_pages == 0) return SPIN_OK;
  if (!src_k || !src_v || !slots || !kv_pool) return SPIN_ERR_INVALID;
  if (n_pages > 0x7fffffffLL) return SPIN_ERR_UNSUPPORTED;
  spin_launch(ctx, SPIN_K_PACK, spin_pack_kernel, dim3((unsigned)n_pages), dim3(256), 0, (hipStream_t)stream,
              (const uint16_t *)src_k, (const uint16_t *)src_v, slots, (uint4 *)kv_pool, pool_slots,
              n_pages, ctx->k_token_major);
  return spin_launch_status();
}
