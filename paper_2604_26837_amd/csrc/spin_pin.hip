// Partitions that always take part in attention besides the sink and recent pages: the outliers an
// Index pass singles out (Section 4.2: outliers and the recent window are kept in GPU memory and
// always participate in attention).  They are pinned by giving them the score +inf between stages
// 1 and 2, so stage 2 takes them before every other candidate and, under a budget, stage 3b
// refreshes their timestamp in every step and never evicts them.
#include "spin_common.h"

__global__ __launch_bounds__(256) void spin_pin_kernel(float *__restrict__ scores, const int32_t *__restrict__ part_offsets,
                                                       const int32_t *__restrict__ pinned,
                                                       const int32_t *__restrict__ npinned, int pinned_stride, int Hkv) {
  const int row = blockIdx.y;
  const int b = row / Hkv, h = row - b * Hkv;
  const int PP = part_offsets[b + 1] - part_offsets[b];
  int n = npinned[row];
  n = n < 0 ? 0 : (n > pinned_stride ? pinned_stride : n);
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const int p = pinned[(size_t)row * pinned_stride + i];
  if (p < 0 || p >= PP) return;                      // ids outside the row are ignored
  scores[(size_t)Hkv * part_offsets[b] + (size_t)h * PP + p] = __builtin_inff();
}

extern "C" int spin_pin_partitions(spin_ctx *ctx, int32_t batch, float *scores, const int32_t *part_offsets,
                                   const int32_t *pinned, const int32_t *npinned, int32_t pinned_stride,
                                   void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch || pinned_stride < 0) return SPIN_ERR_INVALID;
  if (batch == 0 || pinned_stride == 0) return SPIN_OK;
  if (!scores || !part_offsets || !pinned || !npinned) return SPIN_ERR_INVALID;
  const int rows = batch * ctx->cfg.num_kv_heads;
  if (rows > 65535) return SPIN_ERR_UNSUPPORTED;   // rows are the grid's second dimension
  spin_launch(ctx, SPIN_K_SELECT_HIST, spin_pin_kernel, dim3((unsigned)((pinned_stride + 255) / 256), (unsigned)rows),
              dim3(256), 0, (hipStream_t)stream, scores, part_offsets, pinned, npinned, pinned_stride,
              ctx->cfg.num_kv_heads);
  return spin_launch_status();
}
