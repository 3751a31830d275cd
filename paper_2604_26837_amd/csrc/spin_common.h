// Shared host/device declarations of the library's translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spin.h"

#define SPIN_HEAD_DIM 128
#define SPIN_PAGE_TOKENS 16
#define SPIN_SLOT_U4 512      // 8192-byte slot in 16-byte units
#define SPIN_KTILE_U4 256     // 4096-byte K tile in 16-byte units
#define SPIN_WS_HEADER 256    // bytes reserved in front of the workspace (status word)
#define SPIN_DECODE_WAVES 4

struct spin_ctx {
  spin_config cfg;
  int32_t group;          // query heads per KV head
  int32_t max_rows;       // max_batch * num_kv_heads
  int32_t max_pages;      // pages of a max_context request
  int32_t max_parts;      // partitions of a max_context request
  int32_t pages_per_part; // partition_tokens / 16 when >= 16, else 0
  int32_t parts_per_page; // 16 / partition_tokens when < 16, else 0
  int32_t sel_stride;
  int32_t page_stride;
  int32_t dir_stride;
  int32_t splits;
  int32_t kd;             // contraction length of one summary row
  int32_t rows_per_part;  // summary rows per partition (REPMAX: reps, else 1)
  float scale;
  size_t ws_bytes;
  size_t ws_ml_off, ws_acc_off;
};

typedef __attribute__((ext_vector_type(8))) __bf16 spin_bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 spin_bf16x2;
typedef __attribute__((ext_vector_type(4))) float spin_f32x4;
typedef __attribute__((ext_vector_type(4))) short spin_s16x4;

#define SPIN_HIP_CHECK(expr)                 \
  do {                                       \
    hipError_t e_ = (expr);                  \
    if (e_ != hipSuccess) return SPIN_ERR_HIP; \
  } while (0)

static inline int spin_launch_status() {
  return hipGetLastError() == hipSuccess ? SPIN_OK : SPIN_ERR_HIP;
}

#ifdef __HIPCC__
// first device-detected fault wins; later ones are dropped
__device__ inline void spin_raise(int32_t *status, int32_t err) { atomicCAS(status, 0, err); }

__device__ inline float spin_bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
#endif
