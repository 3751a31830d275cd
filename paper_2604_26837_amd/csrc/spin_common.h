// Shared host/device declarations of the library's translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "spin.h"
#include "spin_measure.h"

#define SPIN_HEAD_DIM 128
#define SPIN_PAGE_TOKENS 16
#define SPIN_SLOT_U4 512      // 8192-byte slot in 16-byte units
#define SPIN_KTILE_U4 256     // 4096-byte K tile in 16-byte units
#define SPIN_WS_HEADER 256    // bytes reserved in front of the workspace (status word)

#define SPIN_KERNEL_IDS 13

// Variable-length partitions (Section 5.2: the Meta-partition table holds each
// partition's token count, the Partition Offset table where its page list
// starts).  All three arrays are indexed like `scores`: entry base(row) + p.
// count == NULL means uniform partitions of cfg.partition_tokens tokens.
struct spin_var {
  const int32_t *part_offsets;  // [batch+1] the padded partition offsets the tables are indexed with
  const int32_t *count;       // [rows] partitions of the row
  const int32_t *first_page;  // first logical page of partition p
  const int32_t *tokens;      // tokens of partition p (its last page may be partly filled)
};

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
  int32_t side_wgs;       // workgroups per row that attend the always-attended pages beside stages 2+3 (0: not supported)
  int32_t pstride;        // stage 4's partials per row in the workspace: one per split, then one per such workgroup
  int32_t waves;          // wavefronts per decode workgroup
  int32_t depth;          // page buffers per decode wavefront
  int32_t kd;             // contraction length of one summary row
  int32_t rows_per_part;  // summary rows per partition (REPMAX: reps, else 1)
  float scale;
  size_t ws_bytes;
  size_t ws_ticket_off, ws_ml_off, ws_acc_off;
  size_t ws_hist_off;     // per-row first-digit histograms of stage 2 for long rows; 0 = not used
  size_t ws_zero_bytes;   // leading part of the workspace that spin_workspace_init clears
  size_t ws_skip_off;     // [max_rows][2] list positions attended by the launch of stages 2+3 (always-attended pages)
  spin_var var;           // registered partition tables (all NULL: uniform partitions)
  // CPU page table (Section 5.2): entry host_row_base[row] + logical page -> physical page of the pinned
  // host pool; table == NULL: the identity
  const int32_t *cpu_table;
  int64_t cpu_table_entries, cpu_pages;
  int32_t k_token_major;  // layout of a slot's K tile, see spin_k_unit(): 1 for partitions smaller than a page
  // optional per-kernel timing: pairs of HIP events handed to the launches
  int32_t prof_cap;
  int32_t prof_n[SPIN_KERNEL_IDS];
  hipEvent_t *prof_ev[SPIN_KERNEL_IDS];   // [2 * prof_cap]: start, stop, start, stop, ...
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

// attention over a row's always-attended pages beside stages 2+3, the rest in stage 4: all-resident mode,
// uniform partitions of whole pages, rows short enough for the 512-thread selection
static inline bool spin_forced_split_supported(const spin_ctx *ctx) { return ctx->side_wgs > 0; }

static inline int spin_launch_status() {
  return hipGetLastError() == hipSuccess ? SPIN_OK : SPIN_ERR_HIP;
}

// host-side bodies of stages 1 and 2, shared by the stage calls and the combined call.
// hist != NULL: stage 1 also counts the leading 12 key bits of every candidate's score into the
// per-row histograms stage 2 of long rows starts from; hist_ready: stage 2 finds them filled.
int spin_score_impl(spin_ctx *ctx, int32_t batch, const void *q, const void *summaries, const int32_t *chan_idx,
                    const int32_t *part_offsets, const int32_t *seq_lens, float *scores, void *workspace,
                    void *stream, int32_t *hist);
// `res` != NULL (all-resident mode, rows of 16385 - 131072 partitions only): the launch that finishes
// stage 2 also runs stage 3 for its row and stores the results there; SPIN_ERR_UNSUPPORTED elsewhere.
struct spin_resolve_args {
  const int32_t *dir;
  const int32_t *leaf_pool;
  int64_t leaf_chunks;
  int32_t *slots, *page_ids;
  uint16_t *valid_mask;
  int32_t *npages;
};
// Looks the device address of the library's own scratch array up for the current device (kept per device
// from then on), so that spin_sparse_decode_static need not do it on its first call.
int spin_static_scratch_prepare(void);
int spin_select_impl(spin_ctx *ctx, int32_t batch, const float *scores, const int32_t *part_offsets,
                     const int32_t *seq_lens, int32_t *sel, int32_t *nsel, void *workspace, void *stream,
                     bool hist_ready, const spin_resolve_args *res);

#ifdef __HIPCC__
// Launch `kernel` on `st`; when timing is enabled the launch carries a start
// and a stop event that take the kernel's own begin and end timestamps.
template <typename K, typename... Args>
static inline void spin_launch(spin_ctx *ctx, int kid, K kernel, dim3 grid, dim3 block, size_t lds, hipStream_t st,
                               Args... args) {
  if (ctx->prof_cap > 0 && ctx->prof_n[kid] < ctx->prof_cap) {
    const int i = ctx->prof_n[kid]++;
    hipExtLaunchKernelGGL(kernel, grid, block, lds, st, ctx->prof_ev[kid][2 * i], ctx->prof_ev[kid][2 * i + 1], 0,
                          args...);
  } else {
    hipLaunchKernelGGL(kernel, grid, block, lds, st, args...);
  }
}

// first device-detected fault wins; later ones are dropped
__device__ inline void spin_raise(int32_t *status, int32_t err) { atomicCAS(status, 0, err); }

__device__ inline float spin_bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// device-scope (all compute dies) relaxed accesses: written through / read from
// the level every die sees, without cache-wide write-back or invalidate
__device__ inline void spin_dev_store(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline float spin_dev_load(const float *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// 16-byte load marked non-temporal (streamed once, not worth keeping in cache)
typedef __attribute__((ext_vector_type(4))) unsigned int spin_u32x4;
__device__ inline uint4 spin_nt_load(const uint4 *p) {
  return __builtin_bit_cast(uint4, __builtin_nontemporal_load((const spin_u32x4 *)p));
}

typedef __attribute__((ext_vector_type(2))) unsigned int spin_u32x2;
__device__ inline uint2 spin_nt_load2(const uint2 *p) {
  return __builtin_bit_cast(uint2, __builtin_nontemporal_load((const spin_u32x2 *)p));
}

// fp32 -> bf16 bits, round to nearest even
__device__ inline uint16_t spin_f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;
  return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

// logical page -> slot through the two-level table; -1 when the leaf or the
// entry is missing
__device__ inline int32_t spin_walk(const int32_t *__restrict__ dir, const int32_t *__restrict__ leaf_pool,
                                    int64_t leaf_chunks, int row, int dir_stride, int leaf_entries, int page) {
  if (page < 0) return -1;
  const int ci = page / leaf_entries;
  if (ci >= dir_stride) return -1;
  const int32_t chunk = dir[(size_t)row * dir_stride + ci];
  if (chunk < 0 || (int64_t)chunk >= leaf_chunks) return -1;
  return leaf_pool[(size_t)chunk * leaf_entries + (page - ci * leaf_entries)];
}

// variable-length partitions: first table entry of a row
__device__ inline size_t spin_var_base(const spin_var &v, int row, int Hkv) {
  const int b = row / Hkv, h = row - b * Hkv;
  const int off = v.part_offsets[b];
  return (size_t)Hkv * off + (size_t)h * (v.part_offsets[b + 1] - off);
}
// variable-length partitions: pages of partition p, and the row's page count
__device__ inline int spin_var_npages(const spin_var &v, size_t base, int p) { return (v.tokens[base + p] + 15) >> 4; }
__device__ inline int spin_var_row_pages(const spin_var &v, size_t base, int P) {
  return P > 0 ? v.first_page[base + P - 1] + spin_var_npages(v, base, P - 1) : 0;
}
// first p in [0, P) whose first page is >= page (P if none); first pages ascend
__device__ inline int spin_var_lower_bound_start(const spin_var &v, size_t base, int P, int page) {
  int lo = 0, hi = P;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (v.first_page[base + mid] >= page) hi = mid; else lo = mid + 1;
  }
  return lo;
}
// number of leading partitions that end at or before `page`
__device__ inline int spin_var_count_end_le(const spin_var &v, size_t base, int P, int page) {
  int lo = 0, hi = P;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (v.first_page[base + mid] + spin_var_npages(v, base, mid) <= page) lo = mid + 1; else hi = mid;
  }
  return lo;
}

// DPP lane exchanges inside a row of 16 lanes
#define SPIN_DPP_XOR1 0xB1        /* quad_perm [1,0,3,2] */
#define SPIN_DPP_XOR2 0x4E        /* quad_perm [2,3,0,1] */
#define SPIN_DPP_HALF_MIRROR 0x141
#define SPIN_DPP_MIRROR 0x140
template <int CTRL>
__device__ inline float spin_dpp(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
// 16-byte unit of (token t, 8-channel chunk ch) inside a slot's K tile.  Partitions of whole pages:
// chunk-major [chunk][token], the matrix operand's register image (a wavefront load is one
// contiguous KiB).  Partitions smaller than a page: token-major [token][chunk], a token's key is
// 256 contiguous bytes, so attending to one token of a page touches two cache lines, not sixteen
// (the V tile of such a slot is token-major too: the slot is simply K[16][128] then V[16][128]).
__device__ inline int spin_k_unit(int token_major, int t, int ch) { return token_major ? t * 16 + ch : ch * 16 + t; }
template <int CTRL>
__device__ inline int spin_dpp_i(int v) {   // lanes whose source lies outside the row read 0
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}
// inclusive prefix sum over the 64 lanes of a wavefront: four row shifts inside each row of 16
// lanes, then the totals of the rows before (three lane reads); no trip through LDS
__device__ inline int spin_wave_inclusive_scan(int v) {
  v += spin_dpp_i<0x111>(v);   // row_shr:1
  v += spin_dpp_i<0x112>(v);   // row_shr:2
  v += spin_dpp_i<0x114>(v);   // row_shr:4
  v += spin_dpp_i<0x118>(v);   // row_shr:8
  const int t0 = __builtin_amdgcn_readlane(v, 15), t1 = __builtin_amdgcn_readlane(v, 31),
            t2 = __builtin_amdgcn_readlane(v, 47);
  const int row = (threadIdx.x & 63) >> 4;
  return v + (row >= 1 ? t0 : 0) + (row >= 2 ? t1 : 0) + (row >= 3 ? t2 : 0);
}
// maximum / minimum of an unsigned word over the wavefront, result uniform
__device__ inline uint32_t spin_wave_max_u32(uint32_t v) {
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, SPIN_DPP_XOR1, 0xf, 0xf, false));
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, SPIN_DPP_XOR2, 0xf, 0xf, false));
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, SPIN_DPP_HALF_MIRROR, 0xf, 0xf, false));
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, SPIN_DPP_MIRROR, 0xf, 0xf, false));
  return max(max((uint32_t)__builtin_amdgcn_readlane((int)v, 0), (uint32_t)__builtin_amdgcn_readlane((int)v, 16)),
             max((uint32_t)__builtin_amdgcn_readlane((int)v, 32), (uint32_t)__builtin_amdgcn_readlane((int)v, 48)));
}
__device__ inline uint32_t spin_wave_min_u32(uint32_t v) { return ~spin_wave_max_u32(~v); }

// Order-preserving 32-bit key of a score, the order stage 2 ranks by.
__device__ inline uint32_t score_key(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) u = 0xff800000u;  // NaN ranks as -inf
  if (u == 0x80000000u) u = 0u;                          // -0 ties +0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// bins of the chip-wide histogram of the leading 12 key bits (stage 2 of long rows)
#define BIG_BINS 4096
#endif
