// Index at decode time (Section 4.1: Index is invoked during decode to
// incorporate newly generated tokens): append one token's K/V per row into its
// page slot and bring the summaries of the partition it lands in up to date.
//
// One workgroup of 128 threads per row, thread d = channel d.  The summary
// update reproduces what a full rebuild would store: min/max fold in the new key
// (or restart on the first token of a partition), the sketch row is written,
// and a block representative is recomputed from the keys in the pool with the
// same exact fp64 sum and single rounding as the bulk builder.
#include "spin_common.h"

__device__ inline size_t k_elem(int token_major, int t, int d) { return ((size_t)spin_k_unit(token_major, t, d >> 3) << 3) + (d & 7); }
__device__ inline size_t v_elem(int token_major, int t, int d) {
  if (token_major) return (size_t)t * SPIN_HEAD_DIM + d;
  return (((size_t)((d >> 5) * 64 + (t >> 2) * 16 + (d & 15)) * 2 + ((d >> 4) & 1)) << 2) + (t & 3);
}
__device__ inline size_t summ_elem(size_t R, int e, int kd, int kc) {
  return (R >> 4) * (size_t)(16 * kd) + ((size_t)(e / kc) * 16 + (R & 15)) * kc + (e % kc);
}
__device__ inline uint16_t f64_to_bf16(double x) {
  float f = __double2float_rz(x);
  uint32_t u = __float_as_uint(f);
  if ((double)f != x) u |= 1u;   // sticky bit: round to odd, then one rounding to bf16
  return spin_f32_to_bf16(__uint_as_float(u));
}

__global__ __launch_bounds__(128) void spin_append_kernel(
    const uint16_t *__restrict__ k_new, const uint16_t *__restrict__ v_new, const int32_t *__restrict__ seq_lens,
    uint16_t *pool, int64_t pool_slots, const int32_t *__restrict__ dir, const int32_t *__restrict__ leaf_pool,
    int64_t leaf_chunks, const int32_t *__restrict__ part_offsets, const int32_t *__restrict__ chan,
    uint16_t *summ, int Hkv, int tp, int kind, int reps, int dir_stride, int leaf_entries, int k_token_major,
    int32_t *status) {
  const int row = blockIdx.x, d = threadIdx.x;
  const int b = row / Hkv, h = row - b * Hkv;
  const int t = seq_lens[b];                 // position of the new token
  const int PP = part_offsets[b + 1] - part_offsets[b];
  const int p = t / tp;
  if (t < 0 || p >= PP) {                     // no room reserved for this partition
    if (d == 0) spin_raise(status, SPIN_ERR_INVALID);
    return;
  }
  const int32_t slot = spin_walk(dir, leaf_pool, leaf_chunks, row, dir_stride, leaf_entries, t >> 4);
  if (slot < 0 || (int64_t)slot >= pool_slots) {
    if (d == 0) spin_raise(status, SPIN_ERR_NOT_RESIDENT);
    return;
  }
  uint16_t *page = pool + (size_t)slot * (SPIN_SLOT_U4 * 8);
  const uint16_t kb = k_new[(size_t)row * SPIN_HEAD_DIM + d];
  const uint16_t vb = v_new[(size_t)row * SPIN_HEAD_DIM + d];
  page[k_elem(k_token_major, t & 15, d)] = kb;
  page[SPIN_KTILE_U4 * 8 + v_elem(k_token_major, t & 15, d)] = vb;

  const size_t base = (size_t)Hkv * part_offsets[b] + (size_t)h * PP;
  const bool first_in_part = (t == p * tp);
  if (kind == SPIN_SCORE_MINMAX) {
    const size_t R = base + p;
    uint16_t *mx = summ + summ_elem(R, d, 256, 8), *mn = summ + summ_elem(R, 128 + d, 256, 8);
    const float k = spin_bf16_to_f32(kb);
    if (first_in_part) { *mx = kb; *mn = kb; }
    else {
      if (k > spin_bf16_to_f32(*mx)) *mx = kb;
      if (k < spin_bf16_to_f32(*mn)) *mn = kb;
    }
  } else if (kind == SPIN_SCORE_SKETCH) {
    if (d < 16) summ[summ_elem(base + t, d, 16, 4)] = k_new[(size_t)row * SPIN_HEAD_DIM + chan[h * 16 + d]];
  } else {
    // representative of the sub-range the token lands in: mean of its keys so far
    const int sub = tp / reps;
    const int r = (t - p * tp) / sub;
    const int t0 = p * tp + r * sub;
    double acc = (double)spin_bf16_to_f32(kb);
    for (int u = t0; u < t; ++u) {
      const int32_t s2 = spin_walk(dir, leaf_pool, leaf_chunks, row, dir_stride, leaf_entries, u >> 4);
      if (s2 < 0 || (int64_t)s2 >= pool_slots) { spin_raise(status, SPIN_ERR_NOT_RESIDENT); continue; }
      acc += (double)spin_bf16_to_f32(pool[(size_t)s2 * (SPIN_SLOT_U4 * 8) + k_elem(k_token_major, u & 15, d)]);
    }
    const uint16_t m = f64_to_bf16(acc / (double)(t - t0 + 1));
    const size_t R = (base + p) * reps;
    summ[summ_elem(R + r, d, 128, 8)] = m;
    // sub-ranges that hold no token yet repeat representative 0
    if (r == 0)
      for (int r2 = 1; r2 < reps; ++r2) summ[summ_elem(R + r2, d, 128, 8)] = m;
  }
}

extern "C" int spin_append_kv(spin_ctx *ctx, int32_t batch, const void *k_new, const void *v_new,
                              const int32_t *seq_lens, void *kv_pool, int64_t pool_slots, const int32_t *dir,
                              const int32_t *leaf_pool, int64_t leaf_chunks, const int32_t *part_offsets,
                              const int32_t *chan_idx, void *summaries, void *workspace, void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch || pool_slots <= 0 || leaf_chunks <= 0) return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!k_new || !v_new || !seq_lens || !kv_pool || !dir || !leaf_pool || !part_offsets || !summaries)
    return SPIN_ERR_INVALID;
  if (!workspace) return SPIN_ERR_WORKSPACE;
  // the kernel finds the token's partition by division: not with registered partition tables
  if (ctx->var.count) return SPIN_ERR_UNSUPPORTED;
  const spin_config &c = ctx->cfg;
  if (c.score_kind == SPIN_SCORE_SKETCH && (!chan_idx || c.partition_tokens != 1)) return SPIN_ERR_INVALID;
  const int rows = batch * c.num_kv_heads;
  spin_launch(ctx, SPIN_K_APPEND, spin_append_kernel, dim3((unsigned)rows), dim3(128), 0, (hipStream_t)stream,
              (const uint16_t *)k_new, (const uint16_t *)v_new, seq_lens, (uint16_t *)kv_pool, pool_slots, dir,
              leaf_pool, leaf_chunks, part_offsets, chan_idx, (uint16_t *)summaries, c.num_kv_heads,
              c.partition_tokens, c.score_kind, c.reps_per_partition, ctx->dir_stride, c.leaf_entries,
              ctx->k_token_major, (int32_t *)workspace);
  return spin_launch_status();
}
