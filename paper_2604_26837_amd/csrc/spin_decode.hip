// Stage 4: paged GQA decode attention over the resolved pages of each row
// (Section 4.1, Attention: standard attention restricted to the selected KV).
//
// One workgroup = one (row, split) pair; its four wavefronts walk the split's
// pages round-robin.  Per page a wavefront issues eight contiguous 1 KiB loads
// (K tile then V tile of the slot), forms the 16 x 16 logit tile
// S[token][head] = K Q^T with four 16x16x32 bf16 matrix instructions (the
// group's G <= 16 query heads padded to 16 columns), runs the online softmax
// on its four logits per lane, and accumulates O[head][dim] += P V with eight
// 16x16x16 instructions; the logit tile's register layout is exactly the
// operand layout of P, so nothing moves between lanes except two max
// exchanges.  Wavefront partials (m, l, O) are merged through LDS in wave
// order; with more than one split the workgroup partials go to the workspace
// and a second kernel merges them in split order, so results are reproducible.
#include "spin_common.h"

#define NEG_INF (-__builtin_inff())

template <int WAVES>
__global__ __launch_bounds__(WAVES * 64) void spin_decode_kernel(
    const uint16_t *__restrict__ q, const uint4 *__restrict__ pool, int64_t pool_slots,
    const int32_t *__restrict__ slots, const uint16_t *__restrict__ masks,
    const int32_t *__restrict__ npages, int page_stride, int G, int Hq, int Hkv, int nsplit,
    float scale_log2e, float *__restrict__ part_ml, float *__restrict__ part_acc,
    uint16_t *__restrict__ out, float *__restrict__ lse, int32_t *status) {
  extern __shared__ float smem[];
  float *s_acc = smem;                                  // [WAVES][G][128]
  float *s_m = smem + WAVES * G * SPIN_HEAD_DIM;        // [WAVES][G]
  float *s_l = s_m + WAVES * G;                         // [WAVES][G]

  const int row = blockIdx.x / nsplit;
  const int split = blockIdx.x - row * nsplit;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int n = lane & 15;   // column: query head of the group (logits), channel-in-block (output)
  const int c = lane >> 4;   // token quad (logits) / head quad (output)
  const int b = row / Hkv;
  const int h = row - b * Hkv;

  int np = npages[row];
  np = np < 0 ? 0 : (np > page_stride ? page_stride : np);
  const int per = (np + nsplit - 1) / nsplit;
  const int p0 = split * per;
  const int p1 = (p0 + per) < np ? (p0 + per) : np;

  // the group's queries as the B operand: column n = head, k = channels 32j+8c..+8
  spin_bf16x8 qf[4];
  {
    const uint4 *qrow = (const uint4 *)(q + ((size_t)(b * Hq + h * G + (n < G ? n : 0))) * SPIN_HEAD_DIM);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      uint4 v = qrow[j * 4 + c];
      if (n >= G) v = make_uint4(0, 0, 0, 0);
      qf[j] = __builtin_bit_cast(spin_bf16x8, v);
    }
  }

  float m = NEG_INF, l = 0.f;
  spin_f32x4 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = (spin_f32x4){0.f, 0.f, 0.f, 0.f};

  const int32_t *rslots = slots + (size_t)row * page_stride;
  const uint16_t *rmask = masks + (size_t)row * page_stride;

  for (int p = p0 + wave; p < p1; p += WAVES) {
    const int slot = __builtin_amdgcn_readfirstlane(rslots[p]);
    const unsigned mask = (unsigned)__builtin_amdgcn_readfirstlane((int)rmask[p]);
    if (slot < 0 || (int64_t)slot >= pool_slots) {
      if (lane == 0) spin_raise(status, SPIN_ERR_SLOT_RANGE);
      continue;
    }
    const uint4 *kp = pool + (size_t)slot * SPIN_SLOT_U4;
    uint4 kv[4], vv[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) kv[j] = kp[j * 64 + lane];
#pragma unroll
    for (int j = 0; j < 4; ++j) vv[j] = kp[SPIN_KTILE_U4 + j * 64 + lane];

    // S[token 4c+i][head n]
    spin_f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 4; ++j)
      s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(spin_bf16x8, kv[j]), qf[j], s, 0, 0, 0);

    const unsigned mbits = (mask >> (4 * c)) & 0xFu;
    float sv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) sv[i] = ((mbits >> i) & 1u) ? s[i] * scale_log2e : NEG_INF;
    float pm = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
    pm = fmaxf(pm, __shfl_xor(pm, 16));
    pm = fmaxf(pm, __shfl_xor(pm, 32));
    const float m_new = fmaxf(m, pm);
    const float m_safe = (m_new == NEG_INF) ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m - m_safe);
    float pr[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) pr[i] = __builtin_amdgcn_exp2f(sv[i] - m_safe);
    l = l * alpha + ((pr[0] + pr[1]) + (pr[2] + pr[3]));
    m = m_new;

    // rescale the accumulator rows (head 4c+i) by that head's alpha
    float ar[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) ar[i] = __shfl(alpha, 4 * c + i);
#pragma unroll
    for (int jn = 0; jn < 8; ++jn)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[jn][i] *= ar[i];

    // P as the A operand: row n = head, k = tokens 4c..4c+3
    spin_bf16x2 p01 = {(__bf16)pr[0], (__bf16)pr[1]};
    spin_bf16x2 p23 = {(__bf16)pr[2], (__bf16)pr[3]};
    uint2 pk = {__builtin_bit_cast(uint32_t, p01), __builtin_bit_cast(uint32_t, p23)};
    const spin_s16x4 pa = __builtin_bit_cast(spin_s16x4, pk);
#pragma unroll
    for (int jv = 0; jv < 4; ++jv) {
      uint2 lo = {vv[jv].x, vv[jv].y}, hi = {vv[jv].z, vv[jv].w};
      acc[2 * jv] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pa, __builtin_bit_cast(spin_s16x4, lo),
                                                              acc[2 * jv], 0, 0, 0);
      acc[2 * jv + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pa, __builtin_bit_cast(spin_s16x4, hi),
                                                                  acc[2 * jv + 1], 0, 0, 0);
    }
  }

  // denominators: sum the four token-quad lanes of each head
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);

  // wavefront partials -> LDS
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int head = 4 * c + i;
    if (head < G) {
#pragma unroll
      for (int jn = 0; jn < 8; ++jn) s_acc[(wave * G + head) * SPIN_HEAD_DIM + 16 * jn + n] = acc[jn][i];
    }
  }
  if (c == 0 && n < G) {
    s_m[wave * G + n] = m;
    s_l[wave * G + n] = l;
  }
  __syncthreads();

  for (int idx = threadIdx.x; idx < G * SPIN_HEAD_DIM; idx += WAVES * 64) {
    const int g = idx >> 7, d = idx & 127;
    float M = NEG_INF;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) M = fmaxf(M, s_m[w * G + g]);
    const float Ms = (M == NEG_INF) ? 0.f : M;
    float L = 0.f, O = 0.f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      const float wgt = __builtin_amdgcn_exp2f(s_m[w * G + g] - Ms);
      L += s_l[w * G + g] * wgt;
      O += s_acc[(w * G + g) * SPIN_HEAD_DIM + d] * wgt;
    }
    if (nsplit == 1) {
      const size_t o = ((size_t)(b * Hq + h * G + g)) * SPIN_HEAD_DIM + d;
      const float r = L > 0.f ? O / L : 0.f;
      out[o] = __builtin_bit_cast(uint16_t, (__bf16)r);
      if (lse && d == 0)
        lse[b * Hq + h * G + g] = L > 0.f ? (M + __builtin_amdgcn_logf(L)) * 0.6931471805599453f : NEG_INF;
    } else {
      const size_t pi = ((size_t)row * nsplit + split) * G + g;
      part_acc[pi * SPIN_HEAD_DIM + d] = O;
      if (d == 0) {
        part_ml[pi * 2 + 0] = M;
        part_ml[pi * 2 + 1] = L;
      }
    }
  }
}

// merge the split partials of one row in split order
__global__ __launch_bounds__(256) void spin_decode_merge_kernel(const float *__restrict__ part_ml,
                                                                const float *__restrict__ part_acc, int G,
                                                                int Hq, int Hkv, int nsplit,
                                                                uint16_t *__restrict__ out,
                                                                float *__restrict__ lse) {
  const int row = blockIdx.x;
  const int b = row / Hkv, h = row - b * Hkv;
  for (int idx = threadIdx.x; idx < G * SPIN_HEAD_DIM; idx += 256) {
    const int g = idx >> 7, d = idx & 127;
    const size_t base = (size_t)row * nsplit * G;
    float M = NEG_INF;
    for (int s = 0; s < nsplit; ++s) M = fmaxf(M, part_ml[(base + (size_t)s * G + g) * 2]);
    const float Ms = (M == NEG_INF) ? 0.f : M;
    float L = 0.f, O = 0.f;
    for (int s = 0; s < nsplit; ++s) {
      const size_t pi = base + (size_t)s * G + g;
      const float wgt = __builtin_amdgcn_exp2f(part_ml[pi * 2] - Ms);
      L += part_ml[pi * 2 + 1] * wgt;
      O += part_acc[pi * SPIN_HEAD_DIM + d] * wgt;
    }
    const size_t o = ((size_t)(b * Hq + h * G + g)) * SPIN_HEAD_DIM + d;
    const float r = L > 0.f ? O / L : 0.f;
    out[o] = __builtin_bit_cast(uint16_t, (__bf16)r);
    if (lse && d == 0)
      lse[b * Hq + h * G + g] = L > 0.f ? (M + __builtin_amdgcn_logf(L)) * 0.6931471805599453f : NEG_INF;
  }
}

extern "C" int spin_sparse_decode(spin_ctx *ctx, int32_t batch, const void *q, const void *kv_pool,
                                  int64_t pool_slots, const int32_t *slots, const uint16_t *valid_mask,
                                  const int32_t *npages, void *out, float *lse, void *workspace,
                                  void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch || pool_slots <= 0) return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!q || !kv_pool || !slots || !valid_mask || !npages || !out) return SPIN_ERR_INVALID;
  if (!workspace) return SPIN_ERR_WORKSPACE;
  const int rows = batch * ctx->cfg.num_kv_heads;
  const int G = ctx->group, nsplit = ctx->splits;
  char *ws = (char *)workspace;
  float *part_ml = (float *)(ws + ctx->ws_ml_off);
  float *part_acc = (float *)(ws + ctx->ws_acc_off);
  const float scale_log2e = ctx->scale * 1.4426950408889634f;
  const size_t lds = (size_t)SPIN_DECODE_WAVES * G * (SPIN_HEAD_DIM + 2) * sizeof(float);
  hipStream_t st = (hipStream_t)stream;
  spin_launch(ctx, SPIN_K_DECODE, spin_decode_kernel<SPIN_DECODE_WAVES>, dim3((unsigned)(rows * nsplit)),
              dim3(SPIN_DECODE_WAVES * 64), lds, st, (const uint16_t *)q, (const uint4 *)kv_pool,
                     pool_slots, slots, valid_mask, npages, ctx->page_stride, G, ctx->cfg.num_q_heads,
                     ctx->cfg.num_kv_heads, nsplit, scale_log2e, part_ml, part_acc, (uint16_t *)out, lse,
                     (int32_t *)workspace);
  if (nsplit > 1)
    spin_launch(ctx, SPIN_K_MERGE, spin_decode_merge_kernel, dim3((unsigned)rows), dim3(256), 0, st, part_ml, part_acc, G,
                       ctx->cfg.num_q_heads, ctx->cfg.num_kv_heads, nsplit, (uint16_t *)out, lse);
  return spin_launch_status();
}
