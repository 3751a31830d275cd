// Device code of stage 4 shared by the attention kernels and by the launch that attends a row's
// always-attended pages beside stages 2+3: page loads, the logit / softmax / P V step of one
// 16-token tile on the matrix cores, and the merge of wavefront and workgroup partials.
#pragma once
#include "spin_common.h"

#define NEG_INF (-__builtin_inff())

struct page_regs {
  uint4 k[4], v[4];
};

// Loads of a page.  A page whose mask is not full (token partitions, the ragged last page) only
// fetches what its attended tokens need: in the K tile a lane holds 16 bytes of ONE token, in
// the V tile 16 bytes of ONE token quad, so lanes of unattended tokens / quads issue no load
// and hold zeros (their logits are masked and their probabilities are exactly zero, so the
// result has the same bits as with the whole page loaded).
__device__ inline void load_page(page_regs &r, const uint4 *__restrict__ pool, int slot, int lane, unsigned mask) {
  const uint4 *kp = pool + (size_t)slot * SPIN_SLOT_U4 + lane;
  if (mask == 0xffffu) {
#pragma unroll
    for (int j = 0; j < 4; ++j) r.k[j] = spin_nt_load(kp + j * 64);
#pragma unroll
    for (int j = 0; j < 4; ++j) r.v[j] = spin_nt_load(kp + SPIN_KTILE_U4 + j * 64);
  } else {
    const bool kneed = (mask >> (lane & 15)) & 1u;
    const bool vneed = ((mask >> (4 * (lane >> 4))) & 0xfu) != 0u;
#pragma unroll
    for (int j = 0; j < 4; ++j) r.k[j] = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int j = 0; j < 4; ++j) r.v[j] = make_uint4(0, 0, 0, 0);
    if (kneed) {
#pragma unroll
      for (int j = 0; j < 4; ++j) r.k[j] = spin_nt_load(kp + j * 64);
    }
    if (vneed) {
#pragma unroll
      for (int j = 0; j < 4; ++j) r.v[j] = spin_nt_load(kp + SPIN_KTILE_U4 + j * 64);
    }
  }
}

struct softmax_state {
  float m, l;
  spin_f32x4 acc[8];
};

__device__ inline void consume_page(softmax_state &st, const page_regs &r, const spin_bf16x8 (&qf)[4],
                                    unsigned mask, int c, float scale_log2e) {
  // S[token 4c+i][head n]
  spin_f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int j = 0; j < 4; ++j)
    s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(spin_bf16x8, r.k[j]), qf[j], s, 0, 0, 0);

  const unsigned mbits = (mask >> (4 * c)) & 0xFu;
  float sv[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) sv[i] = ((mbits >> i) & 1u) ? s[i] * scale_log2e : NEG_INF;
  float pm = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
  pm = fmaxf(pm, __shfl_xor(pm, 16));
  pm = fmaxf(pm, __shfl_xor(pm, 32));
  const float m_new = fmaxf(st.m, pm);
  const float m_safe = (m_new == NEG_INF) ? 0.f : m_new;
  const float alpha = __builtin_amdgcn_exp2f(st.m - m_safe);
  float pr[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) pr[i] = __builtin_amdgcn_exp2f(sv[i] - m_safe);
  st.l = st.l * alpha + ((pr[0] + pr[1]) + (pr[2] + pr[3]));
  st.m = m_new;

  // rescale the accumulator rows (head 4c+i) by that head's alpha, only when some maximum moved
  if (__any(alpha != 1.0f)) {
    float ar[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) ar[i] = __shfl(alpha, 4 * c + i);
#pragma unroll
    for (int jn = 0; jn < 8; ++jn)
#pragma unroll
      for (int i = 0; i < 4; ++i) st.acc[jn][i] *= ar[i];
  }

  // P as the A operand: row n = head, k = tokens 4c..4c+3
  spin_bf16x2 p01 = {(__bf16)pr[0], (__bf16)pr[1]};
  spin_bf16x2 p23 = {(__bf16)pr[2], (__bf16)pr[3]};
  uint2 pk = {__builtin_bit_cast(uint32_t, p01), __builtin_bit_cast(uint32_t, p23)};
  const spin_s16x4 pa = __builtin_bit_cast(spin_s16x4, pk);
#pragma unroll
  for (int jv = 0; jv < 4; ++jv) {
    uint2 lo = {r.v[jv].x, r.v[jv].y}, hi = {r.v[jv].z, r.v[jv].w};
    st.acc[2 * jv] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pa, __builtin_bit_cast(spin_s16x4, lo),
                                                               st.acc[2 * jv], 0, 0, 0);
    st.acc[2 * jv + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pa, __builtin_bit_cast(spin_s16x4, hi),
                                                                   st.acc[2 * jv + 1], 0, 0, 0);
  }
}

// Attends `cnt` (<= 64) pages whose slot and mask are held one per lane (lane i: the i-th page), in
// lane order, through a ring of DEPTH register buffers: DEPTH-1 pages are in flight while one is consumed.
template <int DEPTH>
__device__ __forceinline__ void attend_lane_pages(softmax_state &st, const uint4 *__restrict__ pool, int myslot,
                                                  unsigned mymask, int cnt, int lane, int c,
                                                  const spin_bf16x8 (&qf)[4], float scale_log2e) {
  page_regs r[DEPTH];
#pragma unroll
  for (int d = 0; d < DEPTH - 1; ++d)
    if (d < cnt) load_page(r[d], pool, __builtin_amdgcn_readlane(myslot, d), lane,
                           (unsigned)__builtin_amdgcn_readlane((int)mymask, d));
  for (int i = 0; i < cnt; i += DEPTH) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      const int ahead = i + d + DEPTH - 1;
      if (ahead < cnt) load_page(r[(d + DEPTH - 1) % DEPTH], pool, __builtin_amdgcn_readlane(myslot, ahead), lane,
                                 (unsigned)__builtin_amdgcn_readlane((int)mymask, ahead));
      if (i + d < cnt)
        consume_page(st, r[d], qf, (unsigned)__builtin_amdgcn_readlane((int)mymask, i + d), c, scale_log2e);
    }
  }
}

// the group's queries as the second matrix operand of the logit tile: column n = head, k = channels 32j+8c..+8
__device__ __forceinline__ void load_queries(spin_bf16x8 (&qf)[4], const uint16_t *__restrict__ q, int b, int h, int G,
                                             int Hq, int n, int c) {
  const uint4 *qrow = (const uint4 *)(q + ((size_t)(b * Hq + h * G + (n < G ? n : 0))) * SPIN_HEAD_DIM);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    uint4 v = qrow[j * 4 + c];
    if (n >= G) v = make_uint4(0, 0, 0, 0);
    qf[j] = __builtin_bit_cast(spin_bf16x8, v);
  }
}

__device__ inline void softmax_reset(softmax_state &st) {
  st.m = NEG_INF;
  st.l = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) st.acc[i] = (spin_f32x4){0.f, 0.f, 0.f, 0.f};
}

__device__ inline void write_out(uint16_t *__restrict__ out, float *__restrict__ lse, int qhead, int d, float M,
                                 float L, float O) {
  const float r = L > 0.f ? O / L : 0.f;
  out[(size_t)qhead * SPIN_HEAD_DIM + d] = __builtin_bit_cast(uint16_t, (__bf16)r);
  if (lse && d == 0) lse[qhead] = L > 0.f ? (M + __builtin_amdgcn_logf(L)) * 0.6931471805599453f : NEG_INF;
}

// After a workgroup's wavefronts have consumed their tiles: merge the wavefront partials through
// LDS and, with several splits, the workgroup partials through the workspace (see the header).
// Partial `s` of a row lives at index row * pstride + s (pstride = splits + the partials earlier launches may leave); the row's output is
// the merge, in index order, of the partials 0 .. nsplit-1 of the calling launch.
// ONLY_PARTIAL (then `split` is the index j of the calling workgroup among those that attend a row's
// always-attended pages): the workgroup only stores its partial, at index nsplit + j, for a later
// launch on the same stream to start from.
// to_partial: the merged result of the row is stored there as well, unnormalised, instead of being
// written to `out` (the first of two attention passes over one page list).
// Returns true in the workgroup that wrote the row's output.
template <int WAVES, bool ONLY_PARTIAL = false>
__device__ __forceinline__ bool decode_finish(softmax_state &st, int row, int split, int b, int h, int lane, int wave,
                                              int n, int c, int G, int Hq, int nsplit, int pstride,
                                              float *part_ml, float *part_acc, int32_t *tickets,
                                              uint16_t *__restrict__ out, float *__restrict__ lse,
                                              bool to_partial = false) {
  extern __shared__ float smem[];
  float *s_acc = smem;                                  // [WAVES][G][128]
  float *s_m = smem + WAVES * G * SPIN_HEAD_DIM;        // [WAVES][G]
  float *s_l = s_m + WAVES * G;                         // [WAVES][G]
  __shared__ int s_last;
  // denominators: sum the four token-quad lanes of each head
  float l = st.l;
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);

  // wavefront partials -> LDS
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int head = 4 * c + i;
    if (head < G) {
#pragma unroll
      for (int jn = 0; jn < 8; ++jn) s_acc[(wave * G + head) * SPIN_HEAD_DIM + 16 * jn + n] = st.acc[jn][i];
    }
  }
  if (c == 0 && n < G) {
    s_m[wave * G + n] = st.m;
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
    if (ONLY_PARTIAL || (nsplit == 1 && to_partial)) {
      // read by a later launch on the same stream: plain stores
      const size_t pi = ((size_t)row * pstride + nsplit + (ONLY_PARTIAL ? split : 0)) * G + g;
      part_acc[pi * SPIN_HEAD_DIM + d] = O;
      if (d == 0) {
        part_ml[pi * 2 + 0] = M;
        part_ml[pi * 2 + 1] = L;
      }
    } else if (nsplit == 1) {
      write_out(out, lse, b * Hq + h * G + g, d, M, L, O);
    } else {
      // device-scope stores: written through to where every compute die sees them
      const size_t pi = ((size_t)row * pstride + split) * G + g;
      spin_dev_store(&part_acc[pi * SPIN_HEAD_DIM + d], O);
      if (d == 0) {
        spin_dev_store(&part_ml[pi * 2 + 0], M);
        spin_dev_store(&part_ml[pi * 2 + 1], L);
      }
    }
  }
  if (ONLY_PARTIAL) return false;
  if (nsplit == 1) return true;

  // Ticket: the last workgroup of the row to arrive merges all splits in split
  // order.  Partials travel through device-scope atomic stores and loads (no
  // cache-wide write-back or invalidate); each thread waits for its own stores
  // to be acknowledged, the barrier orders them before thread 0's ticket.
  __builtin_amdgcn_s_waitcnt(0);
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __syncthreads();
  if (threadIdx.x == 0)
    s_last = (__hip_atomic_fetch_add(&tickets[row], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == nsplit - 1);
  __syncthreads();
  if (!s_last) return false;
  // All loads of the merge are independent of each other: the (m, l) pairs are
  // staged through LDS by one thread each, and every thread issues its
  // accumulator loads eight splits at a time, the first batch before the
  // barrier, so the merge costs about one memory round trip.
  const size_t pbase = (size_t)row * pstride * G;
  float *t_m = s_acc, *t_l = s_acc + nsplit * G;   // s_acc is free: the wave partials were consumed above
  constexpr int CH = 8;        // splits whose accumulators a thread requests at a time
  constexpr int KPRE = 4;      // output elements per thread requested before the barrier (groups of up to
                               // 16 heads with 8 wavefronts; further ones are requested in the loop)
  constexpr int NT = WAVES * 64;
  const int GD = G * SPIN_HEAD_DIM;
  float a0[KPRE][CH];
#pragma unroll
  for (int k = 0; k < KPRE; ++k) {
    const int idx = threadIdx.x + k * NT;
    const int g = idx >> 7, d = idx & 127;
#pragma unroll
    for (int s = 0; s < CH; ++s)
      a0[k][s] = (idx < GD && s < nsplit) ? spin_dev_load(&part_acc[(pbase + (size_t)s * G + g) * SPIN_HEAD_DIM + d]) : 0.f;
  }
  for (int i = threadIdx.x; i < nsplit * G; i += NT) {
    t_m[i] = spin_dev_load(&part_ml[(pbase + i) * 2]);
    t_l[i] = spin_dev_load(&part_ml[(pbase + i) * 2 + 1]);
  }
  __syncthreads();
  // output element idx = (head g, channel d): the splits merged in split order
  auto merge_one = [&](int idx, const float (&first)[CH], bool have_first) {
    const int g = idx >> 7, d = idx & 127;
    float M = NEG_INF;
    for (int s = 0; s < nsplit; ++s) M = fmaxf(M, t_m[s * G + g]);
    const float Ms = (M == NEG_INF) ? 0.f : M;
    float L = 0.f, O = 0.f;
    for (int s0 = 0; s0 < nsplit; s0 += CH) {
      float a[CH];
#pragma unroll
      for (int s = 0; s < CH; ++s) {
        if (have_first && s0 == 0) a[s] = first[s];
        else a[s] = (s0 + s < nsplit) ? spin_dev_load(&part_acc[(pbase + (size_t)(s0 + s) * G + g) * SPIN_HEAD_DIM + d]) : 0.f;
      }
#pragma unroll
      for (int s = 0; s < CH; ++s) {
        if (s0 + s < nsplit) {
          const float wgt = __builtin_amdgcn_exp2f(t_m[(s0 + s) * G + g] - Ms);
          L += t_l[(s0 + s) * G + g] * wgt;
          O += a[s] * wgt;
        }
      }
    }
    if (to_partial) {
      const size_t pi = ((size_t)row * pstride + nsplit) * G + g;
      part_acc[pi * SPIN_HEAD_DIM + d] = O;
      if (d == 0) {
        part_ml[pi * 2 + 0] = M;
        part_ml[pi * 2 + 1] = L;
      }
    } else {
      write_out(out, lse, b * Hq + h * G + g, d, M, L, O);
    }
  };
#pragma unroll
  for (int k = 0; k < KPRE; ++k) {
    const int idx = threadIdx.x + k * NT;
    if (idx < GD) merge_one(idx, a0[k], true);
  }
  for (int idx = threadIdx.x + KPRE * NT; idx < GD; idx += NT) merge_one(idx, a0[0], false);
  if (threadIdx.x == 0)   // ready for the next launch
    __hip_atomic_store(&tickets[row], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return true;
}

