// Stage 4: paged GQA decode attention over the resolved pages of each row
// (Section 4.1, Attention: standard attention restricted to the selected KV).
//
// One workgroup = one (row, split) pair; its wavefronts are dealt the split's
// pages round-robin.  Per page a wavefront issues eight contiguous 1 KiB loads
// (K tile then V tile of the slot), forms the 16 x 16 logit tile
// S[token][head] = K Q^T with four 16x16x32 bf16 matrix instructions (the
// group's G <= 16 query heads padded to 16 columns), runs the online softmax
// on its four logits per lane, and accumulates O[head][dim] += P V with eight
// 16x16x16 instructions; the logit tile's register layout is exactly the
// operand layout of P, so nothing moves between lanes except two max
// exchanges.  The loads of the next page are issued before the current page is
// consumed (two register buffers), and a wavefront fetches the slot ids and
// masks of all its pages with one load up front, so the only dependent memory
// round trips per wavefront are that one and the first page.
//
// Wavefront partials (m, l, O) are merged through LDS in wave order.  With
// more than one split the workgroup partials go to the workspace and the
// last workgroup of the row to arrive (a ticket counter in the workspace
// header) merges them in split order, so results are reproducible.
#include <mutex>

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

__device__ inline void write_out(uint16_t *__restrict__ out, float *__restrict__ lse, int qhead, int d, float M,
                                 float L, float O) {
  const float r = L > 0.f ? O / L : 0.f;
  out[(size_t)qhead * SPIN_HEAD_DIM + d] = __builtin_bit_cast(uint16_t, (__bf16)r);
  if (lse && d == 0) lse[qhead] = L > 0.f ? (M + __builtin_amdgcn_logf(L)) * 0.6931471805599453f : NEG_INF;
}

// After a workgroup's wavefronts have consumed their tiles: merge the wavefront partials through
// LDS and, with several splits, the workgroup partials through the workspace (see the header).
template <int WAVES>
__device__ __forceinline__ void decode_finish(softmax_state &st, int row, int split, int b, int h, int lane, int wave,
                                              int n, int c, int G, int Hq, int nsplit, float *part_ml, float *part_acc,
                                              int32_t *tickets, uint16_t *__restrict__ out, float *__restrict__ lse) {
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
    if (nsplit == 1) {
      write_out(out, lse, b * Hq + h * G + g, d, M, L, O);
    } else {
      // device-scope stores: written through to where every compute die sees them
      const size_t pi = ((size_t)row * nsplit + split) * G + g;
      spin_dev_store(&part_acc[pi * SPIN_HEAD_DIM + d], O);
      if (d == 0) {
        spin_dev_store(&part_ml[pi * 2 + 0], M);
        spin_dev_store(&part_ml[pi * 2 + 1], L);
      }
    }
  }
  if (nsplit == 1) return;

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
  if (!s_last) return;
  // All loads of the merge are independent of each other: the (m, l) pairs are
  // staged through LDS by one thread each, and every thread issues its
  // accumulator loads eight splits at a time, the first batch before the
  // barrier, so the merge costs about one memory round trip.
  const size_t pbase = (size_t)row * nsplit * G;
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
    write_out(out, lse, b * Hq + h * G + g, d, M, L, O);
  };
#pragma unroll
  for (int k = 0; k < KPRE; ++k) {
    const int idx = threadIdx.x + k * NT;
    if (idx < GD) merge_one(idx, a0[k], true);
  }
  for (int idx = threadIdx.x + KPRE * NT; idx < GD; idx += NT) merge_one(idx, a0[0], false);
  if (threadIdx.x == 0)   // ready for the next launch
    __hip_atomic_store(&tickets[row], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int WAVES, int DEPTH>
__global__ __launch_bounds__(WAVES * 64) void spin_decode_kernel(
    const uint16_t *__restrict__ q, const uint4 *__restrict__ pool, int64_t pool_slots,
    const int32_t *__restrict__ slots, const uint16_t *__restrict__ masks,
    const int32_t *__restrict__ npages, int page_stride, int G, int Hq, int Hkv, int nsplit,
    float scale_log2e, float *part_ml, float *part_acc, int32_t *tickets, uint16_t *__restrict__ out,
    float *__restrict__ lse, int32_t *status) {
  const int row = blockIdx.x / nsplit;
  const int split = blockIdx.x - row * nsplit;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int n = lane & 15;   // column: query head of the group (logits), channel-in-block (output)
  const int c = lane >> 4;   // token quad (logits) / head quad (output)
  const int b = row / Hkv;
  const int h = row - b * Hkv;

  // Pages are dealt round-robin: page p belongs to split p % nsplit and, inside
  // it, to wavefront (p / nsplit) % WAVES.  The addresses of this wavefront's
  // slot entries therefore do not depend on the row's page count, and their
  // load is issued together with it.
  const int32_t *rslots = slots + (size_t)row * page_stride;
  const uint16_t *rmask = masks + (size_t)row * page_stride;
  const int first = wave * nsplit + split, stride = WAVES * nsplit;
  int np = npages[row];
  np = np < 0 ? 0 : (np > page_stride ? page_stride : np);

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

  softmax_state st;
  st.m = NEG_INF;
  st.l = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) st.acc[i] = (spin_f32x4){0.f, 0.f, 0.f, 0.f};

  // this wavefront's pages: first + i * stride, i < nw
  const int nw_max = (page_stride - first + stride - 1) / stride;   // entries that exist in the buffer
  for (int base = 0; base < nw_max; base += 64) {
    int myslot = 0;
    unsigned mymask = 0;
    const int p = first + (base + lane) * stride;
    if (p < page_stride) {
      myslot = rslots[p];
      mymask = rmask[p];
    }
    const int nw = np > first ? (np - first + stride - 1) / stride : 0;
    if (base >= nw) break;
    const int cnt = (nw - base) < 64 ? (nw - base) : 64;
    if (lane < cnt) {
      if (myslot < 0 || (int64_t)myslot >= pool_slots) {
        spin_raise(status, SPIN_ERR_SLOT_RANGE);
        myslot = 0;   // read a valid slot, attend to none of it
        mymask = 0;
      }
    }
    // ring of DEPTH register buffers: DEPTH-1 pages are in flight while one is consumed
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

  decode_finish<WAVES>(st, row, split, b, h, lane, wave, n, c, G, Hq, nsplit, part_ml, part_acc, tickets, out, lse);
}

// ---------------------------------------------------------------------------
// Partitions smaller than a page (token-major slots): most attended pages hold one or two
// attended tokens, so a tile is not a physical page but 16 ATTENDED tokens gathered from
// wherever they live.  A wavefront expands the masks of its pages (dealt round-robin exactly as
// above) into a token list in LDS -- page order, then token order, so the accumulation order is
// fixed -- and then treats every 16 list entries as one tile: lane (n, c) fetches 64 contiguous
// bytes of the key of tile row n per load, and the values of tile rows 4c .. 4c+3 for its 8
// output channels with 2-byte loads that land in the operand layout of P V directly.  Per
// attended token that is the algorithmic 512 bytes (two cache lines of K, two of V) instead of
// the page's 8 KiB, and sixteen times fewer matrix tiles.  Logits, softmax and merge are the
// code of the page kernel.
#define TOK_LIST 1024   // list entries per wavefront and batch of 64 pages

struct tile_src {
  const uint4 *k;           // key row of tile row n (lane % 16), chunk c (lane / 16): + 4 j
  const uint16_t *v[4];     // value rows of tile rows 4c .. 4c+3 at channel n: + 16 jn
};

// Rows past the end of the list repeat its last entry: their loads stay inside attended data, their
// logits are masked and their probabilities are exactly zero.
__device__ inline tile_src tile_source(const uint4 *__restrict__ pool, const uint32_t *tok, int first, int count, int lane) {
  tile_src s;
  const int n = lane & 15, c = lane >> 4;
  const int last = count - 1 - first;                    // >= 0: the tile exists
  const uint32_t e = tok[first + min(n, last)];          // slot * 16 + token
  s.k = pool + (size_t)(e >> 4) * SPIN_SLOT_U4 + (e & 15u) * 16 + c;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t ev = tok[first + min(4 * c + i, last)];
    s.v[i] = (const uint16_t *)(pool + (size_t)(ev >> 4) * SPIN_SLOT_U4 + SPIN_KTILE_U4) + (ev & 15u) * SPIN_HEAD_DIM + n;
  }
  return s;
}

__device__ inline void load_tile(page_regs &r, const tile_src &s) {
#pragma unroll
  for (int j = 0; j < 4; ++j) r.k[j] = spin_nt_load(s.k + 4 * j);
  // operand layout of P V: r.v[jv] = {rows 4c,4c+1 | rows 4c+2,4c+3} for channel block 2jv, then 2jv+1.
  // Each 16-bit load lands in its half of an operand register, so nothing waits for the data
  // before the tile is consumed.
  typedef unsigned short us8 __attribute__((ext_vector_type(8)));
#pragma unroll
  for (int jv = 0; jv < 4; ++jv) {
    us8 w;
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
      for (int i = 0; i < 4; ++i) w[4 * blk + i] = s.v[i][16 * (2 * jv + blk)];
    r.v[jv] = __builtin_bit_cast(uint4, w);
  }
}

template <int WAVES>
__global__ __launch_bounds__(WAVES * 64) void spin_decode_tokens_kernel(
    const uint16_t *__restrict__ q, const uint4 *__restrict__ pool, int64_t pool_slots,
    const int32_t *__restrict__ slots, const uint16_t *__restrict__ masks,
    const int32_t *__restrict__ npages, int page_stride, int G, int Hq, int Hkv, int nsplit,
    float scale_log2e, float *part_ml, float *part_acc, int32_t *tickets, uint16_t *__restrict__ out,
    float *__restrict__ lse, int32_t *status) {
  extern __shared__ float smem[];
  // the token lists live behind the merge buffers of decode_finish
  uint32_t *tok = (uint32_t *)(smem + WAVES * G * (SPIN_HEAD_DIM + 2)) + (threadIdx.x >> 6) * TOK_LIST;

  const int row = blockIdx.x / nsplit;
  const int split = blockIdx.x - row * nsplit;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int n = lane & 15, c = lane >> 4;
  const int b = row / Hkv;
  const int h = row - b * Hkv;
  const int32_t *rslots = slots + (size_t)row * page_stride;
  const uint16_t *rmask = masks + (size_t)row * page_stride;
  const int first = wave * nsplit + split, stride = WAVES * nsplit;
  int np = npages[row];
  np = np < 0 ? 0 : (np > page_stride ? page_stride : np);

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
  softmax_state st;
  st.m = NEG_INF;
  st.l = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) st.acc[i] = (spin_f32x4){0.f, 0.f, 0.f, 0.f};

  const int nw_max = (page_stride - first + stride - 1) / stride;
  for (int base = 0; base < nw_max; base += 64) {
    int myslot = 0;
    unsigned mymask = 0;
    const int p = first + (base + lane) * stride;
    if (p < page_stride) {
      myslot = rslots[p];
      mymask = rmask[p];
    }
    const int nw = np > first ? (np - first + stride - 1) / stride : 0;
    if (base >= nw) break;
    const int cnt = (nw - base) < 64 ? (nw - base) : 64;
    if (lane >= cnt) mymask = 0;
    else if (myslot < 0 || (int64_t)myslot >= pool_slots) {
      spin_raise(status, SPIN_ERR_SLOT_RANGE);
      myslot = 0;
      mymask = 0;
    }
    // token list of this batch of pages: page order, then token order
    const int mine = __popc(mymask);
    const int incl = spin_wave_inclusive_scan(mine);
    const int total = __builtin_amdgcn_readlane(incl, 63);
    {
      int pos = incl - mine;
      unsigned m = mymask;
      while (m) {
        const int t = __ffs(m) - 1;
        m &= m - 1;
        tok[pos++] = ((uint32_t)myslot << 4) | (uint32_t)t;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the wavefront reads its own list: program order
    // two register buffers: the next tile's loads are issued before the current one is consumed
    page_regs r[2];
    const int ntiles = (total + 15) >> 4;
    if (ntiles > 0) load_tile(r[0], tile_source(pool, tok, 0, total, lane));
    for (int k = 0; k < ntiles; k += 2) {
      if (k + 1 < ntiles) load_tile(r[1], tile_source(pool, tok, 16 * (k + 1), total, lane));
      const int left0 = total - 16 * k;
      consume_page(st, r[0], qf, left0 >= 16 ? 0xffffu : ((1u << left0) - 1u), c, scale_log2e);
      if (k + 2 < ntiles) load_tile(r[0], tile_source(pool, tok, 16 * (k + 2), total, lane));
      if (k + 1 < ntiles) {
        const int left1 = total - 16 * (k + 1);
        consume_page(st, r[1], qf, left1 >= 16 ? 0xffffu : ((1u << left1) - 1u), c, scale_log2e);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // before the next batch overwrites the list
  }
  __syncthreads();   // the merge buffers are separate from the lists, but keep the phases apart
  decode_finish<WAVES>(st, row, split, b, h, lane, wave, n, c, G, Hq, nsplit, part_ml, part_acc, tickets, out, lse);
}

// Host side of stage 4: checks, then the launch; the split-K scratch (row tickets, (m, l) pairs and
// accumulators of the workgroup partials) and the status word are handed in by the two entry points.
static int decode_launch(spin_ctx *ctx, int32_t batch, const void *q, const void *kv_pool, int64_t pool_slots,
                         const int32_t *slots, const uint16_t *valid_mask, const int32_t *npages, void *out,
                         float *lse, float *part_ml, float *part_acc, int32_t *tickets, int32_t *status,
                         void *stream) {
  const int rows = batch * ctx->cfg.num_kv_heads;
  const int G = ctx->group, nsplit = ctx->splits;
  const float scale_log2e = ctx->scale * 1.4426950408889634f;
  const int W = ctx->waves;
  const size_t lds = (size_t)W * G * (SPIN_HEAD_DIM + 2) * sizeof(float);
  if (ctx->k_token_major) {
    // token-major slots: tiles of gathered tokens (always 8 wavefronts: the waves and depth knobs do not
    // apply, and the merge buffers are sized for 8 whatever the waves knob says)
    const size_t lds_tok = (size_t)8 * G * (SPIN_HEAD_DIM + 2) * sizeof(float) + (size_t)8 * TOK_LIST * sizeof(uint32_t);
    spin_launch(ctx, SPIN_K_DECODE, spin_decode_tokens_kernel<8>, dim3((unsigned)(rows * nsplit)), dim3(512), lds_tok,
                (hipStream_t)stream, (const uint16_t *)q, (const uint4 *)kv_pool, pool_slots, slots, valid_mask, npages,
                ctx->page_stride, G, ctx->cfg.num_q_heads, ctx->cfg.num_kv_heads, nsplit, scale_log2e, part_ml,
                part_acc, tickets, (uint16_t *)out, lse, status);
    return spin_launch_status();
  }
#define SPIN_DECODE_LAUNCH2(WV, DP)                                                                              \
  spin_launch(ctx, SPIN_K_DECODE, spin_decode_kernel<WV, DP>, dim3((unsigned)(rows * nsplit)), dim3(WV * 64), lds, \
              (hipStream_t)stream, (const uint16_t *)q, (const uint4 *)kv_pool, pool_slots, slots, valid_mask,   \
              npages, ctx->page_stride, G, ctx->cfg.num_q_heads, ctx->cfg.num_kv_heads, nsplit, scale_log2e,     \
              part_ml, part_acc, tickets, (uint16_t *)out, lse, status)
#define SPIN_DECODE_LAUNCH(WV)                          \
  do {                                                  \
    if (ctx->depth == 2) SPIN_DECODE_LAUNCH2(WV, 2);    \
    else if (ctx->depth == 4) SPIN_DECODE_LAUNCH2(WV, 4); \
    else SPIN_DECODE_LAUNCH2(WV, 3);                    \
  } while (0)
  if (W == 2) SPIN_DECODE_LAUNCH(2);
  else if (W == 8) SPIN_DECODE_LAUNCH(8);
  else SPIN_DECODE_LAUNCH(4);
#undef SPIN_DECODE_LAUNCH
#undef SPIN_DECODE_LAUNCH2
  return spin_launch_status();
}

extern "C" int spin_sparse_decode(spin_ctx *ctx, int32_t batch, const void *q, const void *kv_pool,
                                  int64_t pool_slots, const int32_t *slots, const uint16_t *valid_mask,
                                  const int32_t *npages, void *out, float *lse, void *workspace,
                                  void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch || pool_slots <= 0) return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!q || !kv_pool || !slots || !valid_mask || !npages || !out) return SPIN_ERR_INVALID;
  if (!workspace) return SPIN_ERR_WORKSPACE;
  char *ws = (char *)workspace;
  return decode_launch(ctx, batch, q, kv_pool, pool_slots, slots, valid_mask, npages, out, lse,
                       (float *)(ws + ctx->ws_ml_off), (float *)(ws + ctx->ws_acc_off),
                       (int32_t *)(ws + ctx->ws_ticket_off), (int32_t *)workspace, stream);
}

// ---------------------------------------------------------------------------
// Stage 4 for callers that cannot hand over (or allocate) a workspace: the split-K scratch lives in
// a device array of the library itself.  Every GPU the library runs on holds its own copy of the
// array, at its own address, until the process ends.
#define SPIN_STATIC_SCRATCH_DEVICES 64
static __device__ __align__(256) unsigned char scratch[SPIN_STATIC_SCRATCH_BYTES];

// `scratch` above is only a host-side handle in host code: the device address is asked for once per
// device (with that device current) and kept; host code uses that address and never the symbol's name.
static void *g_scratch_ptr[SPIN_STATIC_SCRATCH_DEVICES];
static std::mutex g_scratch_mutex;

static int static_scratch(void **ptr) {
  int dev = -1;
  SPIN_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= SPIN_STATIC_SCRATCH_DEVICES) return SPIN_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    SPIN_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return SPIN_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return SPIN_OK;
}

// clears the words that must be zero when the attention kernel starts (a kernel, not a memset, so
// that a caller may record the call into a HIP graph)
__global__ void spin_static_clear_kernel(int32_t *p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

extern "C" int spin_sparse_decode_static(spin_ctx *ctx, int32_t batch, const void *q, const void *kv_pool,
                                         int64_t pool_slots, const int32_t *slots, const uint16_t *valid_mask,
                                         const int32_t *npages, void *out, float *lse, int32_t *status,
                                         void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch || pool_slots <= 0) return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!q || !kv_pool || !slots || !valid_mask || !npages || !out) return SPIN_ERR_INVALID;
  // layout inside the array, sized for this call's rows: [status word, 256 B][tickets][(m, l)][accumulators]
  const size_t rows = (size_t)batch * ctx->cfg.num_kv_heads;
  const size_t partials = rows * ctx->splits * ctx->group;
  const size_t ticket_off = SPIN_WS_HEADER;
  const size_t ml_off = (ticket_off + rows * sizeof(int32_t) + 255) & ~(size_t)255;
  const size_t acc_off = (ml_off + partials * 2 * sizeof(float) + 255) & ~(size_t)255;
  const size_t need = acc_off + partials * SPIN_HEAD_DIM * sizeof(float);
  if (need > SPIN_STATIC_SCRATCH_BYTES) return SPIN_ERR_STATIC_LIMIT;
  void *base = nullptr;
  const int rc = static_scratch(&base);
  if (rc != SPIN_OK) return rc;
  char *sc = (char *)base;
  // the array keeps the last call's contents: the status word and the row tickets start at zero
  const int nclear = (int)(ml_off / sizeof(int32_t));
  hipLaunchKernelGGL(spin_static_clear_kernel, dim3((nclear + 255) / 256), dim3(256), 0, (hipStream_t)stream,
                     (int32_t *)sc, nclear);
  if (hipGetLastError() != hipSuccess) return SPIN_ERR_HIP;
  return decode_launch(ctx, batch, q, kv_pool, pool_slots, slots, valid_mask, npages, out, lse,
                       (float *)(sc + ml_off), (float *)(sc + acc_off), (int32_t *)(sc + ticket_off),
                       status ? status : (int32_t *)sc, stream);
}
