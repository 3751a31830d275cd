// Stage 2: per row, forced partitions plus the k' best-scoring candidates
// (Table 1, "-> topk"; Section 4.2: the always-attended windows are filtered
// out of the candidates).
//
// One workgroup per row.  Scores become order-preserving 32-bit keys (NaN ->
// -inf, -0 -> +0); an MSB-first radix select (four 8-bit passes, LDS
// histogram, parallel suffix scan) finds the key T of the k'-th best
// candidate; then one index-ordered compaction emits every forced partition,
// every candidate with key > T and the lowest-index candidates with key == T
// that are still needed.  Because emission is in index order the output is
// ascending and ties go to the lower id without any sort.
#include "spin_select_dev.h"

#define SEL_BLOCK 512
#define SEL_WAVES (SEL_BLOCK / 64)

// exclusive prefix sum of one int per thread over the workgroup, plus the total
__device__ inline int block_exclusive_scan(int v, int *s_wave, int &total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int o = __shfl_up(inc, d);
    if (lane >= d) inc += o;
  }
  __syncthreads();  // s_wave may still be read from a previous scan
  if (lane == 63) s_wave[wave] = inc;
  __syncthreads();
  int off = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < SEL_WAVES; ++w) {
    const int x = s_wave[w];
    if (w < wave) off += x;
    tot += x;
  }
  total = tot;
  return off + inc - v;
}

__global__ __launch_bounds__(SEL_BLOCK) void spin_select_kernel(
    const float *__restrict__ scores, const int32_t *__restrict__ part_offsets,
    const int32_t *__restrict__ seq_lens, int Hkv, int tp, int topk, int includes_forced, int sink_pages,
    int recent_pages, int sel_stride, int32_t *__restrict__ sel, int32_t *__restrict__ nsel) {
  __shared__ int s_hist[256];
  __shared__ int s_wave[SEL_WAVES];
  __shared__ int s_digit, s_remaining;

  const int row = blockIdx.x;
  const int b = row / Hkv, h = row - b * Hkv;
  const int N = seq_lens[b];
  const int PP = part_offsets[b + 1] - part_offsets[b];
  const float *rs = scores + (size_t)Hkv * part_offsets[b] + (size_t)h * PP;
  int32_t *rsel = sel + (size_t)row * sel_stride;
  const int tid = threadIdx.x;
  int P = N > 0 ? (N + tp - 1) / tp : 0;
  if (P > PP) P = PP;

  // forced partitions: a prefix [0, nf_lo) and a suffix [first_hi, P)
  const int pages = (N + 15) >> 4;
  int sink_end = min(sink_pages, pages);
  int recent_begin = max(pages - recent_pages, 0);
  if (sink_end >= recent_begin) { sink_end = pages; recent_begin = pages; }
  int nf_lo = (N <= sink_end * 16) ? P : (sink_end * 16) / tp;
  int first_hi = min((recent_begin * 16 + tp - 1) / tp, P);
  if (first_hi <= nf_lo) { nf_lo = P; first_hi = P; }
  const int nforced = nf_lo + (P - first_hi);
  const int ncand = P - nforced;
  int kprime = includes_forced ? max(topk - nforced, 0) : topk;
  kprime = min(kprime, ncand);
  int take = nforced + kprime;
  if (take > sel_stride) {   // cannot happen for strides from spin_sel_stride(); keep stores in range
    kprime = max(sel_stride - nforced, 0);
    take = min(nforced + kprime, sel_stride);
  }

  // contiguous chunk of partitions per thread
  int chunk = (P + SEL_BLOCK - 1) / SEL_BLOCK;
  chunk = (chunk + 3) & ~3;
  const int c0 = min(tid * chunk, P), c1 = min(c0 + chunk, P);

  // ---- radix select of the kprime-th largest candidate key ----
  uint32_t prefix = 0;
  int remaining = kprime;   // rank (1-based) of the wanted key among keys matching the prefix
  if (kprime > 0) {
    for (int shift = 24; shift >= 0; shift -= 8) {
      if (tid < 256) s_hist[tid] = 0;
      __syncthreads();
      for (int p = c0; p < c1; ++p) {
        if (p < nf_lo || p >= first_hi) continue;
        const uint32_t k = score_key(rs[p]);
        if (shift == 24 || (k >> (shift + 8)) == prefix) atomicAdd(&s_hist[(k >> shift) & 255u], 1);
      }
      __syncthreads();
      // suffix sums over digits: thread t looks at digit 255 - t
      int cnt = tid < 256 ? s_hist[255 - tid] : 0, total;
      const int excl = block_exclusive_scan(cnt, s_wave, total);
      if (tid < 256 && excl < remaining && excl + cnt >= remaining) {
        s_digit = 255 - tid;
        s_remaining = remaining - excl;
      }
      __syncthreads();
      prefix = (prefix << 8) | (uint32_t)s_digit;
      remaining = s_remaining;
      __syncthreads();
    }
  }
  const uint32_t T = prefix;
  const int need_eq = kprime > 0 ? remaining : 0;   // how many candidates with key == T to take

  // ---- index-ordered compaction ----
  int my_gt = 0, my_eq = 0;
  for (int p = c0; p < c1; ++p) {
    if (p < nf_lo || p >= first_hi) { ++my_gt; continue; }
    if (kprime == 0) continue;
    const uint32_t k = score_key(rs[p]);
    my_gt += k > T;
    my_eq += k == T;
  }
  int total_eq, total_sel;
  const int eq_before = block_exclusive_scan(my_eq, s_wave, total_eq);
  int eq_quota = min(max(need_eq - eq_before, 0), my_eq);
  const int pos0 = block_exclusive_scan(my_gt + eq_quota, s_wave, total_sel);
  int pos = pos0;
  for (int p = c0; p < c1; ++p) {
    bool pick;
    if (p < nf_lo || p >= first_hi) pick = true;
    else if (kprime == 0) pick = false;
    else {
      const uint32_t k = score_key(rs[p]);
      pick = k > T;
      if (k == T && eq_quota > 0) { pick = true; --eq_quota; }
    }
    if (pick && pos < sel_stride) rsel[pos++] = p;
  }
  for (int i = take + tid; i < sel_stride; i += SEL_BLOCK) rsel[i] = -1;
  if (tid == 0) nsel[row] = min(total_sel, sel_stride);
}

template <int BLOCK, int KPT>
__global__ __launch_bounds__(BLOCK) void spin_select_reg_kernel(
    const float *__restrict__ scores, const int32_t *__restrict__ part_offsets,
    const int32_t *__restrict__ seq_lens, int Hkv, int tp, int topk, int includes_forced, int sink_pages,
    int recent_pages, int sel_stride, int32_t *__restrict__ sel, int32_t *__restrict__ nsel, spin_var var) {
  (void)select_reg_row<BLOCK, KPT, false>(scores, part_offsets, seq_lens, Hkv, tp, topk, includes_forced, sink_pages,
                                          recent_pages, sel_stride, sel, nsel, (int)blockIdx.x, var);
}

extern "C" int spin_select_topk(spin_ctx *ctx, int32_t batch, const float *scores, const int32_t *part_offsets,
                                const int32_t *seq_lens, int32_t *sel, int32_t *nsel, void *workspace,
                                void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch) return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!scores || !part_offsets || !seq_lens || !sel || !nsel) return SPIN_ERR_INVALID;
  (void)workspace;
  const spin_config &c = ctx->cfg;
  const int rows = batch * c.num_kv_heads;
#define SPIN_SELECT_ARGS                                                                                      \
  0, (hipStream_t)stream, scores, part_offsets, seq_lens, c.num_kv_heads, c.partition_tokens, c.topk,         \
      c.topk_includes_forced, c.sink_pages, c.recent_pages, ctx->sel_stride, sel, nsel
  if (ctx->max_parts <= 2048)
    spin_launch(ctx, SPIN_K_SELECT, spin_select_reg_kernel<256, 8>, dim3((unsigned)rows), dim3(256), SPIN_SELECT_ARGS, ctx->var);
  else if (ctx->max_parts <= 4096)
    spin_launch(ctx, SPIN_K_SELECT, spin_select_reg_kernel<512, 8>, dim3((unsigned)rows), dim3(512), SPIN_SELECT_ARGS, ctx->var);
  else if (ctx->max_parts <= 16384)
    spin_launch(ctx, SPIN_K_SELECT, spin_select_reg_kernel<1024, 16>, dim3((unsigned)rows), dim3(1024),
                SPIN_SELECT_ARGS, ctx->var);
  else if (ctx->max_parts <= 65536)
    spin_launch(ctx, SPIN_K_SELECT, spin_select_reg_kernel<1024, 64>, dim3((unsigned)rows), dim3(1024),
                SPIN_SELECT_ARGS, ctx->var);
  else if (ctx->var.count)
    return SPIN_ERR_UNSUPPORTED;   // variable-length partitions: rows of at most 65536 partitions
  else
    spin_launch(ctx, SPIN_K_SELECT, spin_select_kernel, dim3((unsigned)rows), dim3(SEL_BLOCK), SPIN_SELECT_ARGS);
#undef SPIN_SELECT_ARGS
  return spin_launch_status();
}
