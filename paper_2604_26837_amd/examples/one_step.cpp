// One decode step of one layer through the C ABI alone (no Python, no torch): the caller owns every
// buffer (hipMalloc), lays the pages out with spin_pack_kv_pages, fills the two-level page table,
// builds the summaries (Index), then runs score -> select -> resolve -> attention (and the same step as
// stages 1-3 in one call + attention, which must give the same bits; as stage 4 from the library's own
// scratch array; and as the step that attends the sink / recent pages beside stages 2+3) and checks the
// output against dense attention restricted to the pages the library reports (Section 4.1: the
// attention stage is exact on the selected set).  Exit status 0 and a line "one_step: ok" on success.
//
// Build (next to libspin.so):  hipcc -O2 one_step.cpp -I ../../include -L .. -lspin -Wl,-rpath,'$ORIGIN/..' -o one_step
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "spin.h"

#define HIP_OK(x)                                                                       \
  do {                                                                                  \
    hipError_t e_ = (x);                                                                \
    if (e_ != hipSuccess) {                                                             \
      std::fprintf(stderr, "one_step: %s failed: %s\n", #x, hipGetErrorString(e_));     \
      return 2;                                                                         \
    }                                                                                   \
  } while (0)
#define SPIN_OK_OR_DIE(x)                                                               \
  do {                                                                                  \
    int s_ = (x);                                                                       \
    if (s_ != SPIN_OK) {                                                                \
      std::fprintf(stderr, "one_step: %s -> %s\n", #x, spin_status_string(s_));        \
      return 3;                                                                         \
    }                                                                                   \
  } while (0)

static uint16_t to_bf16(float f) {   // round to nearest even
  uint32_t u;
  std::memcpy(&u, &f, 4);
  return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}
static float from_bf16(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}
// small deterministic generator: roughly normal values from twelve uniforms
static uint32_t g_state = 20260427u;
static float next_normal() {
  float s = 0.f;
  for (int i = 0; i < 12; ++i) {
    g_state = g_state * 1664525u + 1013904223u;
    s += (float)(g_state >> 8) * (1.0f / 16777216.0f);
  }
  return s - 6.0f;
}

template <typename T>
static int upload(T **dev, const std::vector<T> &host) {
  HIP_OK(hipMalloc((void **)dev, host.size() * sizeof(T)));
  HIP_OK(hipMemcpy(*dev, host.data(), host.size() * sizeof(T), hipMemcpyHostToDevice));
  return 0;
}

int main() {
  const int Hq = 8, Hkv = 2, D = 128, G = Hq / Hkv, N = 4096 - 5, pages = (N + 15) / 16, rows = Hkv;
  spin_config cfg = {};
  cfg.max_batch = 1; cfg.num_q_heads = Hq; cfg.num_kv_heads = Hkv; cfg.head_dim = D; cfg.page_tokens = 16;
  cfg.partition_tokens = 16; cfg.score_kind = SPIN_SCORE_MINMAX; cfg.sketch_channels = 16; cfg.reps_per_partition = 4;
  cfg.topk = 32; cfg.topk_includes_forced = 1; cfg.sink_pages = 1; cfg.recent_pages = 1; cfg.max_context = 4096;
  cfg.leaf_entries = 512;
  spin_ctx *ctx = nullptr;
  SPIN_OK_OR_DIE(spin_create(&cfg, &ctx));
  const int sel_stride = spin_sel_stride(ctx), page_stride = spin_page_stride(ctx), dir_stride = spin_dir_stride(ctx);

  // keys, values and the query, rounded to bf16; page i of row r is natural page r * pages + i
  const int n_pages = rows * pages;
  std::vector<uint16_t> k((size_t)n_pages * 16 * D), v(k.size()), q((size_t)Hq * D);
  for (auto &x : k) x = to_bf16(next_normal());
  for (auto &x : v) x = to_bf16(next_normal());
  for (auto &x : q) x = to_bf16(next_normal());
  // physical order differs from logical order: slot = a permutation of the natural page index
  const int64_t pool_slots = 512;
  std::vector<int32_t> slot_of(n_pages);
  for (int i = 0; i < n_pages; ++i) slot_of[i] = (i * 37 + 11) % (int)pool_slots;
  // two-level table: one leaf chunk per row here (a chunk covers 512 pages)
  std::vector<int32_t> dir((size_t)rows * dir_stride, -1), leaf((size_t)rows * cfg.leaf_entries, -1);
  for (int r = 0; r < rows; ++r) {
    dir[(size_t)r * dir_stride] = r;
    for (int p = 0; p < pages; ++p) leaf[(size_t)r * cfg.leaf_entries + p] = slot_of[r * pages + p];
  }
  const int padded = ((pages + SPIN_PART_ALIGN - 1) / SPIN_PART_ALIGN) * SPIN_PART_ALIGN;   // partitions = pages here
  std::vector<int32_t> part_offsets = {0, padded}, seq_lens = {N};

  uint16_t *d_k, *d_v, *d_q;
  int32_t *d_slot_of, *d_dir, *d_leaf, *d_off, *d_len;
  if (upload(&d_k, k) || upload(&d_v, v) || upload(&d_q, q) || upload(&d_slot_of, slot_of) || upload(&d_dir, dir) ||
      upload(&d_leaf, leaf) || upload(&d_off, part_offsets) || upload(&d_len, seq_lens))
    return 2;
  void *d_pool, *d_summ, *d_ws;
  float *d_scores, *d_lse;
  int32_t *d_sel, *d_nsel, *d_slots, *d_pids, *d_np;
  uint16_t *d_mask, *d_out;
  HIP_OK(hipMalloc(&d_pool, (size_t)pool_slots * SPIN_SLOT_BYTES));
  HIP_OK(hipMalloc(&d_summ, spin_summary_bytes(ctx, padded)));
  HIP_OK(hipMalloc(&d_ws, spin_workspace_bytes(ctx)));
  HIP_OK(hipMalloc((void **)&d_scores, (size_t)padded * Hkv * sizeof(float)));
  HIP_OK(hipMalloc((void **)&d_sel, (size_t)rows * sel_stride * 4));
  HIP_OK(hipMalloc((void **)&d_nsel, rows * 4));
  HIP_OK(hipMalloc((void **)&d_slots, (size_t)rows * page_stride * 4));
  HIP_OK(hipMalloc((void **)&d_pids, (size_t)rows * page_stride * 4));
  HIP_OK(hipMalloc((void **)&d_mask, (size_t)rows * page_stride * 2));
  HIP_OK(hipMalloc((void **)&d_np, rows * 4));
  HIP_OK(hipMalloc((void **)&d_out, (size_t)Hq * D * 2));
  HIP_OK(hipMalloc((void **)&d_lse, Hq * sizeof(float)));
  HIP_OK(hipMemset(d_summ, 0, spin_summary_bytes(ctx, padded)));

  hipStream_t st = nullptr;   // the default stream
  SPIN_OK_OR_DIE(spin_workspace_init(ctx, d_ws, st));
  // set-up: page layout, summaries
  SPIN_OK_OR_DIE(spin_pack_kv_pages(ctx, n_pages, d_k, d_v, d_slot_of, d_pool, pool_slots, st));
  SPIN_OK_OR_DIE(spin_build_summaries(ctx, 1, d_pool, pool_slots, d_dir, d_leaf, rows, d_off, d_len, nullptr, d_summ, d_ws, st));
  // the decode step
  SPIN_OK_OR_DIE(spin_score_partitions(ctx, 1, d_q, d_summ, nullptr, d_off, d_len, d_scores, d_ws, st));
  SPIN_OK_OR_DIE(spin_select_topk(ctx, 1, d_scores, d_off, d_len, d_sel, d_nsel, d_ws, st));
  SPIN_OK_OR_DIE(spin_resolve_slots(ctx, 1, 0, d_sel, d_nsel, d_len, d_dir, d_leaf, rows, nullptr, nullptr, d_slots, d_pids,
                                    d_mask, d_np, nullptr, nullptr, nullptr, d_ws, st));
  SPIN_OK_OR_DIE(spin_sparse_decode(ctx, 1, d_q, d_pool, pool_slots, d_slots, d_mask, d_np, d_out, d_lse, d_ws, st));
  SPIN_OK_OR_DIE(spin_poll_status(ctx, d_ws, st));   // synchronises; first fault a kernel detected, if any

  std::vector<int32_t> np(rows), pids((size_t)rows * page_stride), slots((size_t)rows * page_stride);
  std::vector<uint16_t> mask((size_t)rows * page_stride), out((size_t)Hq * D);
  HIP_OK(hipMemcpy(np.data(), d_np, rows * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(pids.data(), d_pids, pids.size() * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(slots.data(), d_slots, slots.size() * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(mask.data(), d_mask, mask.size() * 2, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(out.data(), d_out, out.size() * 2, hipMemcpyDeviceToHost));

  // the same step in three launches (stages 1-3 in one call, then attention) must give the same bits
  {
    uint16_t *d_out2;
    HIP_OK(hipMalloc((void **)&d_out2, (size_t)Hq * D * 2));
    HIP_OK(hipMemset(d_np, 0xff, rows * 4));
    SPIN_OK_OR_DIE(spin_score_select_resolve(ctx, 1, d_q, d_summ, nullptr, d_off, d_len, d_scores, d_sel, d_nsel, d_dir, d_leaf,
                                             rows, d_slots, d_pids, d_mask, d_np, d_ws, st));
    SPIN_OK_OR_DIE(spin_sparse_decode(ctx, 1, d_q, d_pool, pool_slots, d_slots, d_mask, d_np, d_out2, d_lse, d_ws, st));
    SPIN_OK_OR_DIE(spin_poll_status(ctx, d_ws, st));
    std::vector<uint16_t> out2(out.size());
    HIP_OK(hipMemcpy(out2.data(), d_out2, out2.size() * 2, hipMemcpyDeviceToHost));
    if (std::memcmp(out.data(), out2.data(), out.size() * 2) != 0) {
      std::fprintf(stderr, "one_step: the three-launch step differs from the four stage calls\n");
      return 1;
    }
  }

  // stage 4 without a workspace (its scratch in the library's own device array) gives the same bits; and the
  // step whose launch of stages 2+3 also attends the sink / recent pages gives the same page list and an output
  // within stage 4's tolerance of the one above (the order of the online-softmax updates differs)
  std::vector<uint16_t> out_forced(out.size());
  {
    uint16_t *d_out3;
    int32_t *d_status;
    HIP_OK(hipMalloc((void **)&d_out3, (size_t)Hq * D * 2));
    HIP_OK(hipMalloc((void **)&d_status, 4));
    HIP_OK(hipMemset(d_status, 0, 4));
    SPIN_OK_OR_DIE(spin_sparse_decode_static(ctx, 1, d_q, d_pool, pool_slots, d_slots, d_mask, d_np, d_out3, d_lse, d_status, st));
    HIP_OK(hipStreamSynchronize(st));
    std::vector<uint16_t> out3(out.size());
    int32_t status = -1;
    HIP_OK(hipMemcpy(out3.data(), d_out3, out3.size() * 2, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(&status, d_status, 4, hipMemcpyDeviceToHost));
    if (status != 0 || std::memcmp(out.data(), out3.data(), out.size() * 2) != 0) {
      std::fprintf(stderr, "one_step: spin_sparse_decode_static differs from spin_sparse_decode (status %d)\n", status);
      return 1;
    }
    std::vector<int32_t> slots_before(slots);
    SPIN_OK_OR_DIE(spin_score_partitions(ctx, 1, d_q, d_summ, nullptr, d_off, d_len, d_scores, d_ws, st));
    SPIN_OK_OR_DIE(spin_select_resolve_forced(ctx, 1, d_scores, d_off, d_len, d_sel, d_nsel, d_dir, d_leaf, rows, d_slots, d_pids,
                                              d_mask, d_np, d_q, d_pool, pool_slots, d_ws, st));
    SPIN_OK_OR_DIE(spin_sparse_decode_rest(ctx, 1, d_q, d_pool, pool_slots, d_slots, d_mask, d_np, d_out3, d_lse, d_ws, st));
    SPIN_OK_OR_DIE(spin_poll_status(ctx, d_ws, st));
    HIP_OK(hipMemcpy(out_forced.data(), d_out3, out_forced.size() * 2, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(slots.data(), d_slots, slots.size() * 4, hipMemcpyDeviceToHost));
    if (slots != slots_before) {
      std::fprintf(stderr, "one_step: spin_select_resolve_forced resolved other slots than the stage calls\n");
      return 1;
    }
    for (size_t i = 0; i < out.size(); ++i) {
      const double a = from_bf16(out[i]), b = from_bf16(out_forced[i]);
      if (!(std::fabs(a - b) <= 2e-2 + 1e-2 * std::fabs(a))) {
        std::fprintf(stderr, "one_step: the step that attends sink / recent pages early differs at %zu: %g vs %g\n", i, b, a);
        return 1;
      }
    }
  }

  // checks: 32 pages per row with the first and the last page among them, slots as in the table, and the
  // output equal to dense attention over exactly those tokens (double precision on the bf16 inputs)
  int bad = 0;
  double worst = 0.0;
  for (int r = 0; r < rows; ++r) {
    const int32_t *pg = &pids[(size_t)r * page_stride];
    if (np[r] != cfg.topk || pg[0] != 0 || pg[np[r] - 1] != pages - 1) { std::fprintf(stderr, "row %d: page list\n", r); ++bad; }
    for (int i = 0; i < np[r]; ++i)
      if (slots[(size_t)r * page_stride + i] != slot_of[r * pages + pg[i]]) { std::fprintf(stderr, "row %d: slot %d\n", r, i); ++bad; }
    for (int g = 0; g < G; ++g) {
      const uint16_t *qh = &q[(size_t)(r * G + g) * D];
      std::vector<double> logit, acc(D, 0.0);
      std::vector<const uint16_t *> vrow;
      double mx = -INFINITY;
      for (int i = 0; i < np[r]; ++i)
        for (int t = 0; t < 16; ++t)
          if ((mask[(size_t)r * page_stride + i] >> t) & 1) {
            const uint16_t *kr = &k[((size_t)(r * pages + pg[i]) * 16 + t) * D];
            double s = 0.0;
            for (int d = 0; d < D; ++d) s += (double)from_bf16(qh[d]) * (double)from_bf16(kr[d]);
            s /= std::sqrt((double)D);
            logit.push_back(s);
            vrow.push_back(&v[((size_t)(r * pages + pg[i]) * 16 + t) * D]);
            mx = s > mx ? s : mx;
          }
      double l = 0.0;
      for (size_t j = 0; j < logit.size(); ++j) {
        const double w = std::exp(logit[j] - mx);
        l += w;
        for (int d = 0; d < D; ++d) acc[d] += w * (double)from_bf16(vrow[j][d]);
      }
      for (int d = 0; d < D; ++d) {
        const double ref = acc[d] / l, got = (double)from_bf16(out[(size_t)(r * G + g) * D + d]);
        const double excess = std::fabs(got - ref) - (2e-2 + 1e-2 * std::fabs(ref));
        worst = excess > worst ? excess : worst;
        if (excess > 0.0) ++bad;
      }
    }
  }
  spin_destroy(ctx);
  if (bad) {
    std::fprintf(stderr, "one_step: %d mismatches (worst excess over tolerance %.3g)\n", bad, worst);
    return 1;
  }
  std::printf("one_step: ok (%d rows, %d of %d pages attended per row, sel stride %d, page stride %d)\n", rows, cfg.topk, pages,
              sel_stride, page_stride);
  return 0;
}
