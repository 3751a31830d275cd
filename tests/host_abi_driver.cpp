// Host-side walk through the C ABI for the sanitizer build (no GPU, no kernel launch): contexts of
// every shape the library supports are created, sized, fed empty batches and bad arguments, and
// destroyed.  Address and undefined-behaviour sanitizers watch the host code meanwhile; the program
// itself only checks return codes.  Built and run by tests/test_host_sanitizers.py.
#include "spin.h"
#include "spin_measure.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

static int failures = 0;
#define EXPECT(cond)                                                          \
  do {                                                                        \
    if (!(cond)) { std::fprintf(stderr, "FAILED line %d: %s\n", __LINE__, #cond); ++failures; } \
  } while (0)

static spin_config base_config() {
  spin_config c;
  std::memset(&c, 0, sizeof c);
  c.max_batch = 4; c.num_q_heads = 32; c.num_kv_heads = 8; c.head_dim = 128; c.page_tokens = 16;
  c.partition_tokens = 16; c.score_kind = SPIN_SCORE_MINMAX; c.sketch_channels = 16; c.reps_per_partition = 4;
  c.topk = 64; c.topk_includes_forced = 1; c.sink_pages = 2; c.recent_pages = 4; c.max_context = 32768;
  c.leaf_entries = 512;
  return c;
}

// every stage call with an empty batch (returns before touching its pointers) and with NULL pointers
static void poke(spin_ctx *x, const spin_config &c) {
  EXPECT(spin_workspace_bytes(x) > 0 && spin_workspace_bytes(x) % 256 == 0);
  EXPECT(spin_sel_stride(x) > 0 && spin_page_stride(x) > 0 && spin_dir_stride(x) > 0 && spin_decode_splits(x) > 0);
  EXPECT(spin_summary_bytes(x, 16) > 0 && spin_summary_bytes(x, -1) == 0);
  void *n = nullptr;
  int dummy_ws = 0;   // a non-NULL workspace address that no path dereferences on the host
  void *ws = &dummy_ws;
  for (int batch : {0, 1, c.max_batch + 1, -1}) {
    const int want_ok = batch == 0;
    int st;
    st = spin_score_partitions(x, batch, n, n, nullptr, nullptr, nullptr, nullptr, ws, n);
    EXPECT(want_ok ? st == SPIN_OK : st == SPIN_ERR_INVALID);
    st = spin_select_topk(x, batch, nullptr, nullptr, nullptr, nullptr, nullptr, ws, n);
    EXPECT(want_ok ? st == SPIN_OK : st == SPIN_ERR_INVALID);
    st = spin_score_select_topk(x, batch, n, n, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, ws, n);
    EXPECT(want_ok ? st == SPIN_OK : st == SPIN_ERR_INVALID);
    st = spin_pin_partitions(x, batch, nullptr, nullptr, nullptr, nullptr, 4, n);
    EXPECT(want_ok ? st == SPIN_OK : st == SPIN_ERR_INVALID);
    st = spin_resolve_slots(x, batch, 0, nullptr, nullptr, nullptr, nullptr, nullptr, 1, nullptr, nullptr, nullptr,
                            nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, ws, n);
    EXPECT(want_ok ? st == SPIN_OK : st < 0);
    st = spin_select_resolve(x, batch, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 1, nullptr,
                             nullptr, nullptr, nullptr, ws, n);
    EXPECT(want_ok ? st == SPIN_OK : st < 0);
    st = spin_score_select_resolve(x, batch, n, n, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                                   nullptr, 1, nullptr, nullptr, nullptr, nullptr, ws, n);
    EXPECT(want_ok ? st == SPIN_OK : st < 0);
    st = spin_sparse_decode(x, batch, n, n, 1, nullptr, nullptr, nullptr, n, nullptr, ws, n);
    EXPECT(want_ok ? st == SPIN_OK : st == SPIN_ERR_INVALID);
    st = spin_sparse_decode_static(x, batch, n, n, 1, nullptr, nullptr, nullptr, n, nullptr, nullptr, n);
    EXPECT(want_ok ? st == SPIN_OK : st == SPIN_ERR_INVALID);
    // the calls below also refuse contexts they do not apply to, before looking at the batch
    st = spin_select_resolve_forced(x, batch, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 1, nullptr,
                                    nullptr, nullptr, nullptr, n, n, 1, ws, n);
    EXPECT(want_ok ? (st == SPIN_OK || st == SPIN_ERR_UNSUPPORTED) : st < 0);
    st = spin_sparse_decode_rest(x, batch, n, n, 1, nullptr, nullptr, nullptr, n, nullptr, ws, n);
    EXPECT(want_ok ? (st == SPIN_OK || st == SPIN_ERR_UNSUPPORTED) : st < 0);
    st = spin_split_hits_misses(x, batch, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, n);
    EXPECT(want_ok ? st == SPIN_OK : st == SPIN_ERR_INVALID);
    st = spin_sparse_decode_begin(x, batch, n, n, 1, nullptr, nullptr, nullptr, ws, n);
    EXPECT(want_ok ? (st == SPIN_OK || st == SPIN_ERR_UNSUPPORTED) : st < 0);
    st = spin_sparse_decode_finish(x, batch, n, n, 1, nullptr, nullptr, nullptr, n, nullptr, ws, n);
    EXPECT(want_ok ? (st == SPIN_OK || st == SPIN_ERR_UNSUPPORTED) : st < 0);
    st = spin_build_summaries(x, batch, n, 1, nullptr, nullptr, 1, nullptr, nullptr, nullptr, n, ws, n);
    EXPECT(want_ok ? st == SPIN_OK : st < 0);
    st = spin_append_kv(x, batch, n, n, nullptr, n, 1, nullptr, nullptr, 1, nullptr, nullptr, n, ws, n);
    EXPECT(want_ok ? st == SPIN_OK : st < 0);
    st = spin_gather_misses(x, batch, n, nullptr, nullptr, nullptr, nullptr, n, 1, ws, n);
    EXPECT(want_ok ? st == SPIN_OK : st < 0);
    st = spin_offload_pages(x, batch, n, 1, n, nullptr, nullptr, nullptr, nullptr, ws, n);
    EXPECT(want_ok ? st == SPIN_OK : st < 0);
    st = spin_copy_misses_host(x, batch, n, nullptr, nullptr, nullptr, nullptr, n, 1, n, nullptr);
    EXPECT(want_ok ? st == SPIN_OK : st < 0);
    st = spin_reclaim_tail(x, batch, nullptr, nullptr, nullptr, nullptr, 1, nullptr, ws, n);
    EXPECT(want_ok ? st == SPIN_OK : st < 0);
    st = spin_alloc_leaves(x, batch, nullptr, nullptr, nullptr, nullptr, nullptr, 1, nullptr, ws, n);
    EXPECT(want_ok ? st == SPIN_OK : st < 0);
    st = spin_free_leaves(x, batch, nullptr, 1, nullptr, ws, n);
    EXPECT(want_ok ? st == SPIN_OK : st < 0);
  }
  EXPECT(spin_pack_kv_pages(x, 0, n, n, nullptr, n, 1, n) == SPIN_OK);
  EXPECT(spin_pack_kv_pages(x, 4, n, n, nullptr, n, 1, n) == SPIN_ERR_INVALID);
  EXPECT(spin_pack_kv_pages(x, -1, n, n, nullptr, n, 1, n) == SPIN_ERR_INVALID);
  EXPECT(spin_workspace_init(x, nullptr, n) == SPIN_ERR_WORKSPACE);
  EXPECT(spin_set_step(x, nullptr, 0, n) == SPIN_ERR_WORKSPACE && spin_set_step(x, ws, -1, n) == SPIN_ERR_INVALID);
  EXPECT(spin_advance_step(x, nullptr, n) == SPIN_ERR_WORKSPACE);
  EXPECT(spin_resolve_slots(x, 1, -2, nullptr, nullptr, nullptr, nullptr, nullptr, 1, nullptr, nullptr, nullptr, nullptr,
                            nullptr, nullptr, nullptr, nullptr, nullptr, ws, n) == SPIN_ERR_INVALID);
  EXPECT(spin_probe_stream_read(x, nullptr, 16, ws, n) < 0);
  EXPECT(spin_profile_enable(x, -1) == SPIN_ERR_INVALID);
  int32_t cnt = 0; float mean = 0, mn = 0;
  EXPECT(spin_profile_read(x, -1, &cnt, &mean, &mn) == SPIN_ERR_INVALID);
  EXPECT(spin_profile_read(x, 1000, &cnt, &mean, &mn) == SPIN_ERR_INVALID);
  EXPECT(spin_profile_read(x, SPIN_K_DECODE, nullptr, &mean, &mn) == SPIN_ERR_INVALID);
  EXPECT(spin_profile_read(x, SPIN_K_META, &cnt, &mean, &mn) == SPIN_OK && cnt == 0);   // nothing timed
  // CPU page table: a table needs positive sizes; NULL returns to the identity
  int32_t cpu_table[4] = {3, 2, 1, 0};
  EXPECT(spin_set_host_page_table(x, cpu_table, 4, 4) == SPIN_OK);
  EXPECT(spin_set_host_page_table(x, cpu_table, 0, 4) == SPIN_ERR_INVALID);
  EXPECT(spin_set_host_page_table(x, cpu_table, 4, 0) == SPIN_ERR_INVALID);
  EXPECT(spin_set_host_page_table(x, nullptr, 0, 40) == SPIN_OK);     // identity, bounded by the pool's size
  EXPECT(spin_set_host_page_table(x, nullptr, 0, -1) == SPIN_ERR_INVALID);
  EXPECT(spin_set_host_page_table(x, nullptr, 0, 0) == SPIN_OK);
  // partition tables: all four or none
  int32_t t[4] = {0, 0, 0, 0};
  EXPECT(spin_set_partition_tables(x, nullptr, nullptr, nullptr, nullptr) == SPIN_OK);
  const int st = spin_set_partition_tables(x, t, t, t, nullptr);
  EXPECT(st < 0);
  if (c.variable_partitions) {
    EXPECT(spin_set_partition_tables(x, t, t, t, t) == SPIN_OK);
    EXPECT(spin_set_partition_tables(x, nullptr, nullptr, nullptr, nullptr) == SPIN_OK);
  }
}

int main() {
  // null handling of the context-free calls
  spin_ctx *x = nullptr;
  EXPECT(spin_create(nullptr, &x) == SPIN_ERR_INVALID && x == nullptr);
  spin_config c0 = base_config();
  EXPECT(spin_create(&c0, nullptr) == SPIN_ERR_INVALID);
  spin_destroy(nullptr);
  EXPECT(spin_workspace_bytes(nullptr) == 0 && spin_sel_stride(nullptr) == 0 && spin_page_stride(nullptr) == 0);
  EXPECT(spin_dir_stride(nullptr) == 0 && spin_decode_splits(nullptr) == 0 && spin_summary_bytes(nullptr, 16) == 0);
  for (int s = 2; s >= -12; --s) EXPECT(spin_status_string(s) != nullptr && std::strlen(spin_status_string(s)) > 0);

  // shapes the library supports
  std::vector<spin_config> good;
  good.push_back(base_config());
  for (int tp : {1, 2, 4, 8, 32, 64, 128, 256}) { spin_config c = base_config(); c.partition_tokens = tp; good.push_back(c); }
  { spin_config c = base_config(); c.partition_tokens = 1; c.score_kind = SPIN_SCORE_SKETCH; c.topk = 1024;
    c.max_context = 65536; c.sink_pages = 0; c.recent_pages = 0; good.push_back(c);
    c.max_context = 131072; good.push_back(c); c.max_context = 262144; good.push_back(c); }
  { spin_config c = base_config(); c.partition_tokens = 128; c.score_kind = SPIN_SCORE_REPMAX; c.topk = 32;
    c.topk_includes_forced = 0; c.sink_pages = 4; c.recent_pages = 64; c.max_context = 131072; good.push_back(c); }
  for (int reps : {1, 2}) { spin_config c = base_config(); c.score_kind = SPIN_SCORE_REPMAX; c.reps_per_partition = reps;
    c.partition_tokens = 64; good.push_back(c); c.partition_tokens = 16; good.push_back(c); }
  { spin_config c = base_config(); c.score_kind = SPIN_SCORE_REPMAX; c.reps_per_partition = 1; c.variable_partitions = 1;
    c.partition_tokens = 128; good.push_back(c); }
  for (int pol : {0, 1}) for (int exact : {0, 1}) {
    spin_config c = base_config(); c.lru_timestamps = 64; c.lru_policy = pol; c.lru_evict_exact = exact;
    c.max_context = 262144; c.max_batch = 32; good.push_back(c);
    c.partition_tokens = 64; good.push_back(c); c.partition_tokens = 4; good.push_back(c);
  }
  { spin_config c = base_config(); c.variable_partitions = 1; c.partition_tokens = 256; good.push_back(c);
    c.lru_timestamps = 16; good.push_back(c); }
  for (int g : {1, 2, 3, 8, 12, 16}) { spin_config c = base_config(); c.num_kv_heads = 2; c.num_q_heads = 2 * g; good.push_back(c); }
  for (int w : {2, 4, 8}) for (int d : {2, 3, 4}) for (int sp : {0, 1, 3, 64, 1000}) {
    spin_config c = base_config(); c.decode_waves = w; c.decode_depth = d; c.decode_splits = sp; good.push_back(c);
  }
  { spin_config c = base_config(); c.max_context = 1; c.topk = 0; c.sink_pages = 0; c.recent_pages = 0; good.push_back(c); }
  { spin_config c = base_config(); c.max_batch = 1024; c.max_context = 1 << 20; c.topk = 4096; good.push_back(c); }
  for (const spin_config &c : good) {
    x = nullptr;
    const int st = spin_create(&c, &x);
    EXPECT(st == SPIN_OK && x != nullptr);
    if (st != SPIN_OK) {
      std::fprintf(stderr, "  config tp=%d kind=%d ctx=%d lru=%d var=%d -> %d\n", c.partition_tokens, c.score_kind,
                   c.max_context, c.lru_timestamps, c.variable_partitions, st);
      continue;
    }
    poke(x, c);
    spin_destroy(x);
  }

  // shapes it must refuse, with *out left alone
  std::vector<spin_config> bad;
  { spin_config c = base_config(); c.head_dim = 64; bad.push_back(c); }
  { spin_config c = base_config(); c.page_tokens = 32; bad.push_back(c); }
  { spin_config c = base_config(); c.partition_tokens = 24; bad.push_back(c); }
  { spin_config c = base_config(); c.partition_tokens = 0; bad.push_back(c); }
  { spin_config c = base_config(); c.partition_tokens = -16; bad.push_back(c); }
  { spin_config c = base_config(); c.num_q_heads = 33; bad.push_back(c); }
  { spin_config c = base_config(); c.num_q_heads = 8 * 17; bad.push_back(c); }
  { spin_config c = base_config(); c.num_kv_heads = 0; bad.push_back(c); }
  { spin_config c = base_config(); c.max_batch = 0; bad.push_back(c); }
  { spin_config c = base_config(); c.max_context = 0; bad.push_back(c); }
  { spin_config c = base_config(); c.score_kind = 7; bad.push_back(c); }
  { spin_config c = base_config(); c.score_kind = SPIN_SCORE_REPMAX; c.reps_per_partition = 3; bad.push_back(c); }
  { spin_config c = base_config(); c.topk = -1; bad.push_back(c); }
  { spin_config c = base_config(); c.sink_pages = -1; bad.push_back(c); }
  { spin_config c = base_config(); c.decode_waves = 3; bad.push_back(c); }
  { spin_config c = base_config(); c.decode_depth = 9; bad.push_back(c); }
  { spin_config c = base_config(); c.decode_splits = -2; bad.push_back(c); }
  { spin_config c = base_config(); c.lru_timestamps = -1; bad.push_back(c); }
  { spin_config c = base_config(); c.lru_policy = 5; bad.push_back(c); }
  { spin_config c = base_config(); c.leaf_entries = 0; bad.push_back(c); }
  { spin_config c = base_config(); c.score_waves = 5; bad.push_back(c); }
  for (const spin_config &c : bad) {
    x = reinterpret_cast<spin_ctx *>(0x10);
    const int st = spin_create(&c, &x);
    EXPECT(st < 0 && x == reinterpret_cast<spin_ctx *>(0x10));
  }
  if (failures) { std::fprintf(stderr, "%d check(s) failed\n", failures); return 1; }
  std::printf("host ABI walk: %zu contexts created and released, %zu refused\n", good.size(), bad.size());
  return 0;
}
