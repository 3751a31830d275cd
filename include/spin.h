/*
 * spin.h -- C ABI of the per-decode-step sparse-attention hot path on MI355X.
 *
 * One decode step of one layer runs four stages, each a call below:
 *
 *   spin_score_partitions   Select, scoring half   (Section 4.1 "Select"; Table 1, score(q, k_sums))
 *   spin_select_topk        Select, top-k half     (Table 1, "-> topk"; Section 4.2)
 *   spin_resolve_slots      Retrieve, lookup half  (Section 5.2 steps 1-2; Section 5.3 bucketed LRU;
 *                                                   Section 5.4 two-level tables)
 *   spin_sparse_decode      Attention              (Section 4.1 "Attention")
 *
 * Around them:
 *   spin_pack_kv_pages, spin_build_summaries, spin_append_kv   Offload's layout and Index (Section 4.1)
 *   spin_gather_misses, spin_copy_misses_host                  Retrieve steps 3-4 (Sections 5.2, 5.5)
 *   spin_offload_pages                                         Offload's copy, slot -> host page (Table 1)
 *   spin_select_resolve                                        stages 2+3 in one launch, same results
 *   spin_select_resolve_forced, spin_sparse_decode_rest        the same, the sink / recent pages attended beside 2+3
 *   spin_score_select_topk                                     stages 1+2 in one call, same results
 *   spin_score_select_resolve                                  stages 1-3 in one call, same results
 *   spin_pin_partitions                                        always-attended outlier partitions (Section 4.2)
 *   spin_set_partition_tables                                  variable-length partitions (Section 5.2)
 *   spin_set_host_page_table                                   CPU page table (Section 5.2)
 *   spin_alloc_leaves, spin_free_leaves, spin_reclaim_tail     on-demand metadata, budget resizing (5.3, 5.4)
 *
 * Conventions
 * -----------
 * - Every pointer named below as DEVICE points to HBM owned by the caller; the
 *   library never allocates, frees or synchronises inside a stage call.  The
 *   library owns only the host-side spin_ctx.
 * - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   Calls enqueue kernels on it and return.
 * - Return value: SPIN_OK (0) or a negative spin_status.  Host-checkable
 *   mistakes (NULL pointer, batch > max_batch, unsupported shape) are returned
 *   before anything is launched.  Faults only the device can see (a selected
 *   page that is not resident, a slot id outside the pool, a budget smaller
 *   than the step's selection) set a sticky status word inside `workspace`,
 *   read back by spin_poll_status(); the offending page/row is skipped so no
 *   access leaves its buffer.
 * - A "row" is one (request b, KV head h) pair, row = b * num_kv_heads + h.
 *   Everything is independent per row.
 * - Identical inputs give identical output bits, run to run.
 *
 * Data layout in HBM (all little endian, bf16 = upper half of an IEEE binary32)
 * ---------------------------------------------------------------------------
 * q            bf16 [batch][num_q_heads][128]
 * kv_pool      one SLOT = one physical page of ONE KV head (head-wise pages,
 *              Section 5.2) = 8192 bytes: the K tile (4096 B) then the V tile
 *              (4096 B) of 16 tokens x 128 channels, each stored in the register
 *              image of the matrix-core operand that consumes it, so that every
 *              wavefront load is one contiguous 1 KiB transaction:
 *                K[t][d] at element ((d/32)*64 + ((d%32)/8)*16 + t)*8 + d%8
 *                V[t][d] at element ((((d/32)*64 + (t/4)*16 + d%16)*2 + (d/16)%2)*4) + t%4
 *              With partition_tokens < 16 both tiles are token-major instead, K[t][d]
 *              and V[t][d] at element t*128 + d of their tile, so that the key and the
 *              value of one attended token are 256 contiguous bytes each.
 *              Use spin_pack_kv_pages to write pages in this layout.
 * part_offsets int32 [batch+1], prefix sum over requests of their partition
 *              count rounded up to a multiple of 16 (SPIN_PART_ALIGN).  Row
 *              (b,h) owns entries [num_kv_heads*part_offsets[b] + h*PP_b, +PP_b)
 *              of `scores` and of the summary array, PP_b = part_offsets[b+1]-part_offsets[b].
 * summaries    per 16 consecutive summary rows one TILE, chunk-major
 *              [KD/KC][16][KC] bf16 (KD = contraction length, KC = elements one lane
 *              feeds to one matrix instruction):
 *                MINMAX  row = partition,       KD = 256: [max(128) | min(128)], KC = 8
 *                REPMAX  row = partition*R + r, KD = 128: representative r,      KC = 8
 *                SKETCH  row = token,           KD = sketch_channels (16),       KC = 4
 *              (written by spin_build_summaries).
 * dir          int32 [rows][dir_stride], dir_stride = ceil(ceil(max_context/page_tokens)/leaf_entries);
 *              entry = index of a leaf chunk in leaf_pool, or -1 (no leaf allocated).
 * leaf_pool    int32 [chunks][leaf_entries]; entry = slot of that logical page, or -1.
 */
#ifndef SPIN_H
#define SPIN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct spin_ctx spin_ctx; /* opaque, host side */

enum spin_status {
  SPIN_OK = 0,
  SPIN_ERR_INVALID = -1,      /* bad argument */
  SPIN_ERR_UNSUPPORTED = -2,  /* shape or mode not built */
  SPIN_ERR_WORKSPACE = -3,    /* workspace missing */
  SPIN_ERR_HIP = -4,          /* a HIP runtime call failed */
  SPIN_ERR_BUDGET = -5,       /* device: a row's slot budget cannot hold its selection */
  SPIN_ERR_NOT_RESIDENT = -6, /* device: a selected page has no leaf or no slot */
  SPIN_ERR_SLOT_RANGE = -7,   /* device: a slot id lies outside the pool */
  SPIN_ERR_LEAF_POOL = -8,    /* device: no free leaf chunk left in the segment pool */
  SPIN_ERR_STATIC_LIMIT = -9  /* spin_sparse_decode_static: the shape needs more than SPIN_STATIC_SCRATCH_BYTES */
};

enum spin_score_kind { SPIN_SCORE_MINMAX = 0, SPIN_SCORE_SKETCH = 1, SPIN_SCORE_REPMAX = 2 };

#define SPIN_PART_ALIGN 16
#define SPIN_SLOT_BYTES 8192
#define SPIN_STATIC_SCRATCH_BYTES (2u << 20) /* device array behind spin_sparse_decode_static, per GPU */

typedef struct spin_config {
  int32_t max_batch;
  int32_t num_q_heads;          /* multiple of num_kv_heads; group size <= 16 */
  int32_t num_kv_heads;
  int32_t head_dim;             /* 128 */
  int32_t page_tokens;          /* 16 */
  int32_t partition_tokens;     /* divides 16, or a multiple of 16 */
  int32_t score_kind;           /* spin_score_kind; SKETCH needs partition_tokens == 1 */
  int32_t sketch_channels;      /* 16 (SKETCH) */
  int32_t reps_per_partition;   /* REPMAX: 1 (one mean key per partition: a landmark or centroid), 2 or 4 */
  int32_t topk;                 /* partitions per row (tokens when partition_tokens == 1) */
  int32_t topk_includes_forced; /* 1: forced partitions count against topk; 0: they come on top */
  int32_t sink_pages;           /* first pages of a context, always attended */
  int32_t recent_pages;         /* last pages of a context, always attended */
  int32_t max_context;          /* tokens; sizes strides and the workspace */
  int32_t leaf_entries;         /* entries per second-level table chunk (512) */
  int32_t lru_timestamps;       /* 0 = all-resident mode; n > 0 = bucketed LRU with n timestamp values (n <= 256) */
  int32_t lru_evict_exact;      /* 0 = evict whole buckets <= x; 1 = only as many pages of bucket x as needed */
  int32_t lru_policy;           /* budget mode: 0 = bucketed LRU (Section 5.3); 1 = 8-way set-associative placement:
                                   home set = mix32(row, page) mod (slots / 8), see spin_resolve_slots */
  int32_t decode_splits;        /* split-K factor of spin_sparse_decode; 0 = choose from the shape */
  int32_t decode_waves;         /* wavefronts per decode workgroup: 2, 4 or 8; 0 = 8 */
  int32_t decode_depth;         /* page buffers per decode wavefront (pages in flight + 1): 2, 3 or 4; 0 = choose */
  int32_t score_tiles_per_wg;   /* 16-row summary tiles per stage-1 workgroup; 0 = choose */
  int32_t score_waves;          /* wavefronts per stage-1 workgroup: 1, 2, 4 or 8; 0 = 4 */
  int32_t variable_partitions;  /* 1: strides are sized for spin_set_partition_tables (partitions of 1 page up to
                                   partition_tokens tokens) */
  float softmax_scale;          /* 0 = 1/sqrt(head_dim) */
} spin_config;

/* Create / destroy the host-side context.  `*out` is set only on SPIN_OK. */
int spin_create(const spin_config *cfg, spin_ctx **out);
void spin_destroy(spin_ctx *ctx);
const char *spin_status_string(int status);

/* Sizes the caller needs to allocate buffers. */
size_t spin_workspace_bytes(const spin_ctx *ctx); /* DEVICE scratch, 256-byte aligned */
int32_t spin_sel_stride(const spin_ctx *ctx);     /* entries per row of `sel` */
int32_t spin_page_stride(const spin_ctx *ctx);    /* entries per row of slots / page_ids / valid_mask */
int32_t spin_dir_stride(const spin_ctx *ctx);     /* entries per row of `dir` */
int32_t spin_decode_splits(const spin_ctx *ctx);  /* the split-K factor in use */
/* bytes of the summary array for `padded_partitions` = part_offsets[batch] */
size_t spin_summary_bytes(const spin_ctx *ctx, int64_t padded_partitions);

/* Clear the workspace's status word and arrival counters (a fill kernel on
 * `stream`; call once after allocating the workspace, whenever a reported device
 * fault was handled, and after a launch was abandoned mid-way). */
int spin_workspace_init(spin_ctx *ctx, void *workspace, void *stream);
/* Synchronise `stream` and return the first device-detected fault since the
 * last init (SPIN_OK if none). */
int spin_poll_status(spin_ctx *ctx, const void *workspace, void *stream);

/* Variable-length partitions (Section 5.2: the Meta-partition table keeps each
 * partition's token count, the Partition Offset table where its page list
 * starts; Section 4.1: a partition may be a block or a cluster of any size).
 * Registers three DEVICE tables, all indexed like `scores` (entry
 * num_kv_heads*part_offsets[b] + h*PP_b + p for partition p of row (b,h)):
 *   part_count      int32 [rows]  partitions of the row
 *   part_first_page int32         first logical page of the partition; partitions own
 *                                 whole pages, ascend, and follow one another without gaps
 *   part_tokens     int32         tokens in the partition (1 .. cfg.partition_tokens); only
 *                                 its last page may be partly filled
 * From then on Index, stage 2 and stage 3 (and spin_select_resolve) take a row's
 * partitions from these tables instead of cutting the context every
 * cfg.partition_tokens tokens: cfg.partition_tokens is then the LARGEST partition
 * (it sizes the strides) and seq_lens is not consulted by stages 2 and 3.  Sink and
 * recent pages are the first / last pages of the row's page list.  Supported for
 * MINMAX scores and for REPMAX with one representative (the mean key of the partition's
 * tokens: a cluster's centroid), in all-resident and in budget mode, rows of at most
 * 65536 partitions.  Passing
 * NULL for the three tables returns to uniform partitions.  The pointers are kept,
 * not copied: the tables must outlive the calls that use them.
 * SPIN_ERR_UNSUPPORTED unless the context was created with variable_partitions = 1.  While
 * tables are registered, spin_append_kv and spin_alloc_leaves (which find a partition's
 * pages from its id alone) return SPIN_ERR_UNSUPPORTED. */
int spin_set_partition_tables(spin_ctx *ctx, const int32_t *part_offsets, const int32_t *part_count,
                              const int32_t *part_first_page, const int32_t *part_tokens);

/* Offload, layout half: write `n_pages` pages given in plain token-major order
 * (src_k, src_v: DEVICE bf16 [n_pages][16][128]) into pool slots `slots[i]`
 * (DEVICE int32 [n_pages], each in [0, pool_slots)) in the slot layout above.  A page whose
 * slot lies outside the pool is skipped without a report (the call takes no workspace). */
int spin_pack_kv_pages(spin_ctx *ctx, int64_t n_pages, const void *src_k, const void *src_v,
                       const int32_t *slots, void *kv_pool, int64_t pool_slots, void *stream);

/* Index: build the summaries of every partition of every row from the keys in
 * the pool, reached through the two-level table (every page must be resident).
 * MINMAX: elementwise min and max key over the partition's valid tokens (keys must be finite; where a
 *         channel holds both -0 and +0 inside one partition, which zero is stored is unspecified).
 * REPMAX: mean key of each of the R equal sub-ranges, rounded to bf16 (an empty
 *         sub-range of a ragged last partition repeats representative 0).
 * SKETCH: the key restricted to chan_idx[h][0..C) (DEVICE int32 [num_kv_heads][C]).
 * Rows of a tile beyond the row's last partition are zero-filled. */
int spin_build_summaries(spin_ctx *ctx, int32_t batch, const void *kv_pool, int64_t pool_slots,
                         const int32_t *dir, const int32_t *leaf_pool, int64_t leaf_chunks,
                         const int32_t *part_offsets, const int32_t *seq_lens,
                         const int32_t *chan_idx, void *summaries, void *workspace, void *stream);

/* Index at decode time (Section 4.1: Index also runs during decode to take in
 * newly generated tokens).  Appends ONE token per request: k_new / v_new are
 * DEVICE bf16 [batch][num_kv_heads][128]; seq_lens (DEVICE int32 [batch]) holds
 * the lengths BEFORE the append, so the token lands at position seq_lens[b].
 * Its page must already have a slot in the table (the caller maps a fresh slot
 * when the position starts a new page) and part_offsets must leave room for its
 * partition; otherwise SPIN_ERR_NOT_RESIDENT / SPIN_ERR_INVALID is raised in the
 * status word and the row is left untouched.  The K/V values are written into
 * the slot and the summaries of the partition are updated to exactly what
 * spin_build_summaries would store for the longer context.  The caller then
 * increments its seq_lens. */
int spin_append_kv(spin_ctx *ctx, int32_t batch, const void *k_new, const void *v_new,
                   const int32_t *seq_lens, void *kv_pool, int64_t pool_slots, const int32_t *dir,
                   const int32_t *leaf_pool, int64_t leaf_chunks, const int32_t *part_offsets,
                   const int32_t *chan_idx, void *summaries, void *workspace, void *stream);

/* Stage 1.  scores[row][p] (DEVICE fp32, indexed like the summaries) =
 *   MINMAX  max_g sum_d max(q[g][d]*min[p][d], q[g][d]*max[p][d])
 *   SKETCH  max_g sum_c q[g][chan_idx[h][c]] * sketch[t][c]
 *   REPMAX  max_g max_r q[g] . rep[p][r]
 * over the G query heads of the row's group; bf16 inputs, exact products, fp32
 * accumulation on the matrix cores.  Entries beyond a row's partition count are
 * unspecified.  Summaries must be finite: the kernels pair some summary values
 * with exact zeros of the query-side operand (MINMAX: max[d] with max(q[d], 0),
 * min[d] with min(q[d], 0)), and 0 x inf makes the sum of that head NaN where
 * the definition has a finite term.  The maximum over the group's heads drops
 * NaN operands, so such a partition (SKETCH with groups of up to four heads:
 * each of the up to 64 tokens scored together) scores as the best of its other
 * heads, -inf when none is left, and stage 2 ranks it accordingly. */
int spin_score_partitions(spin_ctx *ctx, int32_t batch, const void *q, const void *summaries,
                          const int32_t *chan_idx, const int32_t *part_offsets,
                          const int32_t *seq_lens, float *scores, void *workspace, void *stream);

/* Stage 2.  Per row: the forced partitions (all of whose pages are sink or
 * recent pages) plus the k' best-scoring other partitions, k' = topk - forced
 * (topk_includes_forced) or topk; ties go to the lower id, +0 and -0 tie, NaN
 * ranks lowest.  sel (DEVICE int32 [rows][sel_stride]) ascending, padded with
 * -1; nsel (DEVICE int32 [rows]).  Contexts configured for rows of 16385 to
 * 131072 partitions run two launches (a histogram of the leading key bits kept
 * in `workspace`, then the selection); the workspace must have been cleared by
 * spin_workspace_init once and is left cleared. */
int spin_select_topk(spin_ctx *ctx, int32_t batch, const float *scores, const int32_t *part_offsets,
                     const int32_t *seq_lens, int32_t *sel, int32_t *nsel, void *workspace,
                     void *stream);

/* Pinned partitions (Section 4.2: outliers found by an algorithm's Index, like the
 * recent window, always participate in attention).  Run between stages 1 and 2:
 * pinned (DEVICE int32 [rows][pinned_stride]) lists npinned[row] (DEVICE int32
 * [rows]) partition ids per row, in any order; their scores become +inf, so stage
 * 2 takes them before every other candidate (they count against k'; ties among
 * +inf scores go to the lower id) and, under a budget, stage 3b keeps their pages
 * resident because they are selected in every step.  Ids outside the row are
 * ignored; forced partitions are unaffected (they are no candidates). */
int spin_pin_partitions(spin_ctx *ctx, int32_t batch, float *scores, const int32_t *part_offsets,
                        const int32_t *pinned, const int32_t *npinned, int32_t pinned_stride, void *stream);

/* Stages 1 and 2 in ONE call: arguments and results are exactly those of
 * spin_score_partitions followed by spin_select_topk, bit for bit (the scores
 * are still written).  With contexts whose stage 2 takes two
 * launches (rows of 16385 to 131072 uniform partitions) stage 1 counts the leading key
 * bits of its scores while it still holds them, so the histogram launch over
 * the score array is saved; every other configuration simply runs the two
 * stages one after the other.  The workspace is needed as for the two calls.
 * (Pinned partitions go between the two stages: use the separate calls then.) */
int spin_score_select_topk(spin_ctx *ctx, int32_t batch, const void *q, const void *summaries,
                           const int32_t *chan_idx, const int32_t *part_offsets, const int32_t *seq_lens,
                           float *scores, int32_t *sel, int32_t *nsel, void *workspace, void *stream);

/* Stage 3.  Expand each row's selection (plus forced pages that lie in no
 * selected partition) to logical pages, walk dir -> leaf -> slot, and emit, in
 * ascending page order, slots / page_ids (DEVICE int32 [rows][page_stride]),
 * valid_mask (DEVICE uint16, bit t = token t of the page is attended) and
 * npages (DEVICE int32 [rows]).
 * All-resident mode (lru_timestamps == 0): rev_table, slot_range, miss_* are
 * NULL; a missing leaf or slot sets SPIN_ERR_NOT_RESIDENT and drops the page.
 * Budget mode (lru_timestamps == n): row r owns the slot_range[r][1] pool slots
 * starting at slot_range[r][0] (DEVICE int32 [rows][2]; ranges of different rows
 * must not overlap; spin_reclaim_tail changes the counts); rev_table (DEVICE
 * int32 [total slots][2] = {resident logical page or -1, timestamp}) and the
 * leaf entries are updated by the four bucketed-LRU steps; missed pages are
 * admitted to freed slots (ascending page id -> ascending free slot) and
 * listed in miss_pages / miss_slots (DEVICE int32 [rows][page_stride]) with
 * nmiss (DEVICE int32 [rows]) for the copy that must complete before stage 4.
 * Leaves must exist for every page range a row can select.  The policies work
 * on pages: with partitions other than one page each (blocks, tokens,
 * variable-length) the selection is first expanded to its page list and masks
 * as in all-resident mode, then replacement runs on that list.
 * Budget mode with lru_policy == 1 (the budget workload's "8-way buckets hashed
 * on (request, page)"; a convention of this library, not the paper's policy):
 * the row's slots form slot_range[r][1] / 8 sets of 8 consecutive slots (slots
 * past the last whole set are not used for placement); the home set of page p
 * is mix32(r, p) mod sets with mix32(r, p) = f(r * 0x9E3779B1 + p) in 32-bit
 * arithmetic, f(x): x ^= x >> 16; x *= 0x85EBCA6B; x ^= x >> 13; x *= 0xC2B2AE35;
 * x ^= x >> 16.  Misses are placed as if one at a time in ascending page id:
 * from the home set on, sets whose 8 ways all hold pages selected in this step
 * are skipped circularly; in the set reached the lowest empty way is taken,
 * else the way not selected in this step with the smallest timestamp (lowest
 * way on ties) is evicted.  Timestamps and every output are as above; at most
 * 32768 slots per row.
 * `step` is the decode step (>= 0) the timestamps are taken from.  A launch that is
 * recorded once and replayed (a HIP graph) would freeze that value: pass
 * SPIN_STEP_FROM_WORKSPACE instead and the kernel reads the workspace's own step
 * counter, which spin_workspace_init zeroes, spin_set_step sets and
 * spin_advance_step increments (small kernels on `stream`, recordable too). */
#define SPIN_STEP_FROM_WORKSPACE (-1)
int spin_resolve_slots(spin_ctx *ctx, int32_t batch, int32_t step, const int32_t *sel,
                       const int32_t *nsel, const int32_t *seq_lens, const int32_t *dir,
                       int32_t *leaf_pool, int64_t leaf_chunks, int32_t *rev_table,
                       const int32_t *slot_range, int32_t *slots, int32_t *page_ids,
                       uint16_t *valid_mask, int32_t *npages, int32_t *miss_pages,
                       int32_t *miss_slots, int32_t *nmiss, void *workspace, void *stream);

int spin_set_step(spin_ctx *ctx, void *workspace, int32_t step, void *stream);
int spin_advance_step(spin_ctx *ctx, void *workspace, void *stream);

/* Stages 2 and 3 together (all-resident mode): ONE launch for rows of at most 16384
 * partitions; for uniform partitions, rows of up to 131072 partitions take stage 2's
 * histogram launch first and the launch that finishes stage 2 resolves.  Anything
 * else is SPIN_ERR_UNSUPPORTED before a kernel is issued, and the two calls above apply.
 * Arguments and results are exactly those of spin_select_topk followed by
 * spin_resolve_slots, bit for bit: the workgroup that selected a row resolves it. */
int spin_select_resolve(spin_ctx *ctx, int32_t batch, const float *scores, const int32_t *part_offsets,
                        const int32_t *seq_lens, int32_t *sel, int32_t *nsel, const int32_t *dir,
                        const int32_t *leaf_pool, int64_t leaf_chunks, int32_t *slots, int32_t *page_ids,
                        uint16_t *valid_mask, int32_t *npages, void *workspace, void *stream);

/* Stages 1, 2 and 3 in two launches: spin_score_partitions (taking stage 2's first
 * histogram along where spin_score_select_topk would) followed by spin_select_resolve.
 * Arguments, results and refusals are those of the stage calls, bit for bit. */
int spin_score_select_resolve(spin_ctx *ctx, int32_t batch, const void *q, const void *summaries,
                              const int32_t *chan_idx, const int32_t *part_offsets, const int32_t *seq_lens,
                              float *scores, int32_t *sel, int32_t *nsel, const int32_t *dir,
                              const int32_t *leaf_pool, int64_t leaf_chunks, int32_t *slots, int32_t *page_ids,
                              uint16_t *valid_mask, int32_t *npages, void *workspace, void *stream);

/* Stages 2+3 with the always-attended pages attended on the side, and the stage 4 that goes
 * with it.  A row's sink and recent pages do not depend on the selection (Section 4.2: such
 * windows always take part in attention), and stages 2+3 occupy one workgroup per row and leave
 * the memory system idle.  spin_select_resolve_forced is spin_select_resolve (same arguments,
 * same results, bit for bit) whose launch carries a second set of workgroups: one per row
 * or a few per row look the row's sink and recent pages up in the two-level table, attend them
 * (q, kv_pool as in spin_sparse_decode) and leave their partial results per query head in
 * `workspace`, together with the number of leading and trailing entries of the row's page list
 * these pages are.
 * spin_sparse_decode_rest is spin_sparse_decode over the remaining entries of the same page
 * list; the first wavefronts of the row's splits start from those partials, so each takes a
 * fixed place in the summation order.  It must follow
 * spin_select_resolve_forced of the same step, on the same stream and workspace, with the same
 * q and kv_pool.  out and lse are stage 4's results to its tolerance (the summation order
 * differs from spin_sparse_decode's, so the bits may), identical from run to run.
 * Supported in all-resident mode with uniform partitions of whole pages, rows of at most 4096
 * partitions and 1 to 1024 sink + recent pages; SPIN_ERR_UNSUPPORTED otherwise, before anything
 * is launched (the plain calls then apply). */
int spin_select_resolve_forced(spin_ctx *ctx, int32_t batch, const float *scores, const int32_t *part_offsets,
                               const int32_t *seq_lens, int32_t *sel, int32_t *nsel, const int32_t *dir,
                               const int32_t *leaf_pool, int64_t leaf_chunks, int32_t *slots, int32_t *page_ids,
                               uint16_t *valid_mask, int32_t *npages, const void *q, const void *kv_pool,
                               int64_t pool_slots, void *workspace, void *stream);
int spin_sparse_decode_rest(spin_ctx *ctx, int32_t batch, const void *q, const void *kv_pool,
                            int64_t pool_slots, const int32_t *slots, const uint16_t *valid_mask,
                            const int32_t *npages, void *out, float *lse, void *workspace, void *stream);

/* Buffer elasticity, mechanism only (Section 5.3: buffer pages are reclaimed from
 * the tail of a request's GPU page table).  Sets the slot count of every row to
 * new_count[r] (DEVICE int32 [rows]): pages resident in slots at or beyond the
 * new count are evicted (forward entry cleared, slot marked empty) and
 * slot_range[r][1] is updated in place.  Growing only raises the count; the added
 * slots must belong to the row and be empty in rev_table.  Which rows give up how
 * many slots is the serving scheduler's policy and not part of this library. */
int spin_reclaim_tail(spin_ctx *ctx, int32_t batch, int32_t *slot_range, const int32_t *new_count,
                      const int32_t *dir, int32_t *leaf_pool, int64_t leaf_chunks, int32_t *rev_table,
                      void *workspace, void *stream);

/* On-demand second-level tables (Section 5.4: segments come from a pre-allocated
 * GPU-resident pool managed by a bitmap allocator, so metadata grows with the
 * mapped pages).  spin_alloc_leaves makes sure a leaf chunk exists for every page
 * range that a row's current selection (and its forced pages) touches: missing
 * ones are taken from leaf_pool by setting a bit of leaf_bitmap (DEVICE uint32
 * [ceil(leaf_chunks/32)], bit c = chunk c in use), filled with -1 and entered in
 * `dir`.  Run it between stage 2 and a budget-mode stage 3.  SPIN_ERR_LEAF_POOL is
 * raised when the pool is exhausted.  spin_free_leaves returns every chunk of the
 * given rows to the pool (for a request that left; its pages must no longer be
 * resident) and clears their directory entries.  Which chunk a range receives
 * depends on arrival order; slots and page ids never do. */
int spin_alloc_leaves(spin_ctx *ctx, int32_t batch, const int32_t *sel, const int32_t *nsel,
                      const int32_t *seq_lens, int32_t *dir, int32_t *leaf_pool, int64_t leaf_chunks,
                      uint32_t *leaf_bitmap, void *workspace, void *stream);
int spin_free_leaves(spin_ctx *ctx, int32_t batch, int32_t *dir, int64_t leaf_chunks, uint32_t *leaf_bitmap,
                     void *workspace, void *stream);

/* CPU page table (Section 5.2: the Partition Offset table says where a partition's
 * page list starts in the CPU page table, a flat array of physical CPU page ids).
 * Without one, page p of row r lives at page host_row_base[r] + p of the pinned
 * host pool.  With one registered, that sum is an OFFSET into cpu_pages
 * (int32 [entries], in pinned host memory so that both the copy kernel and
 * spin_copy_misses_host read it), and the entry there is the physical host page
 * (in [0, host_pages)): a request's pages may lie anywhere in the host pool, e.g.
 * as they were allocated while its context grew.  Applies to
 * spin_gather_misses, spin_offload_pages and spin_copy_misses_host; an offset or
 * entry out of range raises SPIN_ERR_SLOT_RANGE (SPIN_ERR_INVALID from the
 * host-driven copier) and skips the page.  NULL returns to the identity; host_pages > 0
 * then still registers the size of the host pool, so that both copiers refuse a page
 * outside it in the same way (with host_pages == 0 the identity mapping is unchecked and
 * host_row_base / the page lists are the caller's responsibility).  The pointer is kept,
 * not copied. */
int spin_set_host_page_table(spin_ctx *ctx, const int32_t *cpu_pages, int64_t entries, int64_t host_pages);

/* Retrieve steps 3-4 (Section 5.2), after budget-mode stage 3: copy every missed
 * page into the slot assigned to it.  The full KV lives in pinned host memory as
 * pages in the slot layout; page `p` of row r is page host_row_base[r] + p.
 *
 * spin_copy_misses_host: host-driven.  nmiss / miss_pages / miss_slots and
 * host_row_base (int64 [rows]) are HOST copies; one 8 KiB hipMemcpyAsync per
 * miss is issued on `copy_stream`; *pages_copied (may be NULL) gets the count.
 * The caller orders the copies before stage 4 (event on copy_stream).
 *
 * spin_gather_misses: device-driven copy kernel (Section 5.5: one wavefront
 * per page, pages spread over all wavefronts regardless of owner).  host_kv is
 * the device-visible address of the pinned buffer; row_base, nmiss, miss_pages,
 * miss_slots are DEVICE arrays (stage 3's outputs, untouched by the host);
 * enqueued on `stream`, so stage 4 on the same stream simply follows it. */
int spin_copy_misses_host(spin_ctx *ctx, int32_t batch, const void *host_kv, const int64_t *host_row_base,
                          const int32_t *nmiss, const int32_t *miss_pages, const int32_t *miss_slots,
                          void *kv_pool, int64_t pool_slots, void *copy_stream, int64_t *pages_copied);
int spin_gather_misses(spin_ctx *ctx, int32_t batch, const void *host_kv, const int64_t *row_base,
                       const int32_t *nmiss, const int32_t *miss_pages, const int32_t *miss_slots,
                       void *kv_pool, int64_t pool_slots, void *workspace, void *stream);

/* Offload's copy (Table 1: copy(gpu_kv, cpu_kv, map); Section 4.1 Offload), the
 * copy kernel run the other way: for every row r write the pages listed in
 * pages[r][0 .. count[r]) from the slots slots[r][...] to the pinned host copy
 * (page p of row r is host page row_base[r] + p).  count (DEVICE int32 [rows]),
 * pages / slots (DEVICE int32 [rows][page_stride]) have the shape of stage 3's
 * page or miss lists, so those can be passed as they are; host_kv is the
 * device-visible address of the pinned buffer.  Used at decode time to write a
 * page back once its last token has been appended, before it can be evicted.
 * Tables are not touched. */
int spin_offload_pages(spin_ctx *ctx, int32_t batch, const void *kv_pool, int64_t pool_slots, void *host_kv,
                       const int64_t *row_base, const int32_t *count, const int32_t *pages,
                       const int32_t *slots, void *workspace, void *stream);

/* Stage 4.  out[b][hq] (DEVICE bf16 [batch][num_q_heads][128]) =
 * softmax(scale * q K_S^T) V_S over the tokens whose mask bit is set in the
 * row's resolved pages; fp32 online softmax, split over the page list and
 * merged in a fixed order.  lse (DEVICE fp32 [batch][num_q_heads], natural log;
 * may be NULL).  A row with no valid token gives out = 0, lse = -inf.
 * Only the bytes of attended tokens are fetched: a page with a partial mask
 * loads the K rows and V quads its mask names; with partition_tokens < 16
 * (token-major slots) the attended tokens of all pages are gathered 16 at a
 * time into one matrix tile, 512 bytes per token. */
int spin_sparse_decode(spin_ctx *ctx, int32_t batch, const void *q, const void *kv_pool,
                       int64_t pool_slots, const int32_t *slots, const uint16_t *valid_mask,
                       const int32_t *npages, void *out, float *lse, void *workspace,
                       void *stream);

/* Stage 4 in two passes, for a step whose missed pages are still being copied (Section 5.2,
 * Retrieve: pages that hit are in HBM already; Section 3.1, Eq. 3: the copy is the long term of a
 * step under a budget).  spin_split_hits_misses splits the token masks of stage 3b's page list
 * into two of the same shape (DEVICE uint16 [rows][page_stride]): mask_hits keeps the mask of every
 * page that is not in the row's miss list, mask_misses that of every page that is.
 * spin_sparse_decode_begin attends what its masks name and leaves one partial result per query
 * head in `workspace`; spin_sparse_decode_finish, later on the same stream and workspace, attends
 * what ITS masks name starting from that partial and writes out / lse as spin_sparse_decode does
 * (same tolerance; the summation order differs, the bits are the same from run to run).  Between
 * the two the caller makes its stream wait for the copy.  Slots of whole pages only
 * (partition_tokens >= 16); SPIN_ERR_UNSUPPORTED otherwise. */
int spin_split_hits_misses(spin_ctx *ctx, int32_t batch, const int32_t *page_ids, const uint16_t *valid_mask,
                           const int32_t *npages, const int32_t *miss_pages, const int32_t *nmiss,
                           uint16_t *mask_hits, uint16_t *mask_misses, void *stream);
int spin_sparse_decode_begin(spin_ctx *ctx, int32_t batch, const void *q, const void *kv_pool, int64_t pool_slots,
                             const int32_t *slots, const uint16_t *valid_mask, const int32_t *npages,
                             void *workspace, void *stream);
int spin_sparse_decode_finish(spin_ctx *ctx, int32_t batch, const void *q, const void *kv_pool, int64_t pool_slots,
                              const int32_t *slots, const uint16_t *valid_mask, const int32_t *npages, void *out,
                              float *lse, void *workspace, void *stream);

/* Stage 4 for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc and so cannot provide the workspace of
 * spin_sparse_decode.  Same inputs, outputs and output bits as spin_sparse_decode (the same
 * kernels run); the split-K scratch (row tickets and workgroup partials) lives in a device array
 * of SPIN_STATIC_SCRATCH_BYTES that is part of the library image: each GPU the library runs on
 * holds it until the process ends.  The call allocates and frees nothing and enqueues a small
 * clearing kernel plus the attention kernel on `stream`.  The array's device address is looked
 * up once per device: by spin_create for the device that is current then, otherwise by the
 * first call on that device.
 * A call needs 256 + 4 * rows + 8 * P + 512 * P bytes of it (each term rounded up to 256), with
 * rows = batch * num_kv_heads and P = rows * (2 * spin_decode_splits(ctx)) * (num_q_heads /
 * num_kv_heads) at most (the workspace's layout of partials is kept); a larger shape returns SPIN_ERR_STATIC_LIMIT before anything is launched.
 * status (DEVICE int32, may be NULL): receives the first device-detected fault (a slot id
 * outside the pool: SPIN_ERR_SLOT_RANGE) if it held 0 before; the caller clears and reads it.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 * streams, or different host threads) race and must be serialised by the caller. */
int spin_sparse_decode_static(spin_ctx *ctx, int32_t batch, const void *q, const void *kv_pool,
                              int64_t pool_slots, const int32_t *slots, const uint16_t *valid_mask,
                              const int32_t *npages, void *out, float *lse, int32_t *status,
                              void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SPIN_H */
