// Stages 2 and 3 in one launch (all-resident mode; rows of more than 16384
// partitions take the long-row kernels of stage 2, whose finishing launch resolves).  Both stages work on one row per workgroup, so the workgroup
// that selected a row resolves it straight away: the same device functions run
// as in the two stage calls, the results are the same bits, and one launch with
// its start-up latency chain is saved.
#include "spin_resolve_dev.h"
#include "spin_select_dev.h"

template <int BLOCK, int KPT>
__global__ __launch_bounds__(BLOCK) void spin_select_resolve_kernel(
    const float *__restrict__ scores, const int32_t *__restrict__ part_offsets,
    const int32_t *__restrict__ seq_lens, int Hkv, int tp, int topk, int includes_forced, int sink_pages,
    int recent_pages, int sel_stride, int32_t *sel, int32_t *nsel, const int32_t *dir,
    const int32_t *__restrict__ leaf_pool, int64_t leaf_chunks, int page_stride, int dir_stride, int leaf_entries,
    int32_t *__restrict__ slots, int32_t *__restrict__ page_ids, uint16_t *__restrict__ valid_mask,
    int32_t *__restrict__ npages, int32_t *status, spin_var var) {
  const int row = blockIdx.x;
  const int take = select_reg_row<BLOCK, KPT>(scores, part_offsets, seq_lens, Hkv, tp, topk, includes_forced,
                                                     sink_pages, recent_pages, sel_stride, sel, nsel, row, var);
  __syncthreads();   // the selection was written by this workgroup: visible to all its threads from here
  resolve_row<BLOCK>(row, take, sel, seq_lens, dir, leaf_pool, leaf_chunks, Hkv, tp, sink_pages, recent_pages,
                     sel_stride, page_stride, dir_stride, leaf_entries, slots, page_ids, valid_mask, npages, status, var);
}

// hist_ready: stage 1 of this step has filled the long-row histograms already
static int select_resolve_impl(spin_ctx *ctx, int32_t batch, const float *scores, const int32_t *part_offsets,
                               const int32_t *seq_lens, int32_t *sel, int32_t *nsel, const int32_t *dir,
                               const int32_t *leaf_pool, int64_t leaf_chunks, int32_t *slots, int32_t *page_ids,
                               uint16_t *valid_mask, int32_t *npages, void *workspace, void *stream,
                               bool hist_ready) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch || leaf_chunks <= 0) return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!scores || !part_offsets || !seq_lens || !sel || !nsel || !dir || !leaf_pool || !slots || !page_ids ||
      !valid_mask || !npages)
    return SPIN_ERR_INVALID;
  if (!workspace) return SPIN_ERR_WORKSPACE;
  const spin_config &c = ctx->cfg;
  if (c.lru_timestamps > 0) return SPIN_ERR_UNSUPPORTED;
  const int rows = batch * c.num_kv_heads;
  if (ctx->max_parts > 16384) {
    // long rows: the launch that finishes stage 2 resolves its row (refused where that path does not apply)
    const spin_resolve_args res{dir, leaf_pool, leaf_chunks, slots, page_ids, valid_mask, npages};
    return spin_select_impl(ctx, batch, scores, part_offsets, seq_lens, sel, nsel, workspace, stream, hist_ready, &res);
  }
#define SPIN_SR_ARGS                                                                                          \
  0, (hipStream_t)stream, scores, part_offsets, seq_lens, c.num_kv_heads, c.partition_tokens, c.topk,         \
      c.topk_includes_forced, c.sink_pages, c.recent_pages, ctx->sel_stride, sel, nsel, dir, leaf_pool,       \
      leaf_chunks, ctx->page_stride, ctx->dir_stride, c.leaf_entries, slots, page_ids, valid_mask, npages,    \
      (int32_t *)workspace, ctx->var
  if (ctx->max_parts <= 2048)
    spin_launch(ctx, SPIN_K_SELECT, spin_select_resolve_kernel<512, 4>, dim3((unsigned)rows), dim3(512), SPIN_SR_ARGS);
  else if (ctx->max_parts <= 4096)
    spin_launch(ctx, SPIN_K_SELECT, spin_select_resolve_kernel<512, 8>, dim3((unsigned)rows), dim3(512), SPIN_SR_ARGS);
  else
    spin_launch(ctx, SPIN_K_SELECT, spin_select_resolve_kernel<1024, 16>, dim3((unsigned)rows), dim3(1024),
                SPIN_SR_ARGS);
#undef SPIN_SR_ARGS
  return spin_launch_status();
}

extern "C" int spin_select_resolve(spin_ctx *ctx, int32_t batch, const float *scores, const int32_t *part_offsets,
                                   const int32_t *seq_lens, int32_t *sel, int32_t *nsel, const int32_t *dir,
                                   const int32_t *leaf_pool, int64_t leaf_chunks, int32_t *slots,
                                   int32_t *page_ids, uint16_t *valid_mask, int32_t *npages, void *workspace,
                                   void *stream) {
  return select_resolve_impl(ctx, batch, scores, part_offsets, seq_lens, sel, nsel, dir, leaf_pool, leaf_chunks, slots,
                             page_ids, valid_mask, npages, workspace, stream, false);
}

// Stages 1, 2 and 3 in two launches: spin_score_partitions (which, for long SKETCH rows, counts stage 2's
// first histogram as it goes) followed by spin_select_resolve.  Same results as the three stage calls.
extern "C" int spin_score_select_resolve(spin_ctx *ctx, int32_t batch, const void *q, const void *summaries,
                                         const int32_t *chan_idx, const int32_t *part_offsets,
                                         const int32_t *seq_lens, float *scores, int32_t *sel, int32_t *nsel,
                                         const int32_t *dir, const int32_t *leaf_pool, int64_t leaf_chunks,
                                         int32_t *slots, int32_t *page_ids, uint16_t *valid_mask, int32_t *npages,
                                         void *workspace, void *stream) {
  if (!ctx || batch < 0 || batch > ctx->cfg.max_batch || leaf_chunks <= 0) return SPIN_ERR_INVALID;
  if (batch == 0) return SPIN_OK;
  if (!sel || !nsel || !dir || !leaf_pool || !slots || !page_ids || !valid_mask || !npages) return SPIN_ERR_INVALID;
  if (!workspace) return SPIN_ERR_WORKSPACE;
  const spin_config &c = ctx->cfg;
  const int rows = batch * c.num_kv_heads;
  const bool long_rows = ctx->max_parts > 16384;
  // refuse before stage 1 is issued what the second launch would refuse
  if (c.lru_timestamps > 0 || (long_rows && !(ctx->ws_hist_off && rows <= 65535))) return SPIN_ERR_UNSUPPORTED;
  const bool fuse = long_rows && c.score_kind == SPIN_SCORE_SKETCH;
  int32_t *hist = fuse ? (int32_t *)((char *)workspace + ctx->ws_hist_off) : nullptr;
  const int st = spin_score_impl(ctx, batch, q, summaries, chan_idx, part_offsets, seq_lens, scores, workspace, stream,
                                 hist);
  if (st != SPIN_OK) return st;
  return select_resolve_impl(ctx, batch, scores, part_offsets, seq_lens, sel, nsel, dir, leaf_pool, leaf_chunks, slots,
                             page_ids, valid_mask, npages, workspace, stream, fuse);
}
