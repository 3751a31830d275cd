// Entry points not built yet report SPIN_ERR_UNSUPPORTED.
#include "spin_common.h"

extern "C" int spin_build_summaries(spin_ctx *, int32_t, const void *, int64_t, const int32_t *, const int32_t *,
                                    int64_t, const int32_t *, const int32_t *, const int32_t *, void *, void *,
                                    void *) { return SPIN_ERR_UNSUPPORTED; }
extern "C" int spin_score_partitions(spin_ctx *, int32_t, const void *, const void *, const int32_t *,
                                     const int32_t *, const int32_t *, float *, void *, void *) {
  return SPIN_ERR_UNSUPPORTED;
}
extern "C" int spin_select_topk(spin_ctx *, int32_t, const float *, const int32_t *, const int32_t *, int32_t *,
                                int32_t *, void *, void *) { return SPIN_ERR_UNSUPPORTED; }
extern "C" int spin_resolve_slots(spin_ctx *, int32_t, int32_t, const int32_t *, const int32_t *, const int32_t *,
                                  const int32_t *, int32_t *, int64_t, int32_t *, const int32_t *, int32_t *,
                                  int32_t *, uint16_t *, int32_t *, int32_t *, int32_t *, int32_t *, void *,
                                  void *) { return SPIN_ERR_UNSUPPORTED; }
