// placeholder until the ranking kernels land
#include "kge_internal.h"
size_t kge_topk_ws(const kge_model_t &, int64_t, int64_t, int) { return 256; }
int kge_run_topk(const kge_model_t &, const int32_t *, const int32_t *, int64_t, int64_t, int64_t, int, int32_t *,
                 float *, const int32_t *, int64_t *, void *, size_t, hipStream_t) { return KGE_E_UNSUPPORTED; }
