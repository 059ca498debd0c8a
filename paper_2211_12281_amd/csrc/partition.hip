// Partition bucketing (arXiv 2211.12281, Section 4 "Partitioning"): stable counting sort of the
// triples by (shard of head, shard of tail), built on the radix-sort passes of the sparse update.
#include "kge_internal.h"

size_t kge_sort_ws(int64_t M);
int kge_sort_pairs(const int32_t *idx, const int32_t *h, const int32_t *t, int64_t part_size, int D, int64_t M,
                   int64_t key_range, void *ws, const uint32_t **sk, const uint32_t **sp, hipStream_t st);

namespace {

// sorted bucket keys -> exclusive bucket offsets; order = sorted positions widened to 64 bits
__global__ void bucket_offsets_kernel(const uint32_t *sk, const uint32_t *sp, int64_t n, int nb, int64_t *offsets,
                                      int64_t *order) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    order[i] = (int64_t)sp[i];
    const int64_t cur = sk[i];
    const int64_t prev = i > 0 ? (int64_t)sk[i - 1] : -1;
    for (int64_t b = prev + 1; b <= cur; ++b) offsets[b] = i;      // buckets that start here (empty ones included)
    if (i == n - 1) for (int64_t b = cur + 1; b <= nb; ++b) offsets[b] = n;
}

__global__ void bucket_offsets_empty_kernel(int nb, int64_t *offsets) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b <= nb) offsets[b] = 0;
}

}  // namespace

size_t kge_partition_ws(int64_t n, int D) {
    (void)D;
    if (n < 0 || n >= (1ll << 31)) return 0;
    return kge_sort_ws(n);
}

int kge_run_partition(const int32_t *h, const int32_t *t, int64_t n, int64_t part_size, int D, int64_t *offsets,
                      int64_t *order, void *ws, size_t ws_bytes, hipStream_t st) {
    (void)ws_bytes;
    const int nb = D * D;
    if (n == 0) {
        hipLaunchKernelGGL(bucket_offsets_empty_kernel, dim3((nb + 256) / 256), dim3(256), 0, st, nb, offsets);
        return kge_launch_status();
    }
    const uint32_t *sk, *sp;
    int rc = kge_sort_pairs(nullptr, h, t, part_size, D, n, nb, ws, &sk, &sp, st);
    if (rc != KGE_OK) return rc;
    hipLaunchKernelGGL(bucket_offsets_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, sk, sp, n, nb, offsets, order);
    return kge_launch_status();
}
