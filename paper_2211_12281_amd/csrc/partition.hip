// Partition bucketing (arXiv 2211.12281, Section 4 "Partitioning"): stable counting sort of the
// triples by (shard of head, shard of tail), built on the radix-sort passes of the sparse update.
#include "kge_internal.h"

size_t kge_sort_ws(int64_t M);
int kge_sort_pairs(const int32_t *idx, const int32_t *h, const int32_t *t, int64_t part_size, int D, int64_t M,
                   int64_t key_range, void *ws, const uint32_t **sk, const uint32_t **sp, hipStream_t st,
                   const int32_t *r, int64_t n_rel);

namespace {

// sorted bucket keys -> exclusive bucket offsets; order = sorted positions widened to 64 bits
__global__ void bucket_offsets_kernel(const uint32_t *sk, const uint32_t *sp, int64_t n, int64_t nb, int64_t *offsets,
                                      int64_t *order) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    order[i] = (int64_t)sp[i];
    const int64_t cur = sk[i];
    const int64_t prev = i > 0 ? (int64_t)sk[i - 1] : -1;
    for (int64_t b = prev + 1; b <= cur; ++b) offsets[b] = i;      // buckets that start here (empty ones included)
    if (i == n - 1) for (int64_t b = cur + 1; b <= nb; ++b) offsets[b] = n;
}

__global__ void bucket_offsets_empty_kernel(int64_t nb, int64_t *offsets) {
    const int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
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
        hipLaunchKernelGGL(bucket_offsets_empty_kernel, dim3((nb + 256) / 256), dim3(256), 0, st, (int64_t)nb, offsets);
        return kge_launch_status();
    }
    const uint32_t *sk, *sp;
    int rc = kge_sort_pairs(nullptr, h, t, part_size, D, n, nb, ws, &sk, &sp, st, nullptr, 0);
    if (rc != KGE_OK) return rc;
    hipLaunchKernelGGL(bucket_offsets_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, sk, sp, n, (int64_t)nb, offsets, order);
    return kge_launch_status();
}

// ---------------------------------------------------------------------------------------------
// Relation-aware triple sampler (Section 4, "Training"): inside bucket T_ij a triple is drawn with
// p((h, r, t)) = (1 / n_r) * cbrt(n_r) / sum_r' cbrt(n_r'), n_r = triples of relation r in the bucket
// ---------------------------------------------------------------------------------------------
namespace {

// w(n) = floor(2^20 * n^(1/3)): the largest integer whose cube does not exceed n * 2^60 (exact, so that
// every implementation of the sampler draws from the same table); n < 2^32, so w < 2^32
__device__ uint64_t cbrt_weight(uint64_t n) {
    const unsigned __int128 target = (unsigned __int128)n << 60;
    uint64_t w = 0;
    for (int bit = 31; bit >= 0; --bit) {
        const uint64_t c = w | (1ull << bit);
        if ((unsigned __int128)c * c * c <= target) w = c;
    }
    return w;
}

// one workgroup per bucket: inclusive prefix sums of the relations' weights
__global__ void sampler_cdf_kernel(const int64_t *rel_offsets, int64_t n_rel, uint64_t *cdf) {
    __shared__ uint64_t part[256];
    const int64_t b = blockIdx.x;
    const int64_t per = (n_rel + 255) / 256;
    const int64_t lo = threadIdx.x * per, hi = lo + per < n_rel ? lo + per : n_rel;
    uint64_t s = 0;
    for (int64_t q = lo; q < hi; ++q) {
        const int64_t g = b * n_rel + q;
        s += cbrt_weight((uint64_t)(rel_offsets[g + 1] - rel_offsets[g]));
    }
    part[threadIdx.x] = s;
    __syncthreads();
    for (int o = 1; o < 256; o <<= 1) {
        const uint64_t v = threadIdx.x >= (unsigned)o ? part[threadIdx.x - o] : 0ull;
        __syncthreads();
        part[threadIdx.x] += v;
        __syncthreads();
    }
    uint64_t run = threadIdx.x ? part[threadIdx.x - 1] : 0ull;
    for (int64_t q = lo; q < hi; ++q) {
        const int64_t g = b * n_rel + q;
        run += cbrt_weight((uint64_t)(rel_offsets[g + 1] - rel_offsets[g]));
        cdf[g] = run;
    }
}

__device__ __forceinline__ void philox_round(uint32_t (&c)[4], uint32_t k0, uint32_t k1) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c[0]), lo0 = 0xD2511F53u * c[0];
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c[2]), lo1 = 0xCD9E8D57u * c[2];
    const uint32_t n0 = hi1 ^ c[1] ^ k0, n2 = hi0 ^ c[3] ^ k1;
    c[0] = n0; c[1] = lo1; c[2] = n2; c[3] = lo0;
}
__device__ __forceinline__ void philox4x32_10(uint32_t (&c)[4], uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) { philox_round(c, k0, k1); k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
}

// one thread per draw q: counter (q_lo, q_hi, step, tag); x = w1:w0 picks the relation as the first one whose
// cdf exceeds floor(x * total / 2^64), y = w3:w2 the triple floor(y * n_r / 2^64) of its group
__global__ void sample_triples_kernel(uint32_t seed_lo, uint32_t seed_hi, uint32_t step, uint32_t tag, int64_t bucket_lo,
                                      int64_t draws, int64_t per_bucket, int64_t n_rel, const int64_t *rel_offsets,
                                      const uint64_t *cdf, const int64_t *order, const int32_t *h, const int32_t *r,
                                      const int32_t *t, int64_t *out_pos, int32_t *out_h, int32_t *out_r, int32_t *out_t) {
    const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= draws) return;
    const int64_t b = bucket_lo + q / per_bucket;
    const uint64_t *c = cdf + b * n_rel;
    const uint64_t total = c[n_rel - 1];
    int64_t pos = -1;
    if (total > 0) {
        uint32_t w[4] = { (uint32_t)q, (uint32_t)((uint64_t)q >> 32), step, tag };
        philox4x32_10(w, seed_lo, seed_hi);
        const uint64_t x = ((uint64_t)w[1] << 32) | w[0], y = ((uint64_t)w[3] << 32) | w[2];
        const uint64_t pick = __umul64hi(x, total);
        int64_t lo = 0, hi = n_rel - 1;                     // first relation with c[rel] > pick (c[n_rel-1] = total > pick)
        while (lo < hi) {
            const int64_t mid = (lo + hi) >> 1;
            if (c[mid] > pick) hi = mid; else lo = mid + 1;
        }
        const int64_t g = b * n_rel + lo;
        const uint64_t cnt = (uint64_t)(rel_offsets[g + 1] - rel_offsets[g]);
        pos = order[rel_offsets[g] + (int64_t)__umul64hi(y, cnt)];
    }
    if (out_pos) out_pos[q] = pos;
    if (out_h) { out_h[q] = pos >= 0 ? h[pos] : -1; out_r[q] = pos >= 0 ? r[pos] : -1; out_t[q] = pos >= 0 ? t[pos] : -1; }
}

// slot i belongs to entity shard i / per_shard; generator layout of the plain negative sampler (block i / 2)
__global__ void negatives_sharded_kernel(uint32_t seed_lo, uint32_t seed_hi, uint32_t step, uint32_t tag, int64_t part_size,
                                         int64_t n_ent, int64_t per_shard, int64_t n, int32_t *out) {
    const int64_t blk = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (2 * blk >= n) return;
    uint32_t w[4] = { (uint32_t)blk, (uint32_t)((uint64_t)blk >> 32), step, tag };
    philox4x32_10(w, seed_lo, seed_hi);
    for (int half = 0; half < 2; ++half) {
        const int64_t i = 2 * blk + half;
        if (i >= n) break;
        const int64_t lo = (i / per_shard) * part_size, hi = lo + part_size < n_ent ? lo + part_size : n_ent;
        const uint64_t x = ((uint64_t)w[2 * half + 1] << 32) | w[2 * half];
        out[i] = (int32_t)(lo + (int64_t)__umul64hi(x, (uint64_t)(hi - lo)));
    }
}

}  // namespace

size_t kge_sampler_ws(int64_t n) {
    if (n < 0 || n >= (1ll << 31)) return 0;
    return kge_sort_ws(n);
}

int kge_run_sampler_build(const int32_t *h, const int32_t *r, const int32_t *t, int64_t n, int64_t part_size, int D,
                          int64_t n_rel, int64_t *order, int64_t *rel_offsets, uint64_t *cdf, void *ws, hipStream_t st) {
    const int64_t groups = (int64_t)D * D * n_rel;
    if (n == 0) {
        hipLaunchKernelGGL(bucket_offsets_empty_kernel, dim3((unsigned)((groups + 256) / 256)), dim3(256), 0, st, groups, rel_offsets);
    } else {
        const uint32_t *sk, *sp;
        int rc = kge_sort_pairs(nullptr, h, t, part_size, D, n, groups, ws, &sk, &sp, st, r, n_rel);
        if (rc != KGE_OK) return rc;
        hipLaunchKernelGGL(bucket_offsets_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, sk, sp, n, groups, rel_offsets, order);
    }
    hipLaunchKernelGGL(sampler_cdf_kernel, dim3(D * D), dim3(256), 0, st, rel_offsets, n_rel, cdf);
    return kge_launch_status();
}

int kge_run_sample_triples(uint64_t seed, uint64_t step, uint32_t tag, int64_t bucket_lo, int64_t draws, int64_t per_bucket,
                           int64_t n_rel, const int64_t *rel_offsets, const uint64_t *cdf, const int64_t *order,
                           const int32_t *h, const int32_t *r, const int32_t *t, int64_t *out_pos, int32_t *out_h,
                           int32_t *out_r, int32_t *out_t, hipStream_t st) {
    hipLaunchKernelGGL(sample_triples_kernel, dim3((unsigned)((draws + 255) / 256)), dim3(256), 0, st, (uint32_t)seed,
                       (uint32_t)(seed >> 32), (uint32_t)step, tag, bucket_lo, draws, per_bucket, n_rel, rel_offsets, cdf,
                       order, h, r, t, out_pos, out_h, out_r, out_t);
    return kge_launch_status();
}

int kge_run_negatives_sharded(uint64_t seed, uint64_t step, uint32_t tag, int64_t part_size, int64_t n_ent, int64_t per_shard,
                              int64_t n, int32_t *out, hipStream_t st) {
    hipLaunchKernelGGL(negatives_sharded_kernel, dim3((unsigned)(((n + 1) / 2 + 255) / 256)), dim3(256), 0, st, (uint32_t)seed,
                       (uint32_t)(seed >> 32), (uint32_t)step, tag, part_size, n_ent, per_shard, n, out);
    return kge_launch_status();
}
