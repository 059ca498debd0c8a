// Power-rank ensemble of M top-K lists per query (Section 3.2 "Inference", paragraph "Ensemble", eq. (ensemble)):
// s(t) = sum over the models, in model order, of -sgn(p) k^p where t is the k-th entry of the model's list and of
// -[p > 0] (K + 1)^p where the list does not hold t; the K_out entities with the largest s(t) are returned, ties
// to the smaller id.  An entity in no list has the smallest possible score, so only listed entities compete.
// One workgroup per query: the M K entries are packed as (entity, model, rank) keys, sorted in the LDS, every run
// of equal entities is summed by one thread in model order (fp64; the K + 1 possible terms come from the host as
// a kernel argument, so they are the host math library's powers), and the K_out winners are picked one at a time.
#include "kge_internal.h"
#include <math.h>

int kge_run_ensemble(const int32_t *lists, int M, int64_t Q, int K, double p, int K_out, int32_t *out_idx, float *out_score,
                     hipStream_t st);

namespace {

constexpr int ENS_MAX_K = 256, ENS_MAX_M = 128, ENS_MAX_ENTRIES = 8192;    // keys and scores of a query live in the LDS (128 KB)
struct EnsTerms { double rank[ENS_MAX_K]; double absent; };     // rank[k - 1] = -sgn(p) k^p

constexpr uint64_t ENS_PAD = ~0ull;
constexpr double ENS_NONE = -INFINITY;                          // slot that is no candidate (any more)

__device__ __forceinline__ void ens_bitonic(uint64_t *a, int n2) {
    for (int k = 2; k <= n2; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            __syncthreads();
            for (int i = threadIdx.x; i < n2; i += blockDim.x) {
                const int l = i ^ j;
                if (l > i) {
                    const uint64_t x = a[i], y = a[l];
                    const bool up = (i & k) == 0;
                    if ((x > y) == up) { a[i] = y; a[l] = x; }
                }
            }
        }
    __syncthreads();
}

__global__ __launch_bounds__(256) void ens_kernel(const int32_t *lists, int M, int64_t Q, int K, int n2, EnsTerms tm, int K_out,
                                                  int32_t *out_idx, float *out_score) {
    extern __shared__ __attribute__((aligned(16))) char ens_lds[];
    uint64_t *key = (uint64_t *)ens_lds;                        // [n2] sorted (entity, model, rank) keys
    double *sc = (double *)(ens_lds + (size_t)n2 * 8);          // [n2] score of the entity whose run starts here
    __shared__ double red_s[256], terms[ENS_MAX_K + 1];        // terms[k - 1] of rank k, terms[ENS_MAX_K] of an absent entity
    __shared__ int red_e[256], red_i[256];
    for (int i = threadIdx.x; i <= ENS_MAX_K; i += blockDim.x) terms[i] = i < ENS_MAX_K ? tm.rank[i] : tm.absent;
    const int64_t q = blockIdx.x;
    const int n = M * K;
    for (int i = threadIdx.x; i < n2; i += blockDim.x) {
        uint64_t kk = ENS_PAD;
        if (i < n) {
            const int m = i / K, k = i % K;
            const int32_t t = lists[((int64_t)m * Q + q) * K + k];
            if (t >= 0) kk = ((uint64_t)(uint32_t)t << 32) | ((uint64_t)m << 16) | (uint64_t)k;
        }
        key[i] = kk;
    }
    ens_bitonic(key, n2);
    // run heads: one thread sums the run in model order; the first entry of a model (smallest rank) counts
    for (int i = threadIdx.x; i < n2; i += blockDim.x) {
        double s = ENS_NONE;
        const uint64_t kk = key[i];
        const uint32_t t = (uint32_t)(kk >> 32);
        if (kk != ENS_PAD && !(i > 0 && (uint32_t)(key[i - 1] >> 32) == t)) {
            s = 0.0;
            int pos = i;
            for (int m = 0; m < M; ++m) {
                double term = terms[ENS_MAX_K];
                if (pos < n2 && key[pos] != ENS_PAD && (uint32_t)(key[pos] >> 32) == t && (int)((key[pos] >> 16) & 0xffff) == m) {
                    term = terms[(int)(key[pos] & 0xffff)];
                    while (pos < n2 && key[pos] != ENS_PAD && (uint32_t)(key[pos] >> 32) == t && (int)((key[pos] >> 16) & 0xffff) == m) ++pos;
                }
                s += term;
            }
        }
        sc[i] = s;
    }
    __syncthreads();
    for (int o = 0; o < K_out; ++o) {
        double bs = ENS_NONE; int be = 0x7fffffff, bi = -1;
        for (int i = threadIdx.x; i < n2; i += blockDim.x) {
            const double s = sc[i];
            if (s == ENS_NONE) continue;
            const int e = (int)(uint32_t)(key[i] >> 32);
            if (bi < 0 || s > bs || (s == bs && e < be)) { bs = s; be = e; bi = i; }
        }
        red_s[threadIdx.x] = bs; red_e[threadIdx.x] = be; red_i[threadIdx.x] = bi;
        __syncthreads();
        for (int w = 128; w > 0; w >>= 1) {
            if ((int)threadIdx.x < w) {
                const int a = threadIdx.x, b = threadIdx.x + w;
                const bool take = red_i[b] >= 0 && (red_i[a] < 0 || red_s[b] > red_s[a] || (red_s[b] == red_s[a] && red_e[b] < red_e[a]));
                if (take) { red_s[a] = red_s[b]; red_e[a] = red_e[b]; red_i[a] = red_i[b]; }
            }
            __syncthreads();
        }
        if (threadIdx.x == 0) {
            const bool ok = red_i[0] >= 0;
            out_idx[q * K_out + o] = ok ? red_e[0] : -1;
            out_score[q * K_out + o] = ok ? (float)red_s[0] : -INFINITY;
            if (ok) sc[red_i[0]] = ENS_NONE;
        }
        __syncthreads();
    }
}

}  // namespace

int kge_run_ensemble(const int32_t *lists, int M, int64_t Q, int K, double p, int K_out, int32_t *out_idx, float *out_score,
                     hipStream_t st) {
    if (M < 1 || M > ENS_MAX_M || K < 1 || K > ENS_MAX_K || M * K > ENS_MAX_ENTRIES) return KGE_E_UNSUPPORTED;
    EnsTerms tm;
    const double sg = p > 0.0 ? -1.0 : 1.0;
    for (int k = 0; k < ENS_MAX_K; ++k) tm.rank[k] = k < K ? sg * pow((double)(k + 1), p) : 0.0;
    tm.absent = p > 0.0 ? -pow((double)(K + 1), p) : 0.0;
    int n2 = 256;
    while (n2 < M * K) n2 <<= 1;
    const int lds = n2 * 16;
    static KgeLdsLimit lds_limit;
    if (lds_limit.set((const void *)ens_kernel, ENS_MAX_ENTRIES * 16) != KGE_OK) return KGE_E_HIP;
    hipLaunchKernelGGL(ens_kernel, dim3((unsigned)Q), dim3(256), lds, st, lists, M, Q, K, n2, tm, K_out, out_idx, out_score);
    return kge_launch_status();
}
