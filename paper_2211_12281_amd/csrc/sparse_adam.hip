// Duplicate-aware scatter-add + lazy sparse Adam:
//   1. stable LSD radix sort of (table row, position) pairs, 8 bits per pass
//   2. every run of equal rows is reduced in increasing position order (fixed order, no atomics)
//   3. one Adam step on each distinct row, fp32 master weights + moments, optional bf16 shadow
// Only rows that occur in idx are read or written (arXiv 2211.12281, Section 1: sparse access).
#include "kge_internal.h"
#include <math.h>

namespace {

constexpr int64_t SORT_MAX_BLOCKS = 32768;   // bounds the histogram that one workgroup scans

__global__ void sort_init_kernel(const int32_t *idx, int64_t M, uint32_t *keys, uint32_t *pos) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < M) { keys[i] = (uint32_t)idx[i]; pos[i] = (uint32_t)i; }
}

__global__ void sort_init_bucket_kernel(const int32_t *h, const int32_t *t, int64_t n, int64_t part_size, int D,
                                        uint32_t *keys, uint32_t *pos) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) { keys[i] = (uint32_t)((h[i] / part_size) * D + (t[i] / part_size)); pos[i] = (uint32_t)i; }
}

__global__ void sort_hist_kernel(const uint32_t *keys, int64_t M, int shift, int nblk, int rounds, uint32_t *hist) {
    __shared__ uint32_t cnt[256];
    cnt[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * rounds * 256;
    for (int j = 0; j < rounds; ++j) {
        const int64_t i = base + (int64_t)j * 256 + threadIdx.x;
        if (i < M) atomicAdd(&cnt[(keys[i] >> shift) & 255u], 1u);
    }
    __syncthreads();
    hist[(size_t)threadIdx.x * nblk + blockIdx.x] = cnt[threadIdx.x];
}

// exclusive scan of `len` counters in place, one workgroup of 1024 threads
__global__ void sort_scan_kernel(uint32_t *hist, int64_t len) {
    __shared__ uint32_t part[1024];
    const int64_t per = (len + 1023) / 1024;
    const int64_t lo = (int64_t)threadIdx.x * per, hi = lo + per < len ? lo + per : len;
    uint32_t s = 0;
    for (int64_t i = lo; i < hi; ++i) s += hist[i];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {                 // inclusive Hillis-Steele scan of the partial sums
        uint32_t v = threadIdx.x >= (unsigned)o ? part[threadIdx.x - o] : 0u;
        __syncthreads();
        part[threadIdx.x] += v;
        __syncthreads();
    }
    uint32_t run = threadIdx.x ? part[threadIdx.x - 1] : 0u;
    for (int64_t i = lo; i < hi; ++i) { uint32_t c = hist[i]; hist[i] = run; run += c; }
}

// Stable scatter of one pass.  A workgroup walks its tile in rounds of 256 keys; within a round the
// order is (wave, lane), so the rank of a key among the keys of its digit is
//   [keys of that digit in earlier workgroups] + [in earlier rounds] + [in earlier waves] + [in lower lanes].
__global__ void sort_scatter_kernel(const uint32_t *keys, const uint32_t *pos, int64_t M, int shift, int nblk,
                                    int rounds, const uint32_t *gofs, uint32_t *keys_out, uint32_t *pos_out) {
    __shared__ uint32_t wc[4][256];       // keys of each digit per wave in the current round
    __shared__ uint32_t run[256];         // keys of each digit in earlier rounds (plus the global offset)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    run[threadIdx.x] = gofs[(size_t)threadIdx.x * nblk + blockIdx.x];
    const int64_t base = (int64_t)blockIdx.x * rounds * 256;
    for (int j = 0; j < rounds; ++j) {
        for (int w = 0; w < 4; ++w) wc[w][threadIdx.x] = 0;
        __syncthreads();
        const int64_t i = base + (int64_t)j * 256 + threadIdx.x;
        const bool valid = i < M;
        const uint32_t k = valid ? keys[i] : 0u, p = valid ? pos[i] : 0u;
        const uint32_t dg = (k >> shift) & 255u;
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const bool bit = (dg >> b) & 1u;
            const uint64_t m = __ballot(valid && bit);
            peers &= bit ? m : ~m;
        }
        const uint32_t rank = (uint32_t)__popcll(peers & ((1ull << lane) - 1ull));
        if (valid && rank == 0) wc[wave][dg] = (uint32_t)__popcll(peers);
        __syncthreads();
        uint32_t before = 0;              // this thread acts for digit threadIdx.x
        {
            const uint32_t c0 = wc[0][threadIdx.x], c1 = wc[1][threadIdx.x], c2 = wc[2][threadIdx.x], c3 = wc[3][threadIdx.x];
            const uint32_t r0 = run[threadIdx.x];
            wc[0][threadIdx.x] = r0; wc[1][threadIdx.x] = r0 + c0; wc[2][threadIdx.x] = r0 + c0 + c1;
            wc[3][threadIdx.x] = r0 + c0 + c1 + c2;
            before = r0 + c0 + c1 + c2 + c3;
        }
        __syncthreads();
        if (valid) {
            const uint32_t dst = wc[wave][dg] + rank;
            keys_out[dst] = k;
            pos_out[dst] = p;
        }
        __syncthreads();
        run[threadIdx.x] = before;
    }
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf2;
    bf2 v = { (__bf16)lo, (__bf16)hi };
    return __builtin_bit_cast(uint32_t, v);
}

struct AdamConst { float lr, b1, b2, eps, omb1, omb2, inv_bc1, inv_bc2; };

// One wave per sorted position; only the first position of a run of equal rows does work.
__global__ void adam_segment_kernel(const uint32_t *sk, const uint32_t *sp, int64_t M, const float *grads, int dim,
                                    int64_t ld, float *param, uint16_t *shadow, float *mom, float *var,
                                    AdamConst c) {
    const int lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (i >= M) return;
    const uint32_t key = sk[i];
    if (i > 0 && sk[i - 1] == key) return;
    int64_t e = i + 1;
    while (e < M && sk[e] == key) ++e;
    for (int col = lane * 4; col < dim; col += 256) {
        float4 g = make_float4(0.f, 0.f, 0.f, 0.f);
        int64_t k = i;
        for (; k + 4 <= e; k += 4) {                       // four independent loads in flight, fixed add order
            const float4 g0 = *(const float4 *)(grads + (int64_t)sp[k] * dim + col);
            const float4 g1 = *(const float4 *)(grads + (int64_t)sp[k + 1] * dim + col);
            const float4 g2 = *(const float4 *)(grads + (int64_t)sp[k + 2] * dim + col);
            const float4 g3 = *(const float4 *)(grads + (int64_t)sp[k + 3] * dim + col);
            g.x += g0.x; g.y += g0.y; g.z += g0.z; g.w += g0.w;
            g.x += g1.x; g.y += g1.y; g.z += g1.z; g.w += g1.w;
            g.x += g2.x; g.y += g2.y; g.z += g2.z; g.w += g2.w;
            g.x += g3.x; g.y += g3.y; g.z += g3.z; g.w += g3.w;
        }
        for (; k < e; ++k) {
            const float4 g0 = *(const float4 *)(grads + (int64_t)sp[k] * dim + col);
            g.x += g0.x; g.y += g0.y; g.z += g0.z; g.w += g0.w;
        }
        const int64_t o = (int64_t)key * ld + col;
        float4 th = *(float4 *)(param + o), m = *(float4 *)(mom + o), v = *(float4 *)(var + o);
        const float gg[4] = { g.x, g.y, g.z, g.w };
        float tt[4] = { th.x, th.y, th.z, th.w }, mm[4] = { m.x, m.y, m.z, m.w }, vv[4] = { v.x, v.y, v.z, v.w };
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            mm[q] = c.b1 * mm[q] + c.omb1 * gg[q];
            vv[q] = c.b2 * vv[q] + c.omb2 * gg[q] * gg[q];
            tt[q] -= c.lr * (mm[q] * c.inv_bc1) / (sqrtf(vv[q] * c.inv_bc2) + c.eps);
        }
        *(float4 *)(param + o) = make_float4(tt[0], tt[1], tt[2], tt[3]);
        *(float4 *)(mom + o) = make_float4(mm[0], mm[1], mm[2], mm[3]);
        *(float4 *)(var + o) = make_float4(vv[0], vv[1], vv[2], vv[3]);
        if (shadow) *(uint2 *)(shadow + o) = make_uint2(pack_bf16x2(tt[0], tt[1]), pack_bf16x2(tt[2], tt[3]));
    }
}

struct SortWs { uint32_t *ka, *kb, *pa, *pb, *hist; int nblk, rounds; };

size_t sort_carve(int64_t M, void *ws, SortWs &s) {
    char *p = (char *)ws;
    size_t off = 0;
    auto take = [&](size_t bytes) { void *q = p ? p + off : nullptr; off += (bytes + 255) / 256 * 256; return q; };
    s.rounds = 4;                               // 1024 keys per workgroup, more for very long inputs
    while ((M + 256ll * s.rounds - 1) / (256ll * s.rounds) > SORT_MAX_BLOCKS) s.rounds *= 2;
    s.nblk = (int)((M + 256ll * s.rounds - 1) / (256ll * s.rounds));
    if (s.nblk < 1) s.nblk = 1;
    s.ka = (uint32_t *)take((size_t)M * 4); s.kb = (uint32_t *)take((size_t)M * 4);
    s.pa = (uint32_t *)take((size_t)M * 4); s.pb = (uint32_t *)take((size_t)M * 4);
    s.hist = (uint32_t *)take((size_t)256 * s.nblk * 4);
    return off + 256;
}

}  // namespace

size_t kge_sparse_adam_ws(int64_t M) {
    if (M < 0 || M >= (1ll << 31)) return 0;
    SortWs s;
    return sort_carve(M, nullptr, s);
}

size_t kge_sort_ws(int64_t M) { return kge_sparse_adam_ws(M); }

// Sorts (key, position) pairs by key, stable; returns the buffers that hold the result.  Keys are
// either the given row ids, or (when h and t are given) the partition-pair bucket of each triple.
int kge_sort_pairs(const int32_t *idx, const int32_t *h, const int32_t *t, int64_t part_size, int D, int64_t M,
                   int64_t key_range, void *ws, const uint32_t **sk, const uint32_t **sp, hipStream_t st) {
    SortWs s;
    sort_carve(M, ws, s);
    const int grid_e = (int)((M + 255) / 256);
    if (idx) hipLaunchKernelGGL(sort_init_kernel, dim3(grid_e), dim3(256), 0, st, idx, M, s.ka, s.pa);
    else     hipLaunchKernelGGL(sort_init_bucket_kernel, dim3(grid_e), dim3(256), 0, st, h, t, M, part_size, D, s.ka, s.pa);
    int bits = 1;
    while (bits < 32 && (1ll << bits) < key_range) ++bits;
    uint32_t *ki = s.ka, *ko = s.kb, *pi = s.pa, *po = s.pb;
    for (int shift = 0; shift < bits; shift += 8) {
        hipLaunchKernelGGL(sort_hist_kernel, dim3(s.nblk), dim3(256), 0, st, ki, M, shift, s.nblk, s.rounds, s.hist);
        hipLaunchKernelGGL(sort_scan_kernel, dim3(1), dim3(1024), 0, st, s.hist, (int64_t)256 * s.nblk);
        hipLaunchKernelGGL(sort_scatter_kernel, dim3(s.nblk), dim3(256), 0, st, ki, pi, M, shift, s.nblk, s.rounds, s.hist, ko, po);
        uint32_t *tmp = ki; ki = ko; ko = tmp;
        tmp = pi; pi = po; po = tmp;
    }
    *sk = ki; *sp = pi;
    return kge_launch_status();
}

int kge_run_sparse_adam(float *param, void *shadow, float *m, float *v, int64_t n_rows, int dim, int64_t ld,
                        const int32_t *idx, const float *grads, int64_t M, const kge_adam_cfg_t &cfg, void *ws,
                        size_t ws_bytes, hipStream_t st) {
    (void)ws_bytes;
    const uint32_t *sk, *sp;
    int rc;
    {
        KgeProfScope prof(KGE_PROF_SORT, st);
        rc = kge_sort_pairs(idx, nullptr, nullptr, 1, 1, M, n_rows, ws, &sk, &sp, st);
    }
    if (rc != KGE_OK) return rc;
    AdamConst c;
    c.lr = cfg.lr; c.b1 = cfg.beta1; c.b2 = cfg.beta2; c.eps = cfg.eps;
    c.omb1 = 1.f - cfg.beta1; c.omb2 = 1.f - cfg.beta2;
    c.inv_bc1 = (float)(1.0 / (1.0 - pow((double)cfg.beta1, (double)cfg.step)));
    c.inv_bc2 = (float)(1.0 / (1.0 - pow((double)cfg.beta2, (double)cfg.step)));
    const int grid = (int)((M + 3) / 4);
    KgeProfScope prof(KGE_PROF_ADAM, st);
    hipLaunchKernelGGL(adam_segment_kernel, dim3(grid), dim3(256), 0, st, sk, sp, M, grads, dim, ld, param,
                       (uint16_t *)shadow, m, v, c);
    return kge_launch_status();
}
