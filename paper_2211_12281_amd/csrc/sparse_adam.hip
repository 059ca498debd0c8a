// Duplicate-aware scatter-add + lazy sparse Adam:
//   1. stable LSD radix sort of (table row, position) pairs, 8 bits per pass
//   2. every run of equal rows is reduced in increasing position order (fixed order, no atomics)
//   3. one Adam step on each distinct row, fp32 master weights + moments, optional bf16 shadow
// Only rows that occur in idx are read or written (arXiv 2211.12281, Section 1: sparse access).
#include "kge_internal.h"
#include <math.h>
#include <mutex>

// Scratch memory of kge_sparse_adam_static, the variant for callers that cannot allocate: one copy per GPU, held until
// the process ends.  Host code never uses the array's name as an address; it asks the runtime for the device address
// once per device (kge_static_scratch below) and hands that pointer to the kernels like any other workspace.
constexpr size_t KGE_STATIC_SCRATCH_BYTES = (size_t)4 << 20;
static __device__ __align__(256) unsigned char scratch[KGE_STATIC_SCRATCH_BYTES];

namespace {

constexpr int64_t SORT_MAX_BLOCKS = 32768;   // bounds the histogram that one workgroup scans

// Where the keys of a pass come from: the first pass reads the caller's row ids (or computes the
// partition-pair bucket of each triple) and takes the position itself as payload; later passes read
// the (key, position) pairs the previous pass wrote.
struct KeySrc {
    const uint32_t *keys, *pos;       // later passes
    const int32_t *idx;               // first pass, row ids
    const int32_t *h, *t;             // first pass, bucket mode
    int64_t part_size; int D;
    const int32_t *r; int64_t n_rel;  // first pass, (bucket, relation) mode
};
template <int FIRST>   // 0: pairs, 1: row ids, 2: buckets, 3: (bucket, relation)
__device__ __forceinline__ uint32_t load_key(const KeySrc &k, int64_t i) {
    if constexpr (FIRST == 1) return (uint32_t)k.idx[i];
    else if constexpr (FIRST == 2) return (uint32_t)((k.h[i] / k.part_size) * k.D + (k.t[i] / k.part_size));
    else if constexpr (FIRST == 3) return (uint32_t)(((k.h[i] / k.part_size) * k.D + (k.t[i] / k.part_size)) * k.n_rel + k.r[i]);
    else return k.keys[i];
}
template <int FIRST>
__device__ __forceinline__ uint32_t load_pos(const KeySrc &k, int64_t i) {
    if constexpr (FIRST != 0) return (uint32_t)i;
    else return k.pos[i];
}

template <int FIRST>
__global__ void sort_hist_kernel(KeySrc src, int64_t M, int shift, int nblk, int rounds, uint32_t *hist) {
    __shared__ uint32_t cnt[256];
    cnt[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * rounds * 256;
    for (int j = 0; j < rounds; ++j) {
        const int64_t i = base + (int64_t)j * 256 + threadIdx.x;
        if (i < M) atomicAdd(&cnt[(load_key<FIRST>(src, i) >> shift) & 255u], 1u);
    }
    __syncthreads();
    hist[(size_t)threadIdx.x * nblk + blockIdx.x] = cnt[threadIdx.x];
}

// exclusive scan of `len` counters in place, one workgroup of 1024 threads (long inputs only)
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
//   [keys of smaller digits] + [same digit in earlier workgroups] + [in earlier rounds] + [in earlier waves]
//   + [in lower lanes].
// OWN_SCAN: the per-workgroup histograms are raw counts and every workgroup derives its own offsets from
// them (few workgroups: cheaper than a separate scan launch); otherwise `gofs` holds scanned offsets.
template <int FIRST, bool OWN_SCAN>
__global__ void sort_scatter_kernel(KeySrc src, int64_t M, int shift, int nblk, int rounds, const uint32_t *gofs,
                                    uint32_t *keys_out, uint32_t *pos_out) {
    __shared__ uint32_t wc[4][256];       // keys of each digit per wave in the current round
    __shared__ uint32_t run[256];         // destination of the next key of each digit
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if constexpr (OWN_SCAN) {
        // this thread acts for digit threadIdx.x: keys of the digit in earlier workgroups, and in total
        uint32_t before = 0, total = 0;
        for (int b2 = 0; b2 < nblk; ++b2) {
            const uint32_t c = gofs[(size_t)threadIdx.x * nblk + b2];
            before += b2 < (int)blockIdx.x ? c : 0u;
            total += c;
        }
        wc[0][threadIdx.x] = total;
        __syncthreads();
        for (int o = 1; o < 256; o <<= 1) {               // inclusive scan of the digit totals
            const uint32_t v = threadIdx.x >= (unsigned)o ? wc[0][threadIdx.x - o] : 0u;
            __syncthreads();
            wc[0][threadIdx.x] += v;
            __syncthreads();
        }
        run[threadIdx.x] = wc[0][threadIdx.x] - total + before;
        __syncthreads();
    } else {
        run[threadIdx.x] = gofs[(size_t)threadIdx.x * nblk + blockIdx.x];
    }
    const int64_t base = (int64_t)blockIdx.x * rounds * 256;
    for (int j = 0; j < rounds; ++j) {
        for (int w = 0; w < 4; ++w) wc[w][threadIdx.x] = 0;
        __syncthreads();
        const int64_t i = base + (int64_t)j * 256 + threadIdx.x;
        const bool valid = i < M;
        const uint32_t k = valid ? load_key<FIRST>(src, i) : 0u, p = valid ? load_pos<FIRST>(src, i) : 0u;
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
        uint32_t next = 0;                // this thread acts for digit threadIdx.x
        {
            const uint32_t c0 = wc[0][threadIdx.x], c1 = wc[1][threadIdx.x], c2 = wc[2][threadIdx.x], c3 = wc[3][threadIdx.x];
            const uint32_t r0 = run[threadIdx.x];
            wc[0][threadIdx.x] = r0; wc[1][threadIdx.x] = r0 + c0; wc[2][threadIdx.x] = r0 + c0 + c1;
            wc[3][threadIdx.x] = r0 + c0 + c1 + c2;
            next = r0 + c0 + c1 + c2 + c3;
        }
        __syncthreads();
        if (valid) {
            const uint32_t dst = wc[wave][dg] + rank;
            keys_out[dst] = k;
            pos_out[dst] = p;
        }
        __syncthreads();
        run[threadIdx.x] = next;
    }
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf2;
    bf2 v = { (__bf16)lo, (__bf16)hi };
    return __builtin_bit_cast(uint32_t, v);
}

struct AdamConst { float lr, b1, b2, eps, omb1, omb2, inv_bc1, inv_bc2; const uint64_t *step_counter; uint64_t step; };

// 1 / (1 - beta^step) by binary powering in fp64: products only, so the host (plain calls) and the device (steps read
// from a counter in device memory) arrive at the same bits.
__host__ __device__ inline float adam_inv_bias(float beta, uint64_t step) {
    double p = 1.0, b = (double)beta;
    for (; step; step >>= 1) {
        if (step & 1) p *= b;
        b *= b;
    }
    return (float)(1.0 / (1.0 - p));
}

// With a device counter the corrections belong to step + *counter and are formed by the wave that is about to update.
__device__ __forceinline__ void adam_resolve(AdamConst &c) {
    if (c.step_counter) {
        const uint64_t s = c.step + *c.step_counter;
        c.inv_bc1 = adam_inv_bias(c.b1, s);
        c.inv_bc2 = adam_inv_bias(c.b2, s);
    }
}

constexpr int SEG_CHUNK = 32;     // sorted positions per chunk of the two-level reduction

// Sum of the gradient rows at sorted positions [k0, k1), columns col..col+3, in position order.
__device__ __forceinline__ float4 reduce_rows(const uint32_t *sp, int64_t k0, int64_t k1, const float *grads, int dim,
                                              int col) {
    float4 g = make_float4(0.f, 0.f, 0.f, 0.f);
    int64_t k = k0;
    for (; k + 8 <= k1; k += 8) {                          // eight independent loads in flight, fixed add order
        float4 t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = *(const float4 *)(grads + (int64_t)sp[k + u] * dim + col);
#pragma unroll
        for (int u = 0; u < 8; ++u) { g.x += t[u].x; g.y += t[u].y; g.z += t[u].z; g.w += t[u].w; }
    }
    for (; k < k1; ++k) {
        const float4 t = *(const float4 *)(grads + (int64_t)sp[k] * dim + col);
        g.x += t.x; g.y += t.y; g.z += t.z; g.w += t.w;
    }
    return g;
}

__device__ __forceinline__ void adam_apply(uint32_t key, int col, float4 g, int64_t ld, float *param, uint16_t *shadow,
                                           float *mom, float *var, const AdamConst &c) {
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

// Runs of equal rows ("segments") in the sorted order are reduced in two ways:
//  - a segment that lies inside one aligned chunk of SEG_CHUNK positions is summed and updated by the
//    wave of its first position (kernel A): full parallelism over the many short segments;
//  - a segment that crosses a chunk boundary (every long one does) is cut at the boundaries; each piece
//    is summed by the wave of its chunk (kernel B1) and the wave of the chunk where the segment starts
//    adds the pieces in order and updates the row (kernel B2).
// The association order is a function of the sorted positions only: results are run-to-run identical.

// A: one wave per sorted position.
__device__ __forceinline__ void adam_interior_body(int64_t blk, const uint32_t *sk, const uint32_t *sp, int64_t M, const float *grads,
                                                   int dim, int64_t ld, float *param, uint16_t *shadow, float *mom, float *var,
                                                   AdamConst c) {
    const int lane = threadIdx.x & 63;
    const int64_t i = blk * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (i >= M) return;
    const uint32_t key = sk[i];
    if (i > 0 && sk[i - 1] == key) return;                 // not the first position of its segment
    const int64_t chunk_end = (i / SEG_CHUNK + 1) * SEG_CHUNK < M ? (i / SEG_CHUNK + 1) * SEG_CHUNK : M;
    // length of the run inside the chunk: lanes probe the following positions
    const int64_t probe = i + lane;
    const bool same = probe < chunk_end && sk[probe] == key;   // SEG_CHUNK <= 64 lanes
    const uint64_t mask = __ballot(same);
    const int run = __builtin_ctzll(~mask);                // leading ones from lane 0
    const int64_t e = i + run;
    if (e == chunk_end && chunk_end < M && sk[chunk_end] == key) return;   // crosses the boundary: kernels B
    adam_resolve(c);
    for (int col = lane * 4; col < dim; col += 256)
        adam_apply(key, col, reduce_rows(sp, i, e, grads, dim, col), ld, param, shadow, mom, var, c);
}

// B1: one wave per chunk; partial sums of its boundary-crossing pieces.
//   part[2k]   : the run at the chunk start when it continues a segment from chunk k-1
//   part[2k+1] : the run that reaches the chunk end and continues into chunk k+1, unless it is part[2k]
__device__ __forceinline__ void adam_piece_body(int64_t blk, const uint32_t *sk, const uint32_t *sp, int64_t M, const float *grads,
                                                int dim, float *part) {
    const int lane = threadIdx.x & 63;
    const int64_t k = blk * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int64_t c0 = k * SEG_CHUNK;
    if (c0 >= M) return;
    const int64_t c1 = c0 + SEG_CHUNK < M ? c0 + SEG_CHUNK : M;
    const int n = (int)(c1 - c0);
    const uint32_t kv = lane < n ? sk[c0 + lane] : 0u;
    const uint32_t first = __shfl(kv, 0), last = __shfl(kv, n - 1);
    const bool cont_in = c0 > 0 && sk[c0 - 1] == first;
    const bool cont_out = c1 < M && sk[c1] == last;
    const uint64_t valid = n == 64 ? ~0ull : ((1ull << n) - 1ull);
    if (cont_in) {
        const uint64_t m = __ballot(lane < n && kv == first);
        const int run = __builtin_ctzll(~m);
        for (int col = lane * 4; col < dim; col += 256)
            *(float4 *)(part + (2 * k) * (int64_t)dim + col) = reduce_rows(sp, c0, c0 + run, grads, dim, col);
        if (run == n) return;                               // the whole chunk is one continued run
    }
    if (cont_out) {
        const uint64_t m = __ballot(lane < n && kv == last) & valid;
        const uint64_t others = ~m & valid;
        const int start = others ? 64 - __builtin_clzll(others) : 0;   // first position of the trailing run of `last`
        if (cont_in && start == 0) return;
        for (int col = lane * 4; col < dim; col += 256)
            *(float4 *)(part + (2 * k + 1) * (int64_t)dim + col) = reduce_rows(sp, c0 + start, c1, grads, dim, col);
    }
}

// A and B1 in ONE launch (they read the same sorted gradients and write different things: A the rows of the segments
// inside a chunk, B1 the piece sums): the first piece_blocks workgroups run B1, whose few long runs then start first
__global__ void adam_interior_kernel(int piece_blocks, const uint32_t *sk, const uint32_t *sp, int64_t M, const float *grads, int dim,
                                     int64_t ld, float *param, uint16_t *shadow, float *mom, float *var, float *part, AdamConst c) {
    if ((int)blockIdx.x < piece_blocks) adam_piece_body(blockIdx.x, sk, sp, M, grads, dim, part);
    else adam_interior_body((int64_t)blockIdx.x - piece_blocks, sk, sp, M, grads, dim, ld, param, shadow, mom, var, c);
}

// B2: one wave per chunk; if a boundary-crossing segment STARTS in this chunk, add its pieces and update.
__global__ void adam_boundary_kernel(const uint32_t *sk, int64_t M, int dim, int64_t ld, const float *part,
                                     float *param, uint16_t *shadow, float *mom, float *var, AdamConst c) {
    const int lane = threadIdx.x & 63;
    const int64_t k = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int64_t c0 = k * SEG_CHUNK;
    if (c0 >= M) return;
    const int64_t c1 = c0 + SEG_CHUNK < M ? c0 + SEG_CHUNK : M;
    if (c1 >= M) return;                                    // nothing continues past the last chunk
    const uint32_t key = sk[c1 - 1];
    if (sk[c1] != key) return;                              // no segment crosses this chunk's end
    const int n = (int)(c1 - c0);
    const uint32_t kv = lane < n ? sk[c0 + lane] : ~key;
    const bool all_same = __ballot(lane < n && kv == key) == (n == 64 ? ~0ull : ((1ull << n) - 1ull));
    if (all_same && c0 > 0 && sk[c0 - 1] == key) return;    // the segment started in an earlier chunk
    // pieces: part[2k+1] here, then part[2j] of the following chunks while they continue the segment
    int64_t jend = k + 1;                                   // one past the last continuing chunk
    for (;;) {                                              // 64 chunk starts are probed per round
        const int64_t pos = (jend + lane) * SEG_CHUNK;
        const uint64_t cont = __ballot(pos < M && sk[pos] == key);
        const int run = cont == ~0ull ? 64 : __builtin_ctzll(~cont);
        jend += run;
        if (run < 64) break;
    }
    adam_resolve(c);
    for (int col = lane * 4; col < dim; col += 256) {
        float4 g = *(const float4 *)(part + (2 * k + 1) * (int64_t)dim + col);
        int64_t j = k + 1;
        for (; j + 8 <= jend; j += 8) {
            float4 t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = *(const float4 *)(part + (2 * (j + u)) * (int64_t)dim + col);
#pragma unroll
            for (int u = 0; u < 8; ++u) { g.x += t[u].x; g.y += t[u].y; g.z += t[u].z; g.w += t[u].w; }
        }
        for (; j < jend; ++j) {
            const float4 t = *(const float4 *)(part + (2 * j) * (int64_t)dim + col);
            g.x += t.x; g.y += t.y; g.z += t.z; g.w += t.w;
        }
        adam_apply(key, col, g, ld, param, shadow, mom, var, c);
    }
}

struct SortWs { uint32_t *ka, *kb, *pa, *pb, *hist; float *part; int nblk, rounds; };

size_t sort_carve(int64_t M, int dim, void *ws, SortWs &s) {
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
    s.part = (float *)take((size_t)2 * ((M + SEG_CHUNK - 1) / SEG_CHUNK) * (size_t)dim * 4);
    return off + 256;
}

}  // namespace

size_t kge_sparse_adam_ws(int64_t M, int dim) {
    if (M < 0 || M >= (1ll << 31) || dim < 0) return 0;
    SortWs s;
    return sort_carve(M, dim, nullptr, s);
}

size_t kge_sort_ws(int64_t M) { return kge_sparse_adam_ws(M, 0); }

// Sorts (key, position) pairs by key, stable; returns the buffers that hold the result.  Keys are
// either the given row ids, or (when h and t are given) the partition-pair bucket of each triple, or
// (with r as well) bucket * n_rel + relation.
int kge_sort_pairs(const int32_t *idx, const int32_t *h, const int32_t *t, int64_t part_size, int D, int64_t M,
                   int64_t key_range, void *ws, const uint32_t **sk, const uint32_t **sp, hipStream_t st,
                   const int32_t *r, int64_t n_rel) {
    SortWs s;
    sort_carve(M, 0, ws, s);
    int bits = 1;
    while (bits < 32 && (1ll << bits) < key_range) ++bits;
    uint32_t *ki = s.ka, *ko = s.kb, *pi = s.pa, *po = s.pb;       // the first pass writes buffer B
    const bool own_scan = s.nblk <= 64;
    const int first = idx ? 1 : (r ? 3 : 2);
    for (int shift = 0; shift < bits; shift += 8) {
        KeySrc src{ki, pi, idx, h, t, part_size, D, r, n_rel};
        const int mode = shift == 0 ? first : 0;
        const dim3 grid(s.nblk), blk(256);
        if (mode == 1) hipLaunchKernelGGL(sort_hist_kernel<1>, grid, blk, 0, st, src, M, shift, s.nblk, s.rounds, s.hist);
        else if (mode == 2) hipLaunchKernelGGL(sort_hist_kernel<2>, grid, blk, 0, st, src, M, shift, s.nblk, s.rounds, s.hist);
        else if (mode == 3) hipLaunchKernelGGL(sort_hist_kernel<3>, grid, blk, 0, st, src, M, shift, s.nblk, s.rounds, s.hist);
        else hipLaunchKernelGGL(sort_hist_kernel<0>, grid, blk, 0, st, src, M, shift, s.nblk, s.rounds, s.hist);
        if (!own_scan) hipLaunchKernelGGL(sort_scan_kernel, dim3(1), dim3(1024), 0, st, s.hist, (int64_t)256 * s.nblk);
#define KGE_SCATTER(F, O) hipLaunchKernelGGL((sort_scatter_kernel<F, O>), grid, blk, 0, st, src, M, shift, s.nblk, s.rounds, s.hist, ko, po)
        if (own_scan) { if (mode == 1) KGE_SCATTER(1, true); else if (mode == 2) KGE_SCATTER(2, true); else if (mode == 3) KGE_SCATTER(3, true); else KGE_SCATTER(0, true); }
        else          { if (mode == 1) KGE_SCATTER(1, false); else if (mode == 2) KGE_SCATTER(2, false); else if (mode == 3) KGE_SCATTER(3, false); else KGE_SCATTER(0, false); }
#undef KGE_SCATTER
        uint32_t *tmp = ki; ki = ko; ko = tmp;
        tmp = pi; pi = po; po = tmp;
    }
    *sk = ki; *sp = pi;
    return kge_launch_status();
}

// where kge_sort_pairs leaves its result for M pairs with keys below key_range (the passes ping-pong between two buffers)
static void sort_result(int64_t M, int64_t key_range, void *ws, const uint32_t **sk, const uint32_t **sp) {
    SortWs s;
    sort_carve(M, 0, ws, s);
    int bits = 1;
    while (bits < 32 && (1ll << bits) < key_range) ++bits;
    const int passes = (bits + 7) / 8;
    *sk = (passes & 1) ? s.kb : s.ka; *sp = (passes & 1) ? s.pb : s.pa;
}

int kge_run_sparse_adam_plan(int64_t n_rows, const int32_t *idx, int64_t M, void *ws, hipStream_t st) {
    const uint32_t *sk, *sp;
    KgeProfScope prof(KGE_PROF_SORT, st);
    return kge_sort_pairs(idx, nullptr, nullptr, 1, 1, M, n_rows, ws, &sk, &sp, st, nullptr, 0);
}

int kge_run_sparse_adam_apply(float *param, void *shadow, float *m, float *v, int64_t n_rows, int dim, int64_t ld,
                              const float *grads, int64_t M, const kge_adam_cfg_t &cfg, void *ws, hipStream_t st) {
    const uint32_t *sk, *sp;
    sort_result(M, n_rows, ws, &sk, &sp);
    AdamConst c;
    c.lr = cfg.lr; c.b1 = cfg.beta1; c.b2 = cfg.beta2; c.eps = cfg.eps;
    c.omb1 = 1.f - cfg.beta1; c.omb2 = 1.f - cfg.beta2;
    c.inv_bc1 = adam_inv_bias(cfg.beta1, (uint64_t)cfg.step);
    c.inv_bc2 = adam_inv_bias(cfg.beta2, (uint64_t)cfg.step);
    c.step_counter = cfg.step_counter; c.step = (uint64_t)cfg.step;
    SortWs s;
    sort_carve(M, dim, ws, s);                              // the piece buffer lies behind the sort buffers
    KgeProfScope prof(KGE_PROF_ADAM, st);
    const int grid = (int)((M + 3) / 4);
    const int64_t nchunk = (M + SEG_CHUNK - 1) / SEG_CHUNK;
    const int gridc = nchunk > 1 ? (int)((nchunk + 3) / 4) : 0;
    hipLaunchKernelGGL(adam_interior_kernel, dim3(gridc + grid), dim3(256), 0, st, gridc, sk, sp, M, grads, dim, ld, param,
                       (uint16_t *)shadow, m, v, s.part, c);
    if (nchunk > 1) {
        hipLaunchKernelGGL(adam_boundary_kernel, dim3(gridc), dim3(256), 0, st, sk, M, dim, ld, s.part, param,
                           (uint16_t *)shadow, m, v, c);
    }
    return kge_launch_status();
}

int kge_run_sparse_adam(float *param, void *shadow, float *m, float *v, int64_t n_rows, int dim, int64_t ld,
                        const int32_t *idx, const float *grads, int64_t M, const kge_adam_cfg_t &cfg, void *ws,
                        size_t ws_bytes, hipStream_t st) {
    (void)ws_bytes;
    const int rc = kge_run_sparse_adam_plan(n_rows, idx, M, ws, st);
    if (rc != KGE_OK) return rc;
    return kge_run_sparse_adam_apply(param, shadow, m, v, n_rows, dim, ld, grads, M, cfg, ws, st);
}

// Device address and size of the current device's copy of `scratch`.  The address is looked up on the first call on
// each device, with that device current, and kept.
int kge_static_scratch(void **ptr, size_t *bytes) {
    constexpr int MAX_DEVICES = 64;
    static std::mutex mu;
    static void *ptrs[MAX_DEVICES] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return KGE_E_HIP;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return KGE_E_HIP;
        ptrs[dev] = p;
    }
    *ptr = ptrs[dev];
    *bytes = KGE_STATIC_SCRATCH_BYTES;
    return KGE_OK;
}

size_t kge_static_scratch_bytes() { return KGE_STATIC_SCRATCH_BYTES; }
