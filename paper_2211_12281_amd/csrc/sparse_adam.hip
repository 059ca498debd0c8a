// Duplicate-aware scatter-add + lazy sparse Adam:
//   1. stable LSD radix sort of (table row, position) pairs, 8 bits per pass
//   2. every run of equal rows is reduced in increasing position order (fixed order, no atomics)
//   3. one Adam step on each distinct row, fp32 master weights + moments, optional bf16 shadow
// Only rows that occur in idx are read or written (arXiv 2211.12281, Section 1: sparse access).
#include "kge_internal.h"
#include "row_finish.hpp"
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

// ---------------------------------------------------------------------------------------------
// Up to SMALL_MAX row ids in ONE launch (the ids of a training step: 2B + N of them).  Only the grouping of equal ids and
// the position order inside a group matter to the update, so the order is (id & 255, id >> 8, position): workgroup w owns
// the ids whose low byte is w (low five bits, 32 workgroups, for a table of at most SMALL_FEW ids).  Two workgroups share
// a compute unit (66 KB of LDS, 64 registers), so that the 256 + 32 workgroups of a step's entity and relation table run
// in one turn (with the LDS of a whole compute unit each, the 32 past the 256th waited for a second turn: 18-20 us
// instead of 14-18).  It reads ALL ids (a few tens of KB, from L2), counts those of lower workgroups (its place in the
// output) and collects its own in position order; then it orders its list by the remaining bits, stable: a list
// of up to 256 entries by counting, for every entry, the entries that come before it (one entry per thread); a longer
// one (one id repeated thousands of times) after its dominant id has been split off, or, if what remains is still longer,
// by counting passes of four bits; the list lies in LDS, or in the second pair of output buffers when it is longer than
// SMALL_CAP.  No workgroup waits for another; several tables go into one launch (workgroup ranges).
// ---------------------------------------------------------------------------------------------
constexpr int SMALL_MAX = 32768;
constexpr int SMALL_CAP = 3072;                             // longest list that is ordered in LDS
constexpr int SMALL_NT = 1024;                              // threads of a workgroup
constexpr int SMALL_ROUNDS = SMALL_MAX / (4 * SMALL_NT);    // rounds of SMALL_NT threads x 4 consecutive ids
constexpr int SMALL_DIRECT = 256;                           // longest list that is ordered by counting predecessors
constexpr int SMALL_PT = 256;                               // threads that take part in a counting pass (a rare path: its
                                                            // counters are kept small so that two workgroups share a compute unit)
constexpr int SMALL_TABLES = 4;
constexpr int SMALL_FEW = 8192;                            // a table of at most this many ids is cut into 32 parts, not 256
__host__ __device__ constexpr int small_cnt_at(int f) { return f + (f >> 4); }     // one pad word per 16: strided reads spread over banks

struct SmallSort { const int32_t *idx; int M, bits, lb; uint32_t *ka, *kb, *pa, *pb; };   // bits: of the largest id; lb: of the id that select the workgroup
// the low bits that select a table's workgroup (a function of the table alone: the order of the sorted ids, and with it
// the association order of the sums, must not depend on what else is in the launch)
static void small_parts(const int *ms, int n, int *lb) {
    for (int k = 0; k < n; ++k) lb[k] = ms[k] <= SMALL_FEW ? 5 : 8;
}
struct SmallSorts { SmallSort t[SMALL_TABLES]; };

// exclusive scan of one value per thread over the workgroup (in thread order); returns the total through `total`
__device__ __forceinline__ uint32_t small_block_scan(uint32_t v, uint32_t *s_wave, uint32_t &total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t u = __shfl_up(inc, o);
        if (lane >= o) inc += u;
    }
    __syncthreads();                                       // s_wave may still be read from an earlier scan
    if (lane == 63) s_wave[wave] = inc;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int k = 0; k < SMALL_NT / 64; ++k) { const uint32_t x = s_wave[k]; before += k < wave ? x : 0u; all += x; }
    total = all;
    return before + inc - v;
}

// One stable counting pass over a list of n (key, position) pairs by the four key bits at `shift`: thread t owns the
// contiguous piece [t c, (t + 1) c) of the list, c = ceil(n / SMALL_PT), t < SMALL_PT, and moves through it eight entries at a time
// (eight loads in flight: the list may lie in global memory).  dst_off is added to every destination index.
__device__ __forceinline__ void small_pass(const uint32_t *sk, const uint32_t *sp, uint32_t *dk, uint32_t *dp, int n, int shift,
                                           int dst_off, uint32_t *s_cnt, uint32_t *s_wave) {
    const int tid = threadIdx.x;
    const bool part = tid < SMALL_PT;                      // (the other threads only help with the scan and the barriers)
    const int c = (n + SMALL_PT - 1) / SMALL_PT, lo = !part ? n : (tid * c < n ? tid * c : n), hi = lo + c < n ? lo + c : n;
    if (part) {
#pragma unroll
        for (int d = 0; d < 16; ++d) s_cnt[small_cnt_at(d * SMALL_PT + tid)] = 0;
    }
    for (int e = lo; e < hi; e += 8) {
        uint32_t k[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) k[u] = e + u < hi ? sk[e + u] : 0u;
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (e + u < hi) s_cnt[small_cnt_at((int)((k[u] >> shift) & 15u) * SMALL_PT + tid)] += 1;      // own slots only
    }
    __syncthreads();
    // counters in (digit, thread) order: thread t scans the 16 consecutive ones at 16 t
    uint32_t v[16], sum = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) { v[j] = part ? s_cnt[small_cnt_at(tid * 16 + j)] : 0u; sum += v[j]; }
    uint32_t total;
    uint32_t run = small_block_scan(sum, s_wave, total);
    if (part) {
#pragma unroll
        for (int j = 0; j < 16; ++j) { s_cnt[small_cnt_at(tid * 16 + j)] = run; run += v[j]; }
    }
    __syncthreads();
    for (int e = lo; e < hi; e += 8) {
        uint32_t k[8], q[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) { k[u] = e + u < hi ? sk[e + u] : 0u; q[u] = e + u < hi ? sp[e + u] : 0u; }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (e + u < hi) {
                const int slot = small_cnt_at((int)((k[u] >> shift) & 15u) * SMALL_PT + tid);
                const uint32_t at = s_cnt[slot];
                s_cnt[slot] = at + 1;
                dk[dst_off + (int)at] = k[u]; dp[dst_off + (int)at] = q[u];
            }
        }
    }
    __syncthreads();
}

// The same pass when every key of the list has the same four bits at `shift` (decided together; one id repeated through a
// long list): the order stays, the list is copied.
__device__ __forceinline__ bool small_pass_trivial(const uint32_t *sk, const uint32_t *sp, uint32_t *dk, uint32_t *dp, int n, int shift) {
    const uint32_t d0 = (sk[0] >> shift) & 15u;
    int same = 1;
    for (int e = threadIdx.x; e < n; e += SMALL_NT) same &= ((sk[e] >> shift) & 15u) == d0;
    if (!__syncthreads_and(same)) return false;
    for (int e = threadIdx.x; e < n; e += SMALL_NT) { dk[e] = sk[e]; dp[e] = sp[e]; }
    __syncthreads();
    return true;
}

__device__ __forceinline__ void sort_small_body(const SmallSorts &T, const int wg) {
    __shared__ uint32_t s_cnt[16 * SMALL_PT + SMALL_PT];
    __shared__ uint32_t s_rc[SMALL_ROUNDS * (SMALL_NT / 64)];   // own ids of every (round, wave), then their offsets
    __shared__ __attribute__((aligned(16))) uint32_t s_key[2][SMALL_CAP];
    __shared__ uint32_t s_pos[2][SMALL_CAP];
    __shared__ uint32_t s_wave[SMALL_NT / 64];
    // workgroups 0 .. nb0 - 1 take the first table, the next nb1 the second, ...: a table of up to SMALL_FEW ids is cut into
    // 32 parts (by the low five bits), a longer one into 256
    int first = 0, ti = SMALL_TABLES - 1;
    bool found = false;
#pragma unroll
    for (int k = 0; k < SMALL_TABLES - 1; ++k) {           // (the tables of a launch are packed from slot 0 on)
        const int nbk = 1 << T.t[k].lb;
        if (!found) {
            if (wg < first + nbk) { ti = k; found = true; }
            else first += nbk;
        }
    }
    const SmallSort &S = T.t[ti];
    const int32_t *idx = S.idx;
    const int M = S.M;
    const int lb = S.lb;                                   // bits of the id that select the workgroup
    const int passes = S.bits > lb ? (S.bits - lb + 3) / 4 : 0;
    const uint32_t lmask = (1u << lb) - 1u;
    uint32_t *ka = S.ka, *kb = S.kb, *pa = S.pa, *pb = S.pb;
    const int w = wg - first;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rounds = (M + 4 * SMALL_NT - 1) / (4 * SMALL_NT);
    const bool vec = ((uintptr_t)idx & 15) == 0;
    // every id into registers, all loads in flight: thread t of round r holds ids 4 (SMALL_NT r + t) .. + 3 (position order
    // = round, thread, element)
    uint4 id[SMALL_ROUNDS];
#pragma unroll
    for (int r = 0; r < SMALL_ROUNDS; ++r) {
        const int i = 4 * (r * SMALL_NT + tid);
        id[r] = make_uint4(0u, 0u, 0u, 0u);
        if (r < rounds) {
            if (vec && i + 3 < M) id[r] = *(const uint4 *)(idx + i);
            else {
                if (i < M) id[r].x = (uint32_t)idx[i];
                if (i + 1 < M) id[r].y = (uint32_t)idx[i + 1];
                if (i + 2 < M) id[r].z = (uint32_t)idx[i + 2];
                if (i + 3 < M) id[r].w = (uint32_t)idx[i + 3];
            }
        }
    }
    const uint64_t below = (1ull << lane) - 1ull;
    uint32_t lower = 0;                                    // ids of lower workgroups seen by this thread
#pragma unroll
    for (int r = 0; r < SMALL_ROUNDS; ++r) {
        if (r < rounds) {
            const int i = 4 * (r * SMALL_NT + tid);
            const uint32_t e[4] = { id[r].x, id[r].y, id[r].z, id[r].w };
            uint32_t own = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool in = i + j < M;
                lower += in && (int)(e[j] & lmask) < w;
                own += (uint32_t)__builtin_popcountll(__ballot(in && (int)(e[j] & lmask) == w));
            }
            if (lane == 0) s_rc[r * (SMALL_NT / 64) + wave] = own;
        }
    }
    __syncthreads();
    // offsets of the (round, wave) groups in the list
    const int nrc = rounds * (SMALL_NT / 64);
    const uint32_t c0 = tid < nrc ? s_rc[tid] : 0;
    uint32_t n_own, n_lower;
    const uint32_t off = small_block_scan(c0, s_wave, n_own);
    if (tid < nrc) s_rc[tid] = off;
    (void)small_block_scan(lower, s_wave, n_lower);
    __syncthreads();
    const int n = (int)n_own, base = (int)n_lower;
    if (n == 0) return;                                    // (uniform: every thread holds the same totals)
    // the list starts where `passes` exchanges of buffers end in (ka, pa); in LDS the last step writes (ka, pa) itself
    const bool in_lds = n <= SMALL_CAP;
    // the list is collected in LDS, or, when it is longer than SMALL_CAP, in the second pair of output buffers
    uint32_t *lk = in_lds ? (passes == 0 ? ka + base : s_key[0]) : kb + base;
    uint32_t *lp = in_lds ? (passes == 0 ? pa + base : s_pos[0]) : pb + base;
#pragma unroll
    for (int r = 0; r < SMALL_ROUNDS; ++r) {
        if (r < rounds) {
            const int i = 4 * (r * SMALL_NT + tid);
            const uint32_t e[4] = { id[r].x, id[r].y, id[r].z, id[r].w };
            bool mine[4];
            int before = 0;                                // own ids of lower lanes in this round
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                mine[j] = i + j < M && (int)(e[j] & lmask) == w;
                before += __builtin_popcountll(__ballot(mine[j]) & below);
            }
            int at = (int)s_rc[r * (SMALL_NT / 64) + wave] + before;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (mine[j]) { lk[at] = e[j]; lp[at] = (uint32_t)(i + j); ++at; }
        }
    }
    __syncthreads();
    if (passes == 0) return;
    if (n <= SMALL_DIRECT) {
        // the place of entry e: the entries with a smaller id, and those with the same id that come before it
        if (tid < n) {
            const uint32_t key = s_key[0][tid];
            int rank = 0;
            const int n4 = n & ~3;
            for (int j = 0; j < n4; j += 4) {
                const uint4 k4 = *(const uint4 *)&s_key[0][j];              // (the same address in every lane: a broadcast)
                rank += (k4.x < key || (k4.x == key && j < tid)) + (k4.y < key || (k4.y == key && j + 1 < tid)) +
                        (k4.z < key || (k4.z == key && j + 2 < tid)) + (k4.w < key || (k4.w == key && j + 3 < tid));
            }
            for (int j = n4; j < n; ++j) { const uint32_t kj = s_key[0][j]; rank += kj < key || (kj == key && j < tid); }
            ka[base + rank] = key; pa[base + rank] = s_pos[0][tid];
        }
    } else {
        // A long list is usually ONE id repeated (Zipf's hottest rows): the entries with that id keep their order as one
        // group, and only the others are ordered - by counting predecessors among themselves - and placed before or
        // behind the group.  (Which id is taken only decides how fast this is.)
        // the most frequent id among the list's first 64 entries (ties: the earliest), found by every wave for itself
        const uint32_t mine = lk[lane];
        int votes = 0;
        for (int j = 0; j < 64; ++j) votes += mine == (uint32_t)__builtin_amdgcn_readlane((int)mine, j);
        int best = (votes << 6) | (63 - lane);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) { const int other = __shfl_xor(best, o); best = other > best ? other : best; }
        const uint32_t hot = (uint32_t)__builtin_amdgcn_readlane((int)mine, 63 - (best & 63));
        // wave v takes the contiguous piece [v cw, (v + 1) cw) of the list, 64 consecutive entries per step (coalesced: the
        // list may lie in global memory), twice: to count, then to place; ranks inside a step come from ballots
        constexpr int NW = SMALL_NT / 64;
        const int cw = ((n + NW - 1) / NW + 63) & ~63, wlo = wave * cw < n ? wave * cw : n, whi = wlo + cw < n ? wlo + cw : n;
        int cold = 0, less = 0;                            // of the wave (the same in every lane)
        for (int e0 = wlo; e0 < whi; e0 += 512) {
            uint32_t k[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) { const int e = e0 + 64 * u + lane; k[u] = e < whi ? lk[e] : hot; }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                cold += __builtin_popcountll(__ballot(k[u] != hot));
                less += __builtin_popcountll(__ballot(k[u] < hot));
            }
        }
        __syncthreads();                                   // (s_rc is free: the list has been collected)
        if (lane == 0) { s_rc[wave] = (uint32_t)cold; s_rc[NW + wave] = (uint32_t)less; }
        __syncthreads();
        int cold_at = 0, n_cold = 0, n_less = 0;           // cold entries of lower waves; totals
#pragma unroll
        for (int v = 0; v < NW; ++v) {
            const int cv = (int)s_rc[v];
            cold_at += v < wave ? cv : 0; n_cold += cv; n_less += (int)s_rc[NW + v];
        }
        if (n_cold <= SMALL_DIRECT) {                      // (uniform)
            int ci = cold_at;                              // cold entries before the step
            for (int e0 = wlo; e0 < whi; e0 += 512) {
                uint32_t k[8], q[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int e = e0 + 64 * u + lane;
                    k[u] = e < whi ? lk[e] : hot; q[u] = e < whi ? lp[e] : 0u;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int e = e0 + 64 * u + lane;
                    const bool is_cold = k[u] != hot;
                    const uint64_t mc = __ballot(is_cold);
                    const int mine_at = ci + __builtin_popcountll(mc & below);          // cold entries before this one
                    if (e < whi) {
                        if (is_cold) { s_key[1][mine_at] = k[u]; s_pos[1][mine_at] = q[u]; }
                        else { const int at = base + n_less + e - mine_at; ka[at] = hot; pa[at] = q[u]; }
                    }
                    ci += __builtin_popcountll(mc);
                }
            }
            __syncthreads();
            const int nc = n_cold, n_hot = n - nc;
            if (tid < nc) {
                const uint32_t key = s_key[1][tid];
                int rank = 0;
                const int nc4 = nc & ~3;
                for (int j = 0; j < nc4; j += 4) {
                    const uint4 k4 = *(const uint4 *)&s_key[1][j];          // (the same address in every lane: a broadcast)
                    rank += (k4.x < key || (k4.x == key && j < tid)) + (k4.y < key || (k4.y == key && j + 1 < tid)) +
                            (k4.z < key || (k4.z == key && j + 2 < tid)) + (k4.w < key || (k4.w == key && j + 3 < tid));
                }
                for (int j = nc4; j < nc; ++j) { const uint32_t kj = s_key[1][j]; rank += kj < key || (kj == key && j < tid); }
                const int to = base + rank + (key > hot ? n_hot : 0);
                ka[to] = key; pa[to] = s_pos[1][tid];
            }
            return;
        }
        if (in_lds) {
            for (int p = 0; p < passes; ++p) {
                const bool last = p == passes - 1;
                small_pass(s_key[p & 1], s_pos[p & 1], last ? ka : s_key[(p + 1) & 1], last ? pa : s_pos[(p + 1) & 1], n, lb + 4 * p,
                           last ? base : 0, s_cnt, s_wave);
            }
        } else {
            // between the two pairs of output buffers, ending in (ka, pa): an even number of passes starts there (one copy)
            uint32_t *k0 = lk, *p0 = lp, *k1 = ka + base, *p1 = pa + base;
            if (!(passes & 1)) {
                for (int e = tid; e < n; e += SMALL_NT) { k1[e] = k0[e]; p1[e] = p0[e]; }
                __syncthreads();
                uint32_t *tk = k0; k0 = k1; k1 = tk;
                tk = p0; p0 = p1; p1 = tk;
            }
            for (int p = 0; p < passes; ++p) {
                if (!small_pass_trivial(k0, p0, k1, p1, n, lb + 4 * p)) small_pass(k0, p0, k1, p1, n, lb + 4 * p, 0, s_cnt, s_wave);
                uint32_t *tk = k0; k0 = k1; k1 = tk;
                tk = p0; p0 = p1; p1 = tk;
            }
        }
    }
}

__global__ __attribute__((amdgpu_flat_work_group_size(SMALL_NT, SMALL_NT), amdgpu_waves_per_eu(8, 8))) void sort_small_kernel(const SmallSorts T) {
    sort_small_body(T, (int)blockIdx.x);
}
// The sorts of a training step's row ids need the ids alone, the finish of the rows' losses (row_finish.hpp) the forward
// pass alone: they share a launch between the two block kernels, the sorts' workgroups first (two fit a compute unit, and a
// workgroup of the finish, sixteen rows, beside one of them), so that the few microseconds of the finish pass under the sorts.
__global__ __attribute__((amdgpu_flat_work_group_size(SMALL_NT, SMALL_NT), amdgpu_waves_per_eu(8, 8)))
void sort_small_rowfinish_kernel(const SmallSorts T, const int sort_blocks, const KgeRowFinishQArgs q) {
    if ((int)blockIdx.x < sort_blocks) sort_small_body(T, (int)blockIdx.x);
    else kge_rowfinish_qscale_body((int)blockIdx.x - sort_blocks, q);
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
__device__ __forceinline__ void adam_boundary_body(int64_t blk, const uint32_t *sk, int64_t M, int dim, int64_t ld, const float *part,
                                                   float *param, uint16_t *shadow, float *mom, float *var, AdamConst c) {
    const int lane = threadIdx.x & 63;
    const int64_t k = blk * (blockDim.x >> 6) + (threadIdx.x >> 6);
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

// Several tables in one pair of launches (a training step updates the entity table and one or two small relation
// tables: alone, each of the small ones costs two launches for a few microseconds of work).  Same bodies, so the same bits
// as one call per table.  Workgroups: the piece sums of every table first, then the interior rows of every table.
constexpr int ADAM_MAX_TABLES = 4;
struct AdamTable {
    const uint32_t *sk, *sp; int64_t M; const float *grads; int dim; int64_t ld; float *param; uint16_t *shadow; float *mom, *var;
    float *part; int piece_blocks, interior_blocks;
};
struct AdamTables { AdamTable t[ADAM_MAX_TABLES]; };

__global__ void adam_interior_tables_kernel(const AdamTables T, AdamConst c) {
    int b = (int)blockIdx.x;
#pragma unroll
    for (int k = 0; k < ADAM_MAX_TABLES; ++k) {
        const AdamTable &t = T.t[k];
        if (b < t.piece_blocks) { adam_piece_body(b, t.sk, t.sp, t.M, t.grads, t.dim, t.part); return; }
        b -= t.piece_blocks;
    }
#pragma unroll
    for (int k = 0; k < ADAM_MAX_TABLES; ++k) {
        const AdamTable &t = T.t[k];
        if (b < t.interior_blocks) {
            adam_interior_body(b, t.sk, t.sp, t.M, t.grads, t.dim, t.ld, t.param, t.shadow, t.mom, t.var, c);
            return;
        }
        b -= t.interior_blocks;
    }
}

__global__ void adam_boundary_tables_kernel(const AdamTables T, AdamConst c) {
    int b = (int)blockIdx.x;
#pragma unroll
    for (int k = 0; k < ADAM_MAX_TABLES; ++k) {
        const AdamTable &t = T.t[k];
        if (b < t.piece_blocks) { adam_boundary_body(b, t.sk, t.M, t.dim, t.ld, t.part, t.param, t.shadow, t.mom, t.var, c); return; }
        b -= t.piece_blocks;
    }
}

__global__ void adam_boundary_kernel(const uint32_t *sk, int64_t M, int dim, int64_t ld, const float *part,
                                     float *param, uint16_t *shadow, float *mom, float *var, AdamConst c) {
    adam_boundary_body(blockIdx.x, sk, M, dim, ld, part, param, shadow, mom, var, c);
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

// row ids of a step: the one-launch sort (grouped, not ascending: see sort_small_kernel); everything else the radix passes
static bool sort_is_small(bool row_ids, int64_t M) { return row_ids && M <= SMALL_MAX; }

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
    if (sort_is_small(idx != nullptr, M)) {
        SmallSorts T = {};
        const int m1 = (int)M;
        int lb1;
        small_parts(&m1, 1, &lb1);
        T.t[0] = SmallSort{idx, m1, bits, lb1, s.ka, s.kb, s.pa, s.pb};
        hipLaunchKernelGGL(sort_small_kernel, dim3(1 << lb1), dim3(SMALL_NT), 0, st, T);
        *sk = s.ka; *sp = s.pa;
        return kge_launch_status();
    }
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
    if (sort_is_small(true, M)) { *sk = s.ka; *sp = s.pa; return; }
    int bits = 1;
    while (bits < 32 && (1ll << bits) < key_range) ++bits;
    const int passes = (bits + 7) / 8;
    *sk = (passes & 1) ? s.kb : s.ka; *sp = (passes & 1) ? s.pb : s.pa;
}

// Several tables: those of up to SMALL_MAX ids share one launch (256 or 32 workgroups each), longer ones take the radix passes.
// rf: the finish of the rows' losses joins the launch of the small sorts (or gets a launch of the same kernel to itself).
int kge_run_sparse_adam_plan_tables(const kge_adam_plan_t *pl, int n, hipStream_t st, const KgeRowFinishQArgs *rf) {
    KgeProfScope prof(KGE_PROF_SORT, st);
    SmallSorts T = {};
    int small = 0, nwg = 0;
    for (int k = 0; k < n; ++k) {
        if (pl[k].M == 0) continue;
        void *ws = pl[k].ws;
        if (((uintptr_t)ws & 255) != 0) ws = (char *)ws + (256 - ((uintptr_t)ws & 255));
        if (sort_is_small(true, pl[k].M)) {
            SortWs s;
            sort_carve(pl[k].M, 0, ws, s);
            int bits = 1;
            while (bits < 32 && (1ll << bits) < pl[k].n_rows) ++bits;
            T.t[small++] = SmallSort{pl[k].idx, (int)pl[k].M, bits, 0, s.ka, s.kb, s.pa, s.pb};
        } else {
            const uint32_t *sk, *sp;
            const int rc = kge_sort_pairs(pl[k].idx, nullptr, nullptr, 1, 1, pl[k].M, pl[k].n_rows, ws, &sk, &sp, st, nullptr, 0);
            if (rc != KGE_OK) return rc;
        }
    }
    if (small > 0) {
        int ms[SMALL_TABLES], lb[SMALL_TABLES];
        for (int k = 0; k < small; ++k) ms[k] = T.t[k].M;
        small_parts(ms, small, lb);
        for (int k = 0; k < small; ++k) { T.t[k].lb = lb[k]; nwg += 1 << lb[k]; }
        if (!rf) hipLaunchKernelGGL(sort_small_kernel, dim3(nwg), dim3(SMALL_NT), 0, st, T);
    }
    if (rf && rf->Bp > 0) {
        const int rows_wg = SMALL_NT / 64;
        hipLaunchKernelGGL(sort_small_rowfinish_kernel, dim3(nwg + (rf->Bp + rows_wg - 1) / rows_wg), dim3(SMALL_NT), 0, st, T, nwg, *rf);
    } else if (rf && small > 0) hipLaunchKernelGGL(sort_small_kernel, dim3(nwg), dim3(SMALL_NT), 0, st, T);
    return kge_launch_status();
}

int kge_run_sparse_adam_plan(int64_t n_rows, const int32_t *idx, int64_t M, void *ws, hipStream_t st) {
    const uint32_t *sk, *sp;
    KgeProfScope prof(KGE_PROF_SORT, st);
    return kge_sort_pairs(idx, nullptr, nullptr, 1, 1, M, n_rows, ws, &sk, &sp, st, nullptr, 0);
}

static AdamConst adam_const(const kge_adam_cfg_t &cfg) {
    AdamConst c;
    c.lr = cfg.lr; c.b1 = cfg.beta1; c.b2 = cfg.beta2; c.eps = cfg.eps;
    c.omb1 = 1.f - cfg.beta1; c.omb2 = 1.f - cfg.beta2;
    c.inv_bc1 = adam_inv_bias(cfg.beta1, (uint64_t)cfg.step);
    c.inv_bc2 = adam_inv_bias(cfg.beta2, (uint64_t)cfg.step);
    c.step_counter = cfg.step_counter; c.step = (uint64_t)cfg.step;
    return c;
}

// tables with M = 0 are skipped by the caller; n <= ADAM_MAX_TABLES
int kge_run_sparse_adam_apply_tables(const kge_adam_table_t *tb, int n, const kge_adam_cfg_t &cfg, hipStream_t st) {
    AdamTables T = {};
    int pieces = 0, interior = 0;
    for (int k = 0; k < n; ++k) {
        AdamTable &t = T.t[k];
        void *ws = tb[k].ws;
        if (((uintptr_t)ws & 255) != 0) ws = (char *)ws + (256 - ((uintptr_t)ws & 255));
        sort_result(tb[k].M, tb[k].n_rows, ws, &t.sk, &t.sp);
        SortWs s;
        sort_carve(tb[k].M, tb[k].dim, ws, s);
        const int64_t nchunk = (tb[k].M + SEG_CHUNK - 1) / SEG_CHUNK;
        t.M = tb[k].M; t.grads = tb[k].grads; t.dim = tb[k].dim; t.ld = tb[k].ld; t.param = tb[k].param_f32;
        t.shadow = (uint16_t *)tb[k].param_bf16; t.mom = tb[k].m; t.var = tb[k].v; t.part = s.part;
        t.piece_blocks = nchunk > 1 ? (int)((nchunk + 3) / 4) : 0;
        t.interior_blocks = (int)((tb[k].M + 3) / 4);
        pieces += t.piece_blocks; interior += t.interior_blocks;
    }
    const AdamConst c = adam_const(cfg);
    KgeProfScope prof(KGE_PROF_ADAM, st);
    hipLaunchKernelGGL(adam_interior_tables_kernel, dim3(pieces + interior), dim3(256), 0, st, T, c);
    if (pieces > 0) hipLaunchKernelGGL(adam_boundary_tables_kernel, dim3(pieces), dim3(256), 0, st, T, c);
    return kge_launch_status();
}

int kge_run_sparse_adam_apply(float *param, void *shadow, float *m, float *v, int64_t n_rows, int dim, int64_t ld,
                              const float *grads, int64_t M, const kge_adam_cfg_t &cfg, void *ws, hipStream_t st) {
    const uint32_t *sk, *sp;
    sort_result(M, n_rows, ws, &sk, &sp);
    const AdamConst c = adam_const(cfg);
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
