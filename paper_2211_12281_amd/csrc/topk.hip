// Link prediction (arXiv 2211.12281, Section 3.2 "Inference"): every query is scored against a range of
// entity rows and the K best are kept.
//
//   1. prep      build the queries (Table 2), their norms and rounding residuals, squared norms of the candidates
//   2. scan      MFMA scoring of [256 queries] x [candidate tiles]; an accumulator entry that beats the
//                query's current threshold is appended to the query's candidate buffer (rare after warm-up);
//                the table is walked in growing chunks, thresholds are refreshed between chunks
//   3. compact   per query: keep the KP best buffered entries (KP > K), new threshold = the KP-th value
//   4. rescore   survivors get the ranking key in fp64 with a sequential fused-multiply-add loop
//   5. final     sort by (key, index), check with a rigorous rounding bound that no discarded candidate
//                could belong to the top-K, write the list and the rank of the held-out tail
//   6. fallback  queries that fail the check (or overflowed their buffer) are re-ranked by an exhaustive
//                fp64 scan
#include "row_ops.hpp"
#include "block_kernel.hpp"
#include <math.h>

namespace {

constexpr int TK_ST = 32;               // candidate rows per tile
constexpr int TK_HALF = 64;             // entries of one private append area

struct TopkArgs {
    const void *Qmat;                   // [Qp][dp] queries (table element type)
    const void *Wmat;                   // [Qp][dp] unit normals of the queries' relations (TransH), else nullptr
    const float *cq;                    // [Qp] w^ . q' of every query (TransH)
    const char *ent;                    // first candidate row
    int64_t ent_stride;                 // bytes between rows
    int32_t valid_bytes;                // d * sizeof(element)
    int64_t ncand;
    int64_t cand_lo;                    // entity id of candidate 0
    const float *tn;                    // [ncand rounded up to a tile] MINUS the squared norms of the candidates
    const float *thr;                   // [Qp] current threshold (local value units)
    const float *vt;                    // [Qp] value of the held-out tail (local units), +inf when absent
    const int32_t *true_t;              // [Q] entity ids, or nullptr
    uint2 *seg;                         // [Qp][nseg][2][TK_HALF] {value bits, candidate index}: private append
    int32_t *segcnt;                    // [Qp][nseg][2]           areas of each (query, split, lane half)
    int32_t nseg;
    uint32_t *rankcnt;                  // [Qp] candidates whose value beats the held-out tail's
    int32_t nq;                         // number of real queries (rows past it are padding)
    int64_t tile_lo, tile_hi;
    int32_t tiles_per_wg;
    int32_t own_tiles;
    const void *zeros;                  // 16 zero bytes (source of the padding columns)
};

// Asynchronous global -> LDS copies (gfx950): lane l of a wave-wide instruction writes its 16 (or 4)
// bytes to LDS byte address m0 + l*16 (l*4); the data never passes through registers, completion is
// tracked by vmcnt.  The compiler does not see these loads, so the waits are explicit.
__device__ __forceinline__ int tk_swz(int r) { return (((r >> 1) & 3) << 2) | (((r >> 3) & 1) << 1) | (r & 1); }
__device__ __forceinline__ void async_copy16(const void *g, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(g) : "memory");
}
__device__ __forceinline__ void async_copy4(const void *g, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_addr), "v"(g) : "memory");
}
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// "Local value": larger is better; DistMult: q.t; TransE: 2 q.t - |t|^2 (= -dist^2 + |q|^2); TransH (TH): with
// q' = h_perp + r, A = w^ . t and c = w^ . q', -|q' - t_perp|^2 + |q'|^2 + c^2 = 2 q'.t - |t|^2 + (A - c)^2: the
// wave's two row blocks hold q' and w^ of the SAME 32 queries, so both contractions share every fragment read and
// meet lane for lane in the accumulators.
//
// Candidate tiles (32 rows) stream through an LDS ring of NSTAGE stages filled by asynchronous copies,
// so several tiles are in flight per compute unit.  A row of RB bytes is stored unpadded with its
// 16-byte chunks XOR-swizzled by a bit permutation of (row mod 16) (tk_swz): the MFMA A-fragment reads of 16
// consecutive rows at one chunk index then fall into 16 different bank groups (an XOR with row mod 8 reaches half the
// LDS's rate: half of the LDS's active cycles were bank conflicts).  The MFMAs of tile t+1 are issued before the epilogue of tile t, so the
// matrix pipe works while the vector ALU filters.
template <bool BF16, int RB, int KIND, int OB, bool TH = false>
__global__ __attribute__((amdgpu_flat_work_group_size(256, 256), amdgpu_waves_per_eu(2, 2)))
void topk_scan_kernel(const TopkArgs a) {
    static_assert(!TH || (OB == 2 && KIND == KGE_KIND_DIST), "TransH: one block of queries, one of normals");
    constexpr int NQ = TH ? 1 : OB;                     // blocks of 32 queries per wave
    constexpr int KS = RB / 32;
    constexpr int TILE_BYTES = TK_ST * RB;
    constexpr int NINST = TILE_BYTES / 1024;            // wave-wide 1 KB copies per tile
    constexpr int IPW = NINST / 4;                      // ... per wave
    constexpr int LPW = IPW + 1;                        // plus the norms
    constexpr int NSTAGE = RB == 512 ? 4 : 3;
    constexpr int SIDE_SLOTS = NSTAGE + 1;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char *side_base = lds + NSTAGE * TILE_BYTES;        // [SIDE_SLOTS][4 waves][64 floats]
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 31, g = lane >> 5;
    // Workgroups are handed to the 8 XCDs round-robin.  All query tiles that walk the same candidate
    // range are given ids with the same residue mod 8, so they share one XCD's L2 and the range is
    // fetched from HBM once.
    const int xcd = blockIdx.x & 7, kk = blockIdx.x >> 3;
    const int own_tile = kk % a.own_tiles, split = xcd + 8 * (kk / a.own_tiles);
    const int own_base = own_tile * (128 * NQ);
    const int64_t t0 = a.tile_lo + (int64_t)split * a.tiles_per_wg;
    const int64_t t1 = t0 + a.tiles_per_wg < a.tile_hi ? t0 + a.tiles_per_wg : a.tile_hi;
    // Every (query, split, lane half) owns a private append area, so appending needs no atomics: the
    // count lives in a register and is stored once at the end.  Two lanes (g = 0, 1) serve one query.
    if (t0 >= t1) {
        if (split < a.nseg)
            for (int ob = 0; ob < NQ; ++ob)
                a.segcnt[((size_t)(own_base + (wave * NQ + ob) * 32 + lr) * a.nseg + split) * 2 + g] = 0;
        return;
    }

    uint4 own[OB][KS];
    float thr[NQ], vt[NQ];
    int qid[NQ], myc[NQ];
    uint32_t above[NQ];
#pragma unroll
    for (int ob = 0; ob < NQ; ++ob) {
        qid[ob] = own_base + (wave * NQ + ob) * 32 + lr;
        myc[ob] = 0;
        const char *p = (const char *)a.Qmat + (size_t)qid[ob] * RB + g * 16;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) own[ob][ks] = *(const uint4 *)(p + ks * 32);
        thr[ob] = a.thr[qid[ob]];
        vt[ob] = a.vt[qid[ob]];
        above[ob] = 0;
    }
    float cq = 0.f;
    if constexpr (TH) {
        const char *p = (const char *)a.Wmat + (size_t)qid[0] * RB + g * 16;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) own[1][ks] = *(const uint4 *)(p + ks * 32);
        cq = a.cq[qid[0]];
    }

    // ---- loader geometry of this lane: instruction jj covers LDS bytes [(wave*IPW+jj) KB, +1 KB) ----
    // A copy takes a wave-uniform base (the tile's first row, scalar registers) and ONE 32-bit offset per lane that does not
    // change from tile to tile (row in the tile x stride + source chunk), and its LDS address is scalar arithmetic on the
    // wave's number: no vector instruction per copy in the loop.  Rows shorter than RB (padding columns, which read the 16
    // zero bytes) and the table's last, ragged tile take per-lane 64-bit addresses, computed where they are needed.
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    auto ld_row_of = [&](int jj) { return ((wave_u * IPW + jj) * 1024 + lane * 16) / RB; };
    auto ld_col_of = [&](int jj) {
        const int byte = (wave_u * IPW + jj) * 1024 + lane * 16, r = byte / RB, pos = (byte % RB) / 16;
        return (pos ^ tk_swz(r)) * 16;                  // source chunk that belongs at this LDS position
    };
    uint32_t ld_off[IPW];
#pragma unroll
    for (int jj = 0; jj < IPW; ++jj) ld_off[jj] = (uint32_t)(ld_row_of(jj) * a.ent_stride + ld_col_of(jj));
    const bool unpadded = a.valid_bytes == RB && a.ent_stride < (1ll << 26);     // (uniform; 32 rows x stride fits the offset)
    auto issue = [&](int64_t tile, int slot) {
        tile = tile < t1 ? tile : t1 - 1;               // past the end: a harmless repeat keeps vmcnt uniform
        const int stage = slot % NSTAGE;
        const uint32_t lbase = lds0 + stage * TILE_BYTES + wave_u * (IPW * 1024);
        if (unpadded && tile * TK_ST + TK_ST <= a.ncand) {
            const char *tb = a.ent + tile * TK_ST * a.ent_stride;
#pragma unroll
            for (int jj = 0; jj < IPW; ++jj)
                asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lbase + jj * 1024), "v"(ld_off[jj]), "s"(tb) : "memory");
        } else {
#pragma unroll
            for (int jj = 0; jj < IPW; ++jj) {
                int64_t cand = tile * TK_ST + ld_row_of(jj);
                cand = cand < a.ncand ? cand : a.ncand - 1; // rows past the end are masked in the epilogue
                const int col = ld_col_of(jj);
                const char *gp = col < a.valid_bytes ? a.ent + cand * a.ent_stride + col : (const char *)a.zeros;
                async_copy16(gp, lbase + jj * 1024);
            }
        }
        async_copy4(a.tn + tile * TK_ST + lr, lds0 + NSTAGE * TILE_BYTES + ((slot % SIDE_SLOTS) * 4 + wave_u) * 256);
    };
    // ---- A-fragment addresses: chunk (2 ks + g) of row lr sits at position chunk ^ tk_swz(lr) ----------
    int frag_off[8];
#pragma unroll
    for (int b = 0; b < 8; ++b) frag_off[b] = lr * RB + 16 * ((2 * b + g) ^ tk_swz(lr));
    auto mma_tile = [&](int slot, kge_f32x16 (&acc)[OB]) {
        const char *base = lds + (slot % NSTAGE) * TILE_BYTES;
        // Rows of 512 bytes: the fragment of step ks + AH is requested before the MFMAs of step ks are issued, and the
        // scheduler is held to that order (left to itself the compiler reads each fragment right before its two MFMAs and
        // waits for it).  The kernels of 1,024-byte rows have no registers for fragments in flight: held to this order they
        // spill operands inside the loop, so they keep the compiler's.
        constexpr int AH = RB == 512 ? (TH ? 2 : 3) : 0;
        uint4 av[AH > 0 ? AH + 1 : KS];
#pragma unroll
        for (int ks = 0; ks < (AH > 0 ? AH : KS); ++ks) av[ks] = *(const uint4 *)(base + frag_off[ks & 7] + 256 * (ks >> 3));
        if constexpr (KIND == KGE_KIND_DIST) {
            // TransE: the accumulators start at -|t|^2 of their candidate row and the queries are stored
            // doubled, so the contraction itself yields 2 q.t - |t|^2
            const char *tside = side_base + ((slot % SIDE_SLOTS) * 4 + wave_u) * 256;
            // (rows 8 j + 4 g .. + 3 of the tile are registers 4 j .. 4 j + 3: one 16-byte read per j)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // (the side array holds -|t|^2: the accumulators are loaded, not computed)
                const kge_f32x4 tn4 = *(const kge_f32x4 *)(tside + (8 * j + 4 * g) * 4);
#pragma unroll
                for (int ob = 0; ob < NQ; ++ob)
                    for (int u = 0; u < 4; ++u) acc[ob][4 * j + u] = tn4[u];
            }
            if constexpr (TH) for (int i = 0; i < 16; ++i) acc[1][i] = 0.f;
        } else {
#pragma unroll
            for (int ob = 0; ob < OB; ++ob) for (int i = 0; i < 16; ++i) acc[ob][i] = 0.f;
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if constexpr (AH == 0) {
#pragma unroll
                for (int ob = 0; ob < OB; ++ob) acc[ob] = kge_mma16<BF16>(acc[ob], av[ks], own[ob][ks]);
            } else {
                if (ks + AH < KS) av[(ks + AH) % (AH + 1)] = *(const uint4 *)(base + frag_off[(ks + AH) & 7] + 256 * ((ks + AH) >> 3));
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int ob = 0; ob < OB; ++ob) acc[ob] = kge_mma16<BF16>(acc[ob], av[ks % (AH + 1)], own[ob][ks]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

#pragma unroll
    for (int s2 = 0; s2 < NSTAGE - 1; ++s2) issue(t0 + s2, s2);
    wait_vmcnt<(NSTAGE - 2) * LPW>();
    __syncthreads();
    issue(t0 + NSTAGE - 1, NSTAGE - 1);
    kge_f32x16 acc[OB];
    mma_tile(0, acc);

    for (int64_t tile = t0; tile < t1; ++tile) {
        const int slot = (int)(tile - t0);
        // ---- tile + 1: wait for its data, refill the stage that tile `tile` just vacated, start its MFMAs
        kge_f32x16 accn[OB];
        wait_vmcnt<(NSTAGE - 2) * LPW>();
        __syncthreads();
        issue(tile + NSTAGE, slot + NSTAGE);
        mma_tile(slot + 1, accn);                       // (the last iteration recomputes a stale stage: unused)
        // ---- epilogue of tile `tile`: cheap wave-level test first, the append path only on a hit ----
        const bool tile_full = tile * TK_ST + TK_ST <= a.ncand;
        float vv[NQ][16];                               // the values are the accumulators themselves
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if constexpr (TH) { const float x = acc[1][i] - cq; vv[0][i] = fmaf(x, x, acc[0][i]); }
            else {
#pragma unroll
                for (int ob = 0; ob < OB; ++ob) vv[ob][i] = acc[ob][i];
            }
        }
        if (!tile_full) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const bool out = tile * TK_ST + 8 * (i >> 2) + 4 * g + (i & 3) >= a.ncand;
#pragma unroll
                for (int ob = 0; ob < NQ; ++ob) vv[ob][i] = out ? -INFINITY : vv[ob][i];
            }
        }
#pragma unroll
        for (int ob = 0; ob < NQ; ++ob) {
            if (a.true_t) {
                // v > vt exactly when vt - v is negative: the sign bits are shifted into one word (one subtraction and
                // one funnel shift per entry, no compare results through scalar registers) and counted at the end
                uint32_t signs = 0;
#pragma unroll
                for (int i = 0; i < 16; ++i) signs = __builtin_amdgcn_alignbit(signs, __float_as_uint(vt[ob] - vv[ob][i]), 31);
                above[ob] += (uint32_t)__builtin_popcount(signs);
            }
            float mx = vv[ob][0];
#pragma unroll
            for (int i = 1; i < 16; ++i) mx = fmaxf(mx, vv[ob][i]);
            if (__any(mx > thr[ob])) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    if (vv[ob][i] > thr[ob]) {
                        const int64_t cand = tile * TK_ST + 8 * (i >> 2) + 4 * g + (i & 3);
                        // (the area's address is formed here, on the rarely taken path, instead of living in registers)
                        if (myc[ob] < TK_HALF)
                            a.seg[(((size_t)qid[ob] * a.nseg + split) * 2 + g) * TK_HALF + myc[ob]] = make_uint2(__float_as_uint(vv[ob][i]), (uint32_t)cand);
                        ++myc[ob];                      // counts past TK_HALF mark the overflow for the compaction
                    }
                }
            }
        }
#pragma unroll
        for (int ob = 0; ob < OB; ++ob) acc[ob] = accn[ob];
    }
    wait_vmcnt<0>();                                    // no copy may still be in flight when the LDS is released
#pragma unroll
    for (int ob = 0; ob < NQ; ++ob) a.segcnt[((size_t)qid[ob] * a.nseg + split) * 2 + g] = myc[ob];
    if (a.true_t) {
#pragma unroll
        for (int ob = 0; ob < NQ; ++ob) if (above[ob] && qid[ob] < a.nq) atomicAdd(a.rankcnt + qid[ob], above[ob]);
    }
}

// ---------------------------------------------------------------------------------------------
// bitonic sorts in LDS (256 threads)
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t pack_value(uint32_t vbits, uint32_t idx) {
    // unsigned order of the float, then smaller index first: sort DESCENDING on the packed word
    const uint32_t ord = vbits ^ ((vbits >> 31) ? 0xFFFFFFFFu : 0x80000000u);
    return ((uint64_t)ord << 32) | (uint64_t)(0xFFFFFFFFu - idx);
}
__device__ __forceinline__ uint2 unpack_value(uint64_t w) {
    const uint32_t ord = (uint32_t)(w >> 32);
    const uint32_t vbits = ord ^ ((ord >> 31) ? 0x80000000u : 0xFFFFFFFFu);
    return make_uint2(vbits, 0xFFFFFFFFu - (uint32_t)w);
}

__device__ void bitonic_desc_u64(uint64_t *s, int P) {
    for (int k = 2; k <= P; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = threadIdx.x; t < P / 2; t += blockDim.x) {
                const int i = 2 * t - (t & (j - 1)), p = i + j;          // pair (i, i + j)
                const bool desc = (i & k) == 0;
                const uint64_t x = s[i], y = s[p];
                if ((x < y) == desc) { s[i] = y; s[p] = x; }
            }
            __syncthreads();
        }
}

struct KeyIdx { double key; int idx; };
__device__ __forceinline__ bool worse(double ka, int ia, double kb, int ib) { return ka > kb || (ka == kb && ia > ib); }

__device__ void bitonic_asc_pair(double *key, int *idx, int P) {
    for (int k = 2; k <= P; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = threadIdx.x; t < P / 2; t += blockDim.x) {
                const int i = 2 * t - (t & (j - 1)), p = i + j;
                const bool asc = (i & k) == 0;
                const double kx = key[i], ky = key[p];
                const int ix = idx[i], iy = idx[p];
                if (worse(kx, ix, ky, iy) == asc) { key[i] = ky; key[p] = kx; idx[i] = iy; idx[p] = ix; }
            }
            __syncthreads();
        }
}

// per query: merge the kept list with the fresh append areas, keep the KP best, refresh the threshold.
// Two launches per chunk.  After the first chunk a query's list is a few KP long, and a workgroup whose LDS holds
// TK_SORTCAP_SMALL entries leaves room for eight on a compute unit instead of two (the reads of a query's scattered
// entries and the sort's chain of barriers are all latency: what a compute unit needs is more workgroups): the first launch (cap = TK_SORTCAP_SMALL, redo written) takes the queries whose lists
// fit and marks the others, the second (cap = TK_SORTCAP, redo read) takes the marked ones.
constexpr int TK_SORTCAP = 8192;        // entries one workgroup can sort in LDS
constexpr int TK_SORTCAP_SMALL = 2048;
__global__ void topk_compact_kernel(uint2 *keep, int32_t *keepcnt, const uint2 *seg, const int32_t *segcnt, int nseg,
                                    int nsplit, int KP, float *thr, int32_t *flag, int Q, int cap, int32_t *redo, int second) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    uint64_t *s = (uint64_t *)lds;
    __shared__ int total, over;
    const int q = blockIdx.x;
    if (q >= Q) return;
    if (second && !redo[q]) return;
    const int kept = keepcnt[q];
    __shared__ int abase[512 + 1];                          // start of every area's entries in the sort buffer
    const int nareas = nsplit * 2;                          // <= 2 * nseg <= 512
    if (threadIdx.x == 0) over = 0;
    __syncthreads();
    // counts (clamped to the area size), then their exclusive prefix sums behind the kept list: thread t takes the areas
    // 2 t and 2 t + 1 (256 threads, at most 512 areas), a shuffle scan inside every wave, the waves' sums through the LDS
    {
        __shared__ int wsum[4];
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, a0 = 2 * threadIdx.x;
        int c[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            c[j] = a0 + j < nareas ? segcnt[(size_t)q * nseg * 2 + a0 + j] : 0;
            if (c[j] > TK_HALF) { over = 1; c[j] = TK_HALF; }
        }
        int incl = c[0] + c[1];
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) { const int v = __shfl_up(incl, o); if (lane >= o) incl += v; }
        if (lane == 63) wsum[wave] = incl;
        __syncthreads();
        int start = kept + incl - (c[0] + c[1]);
        for (int w = 0; w < wave; ++w) start += wsum[w];
        if (a0 <= nareas) abase[a0] = start;
        if (a0 + 1 <= nareas) abase[a0 + 1] = start + c[0];
        if (a0 + 2 == nareas) abase[a0 + 2] = start + c[0] + c[1];
        __syncthreads();
        if (threadIdx.x == 0) total = abase[nareas];
    }
    __syncthreads();
    if (!second) {                                          // (the same for every thread)
        const bool fits = total <= cap;
        if (threadIdx.x == 0) redo[q] = fits ? 0 : 1;
        if (!fits) return;
    }
    for (int i = threadIdx.x; i < kept; i += blockDim.x) { const uint2 e = keep[(size_t)q * KP + i]; s[i] = pack_value(e.x, e.y); }
    // every thread copies whole areas (an area holds one or two entries as a rule, 64 at most): the loads of different
    // threads are independent, so the memory latency is paid once or twice per thread, not once per area of the query
    // (the order does not matter: the sort below is total)
    for (int a2 = threadIdx.x; a2 < nareas; a2 += blockDim.x) {
        const int base = abase[a2], c = abase[a2 + 1] - base;
        if (c > 0) {
            if (base + c <= cap) {
                const uint2 *src = seg + ((size_t)q * nseg * 2 + a2) * TK_HALF;
                for (int li = 0; li < c; ++li) { const uint2 e = src[li]; s[base + li] = pack_value(e.x, e.y); }
            } else over = 1;
        }
    }
    __syncthreads();
    if (over) { if (threadIdx.x == 0) flag[q] = 1; }         // entries were dropped: exhaustive re-rank later
    int n = total < cap ? total : cap;
    if (over && total > cap) n = kept;                       // partially filled: keep the old list
    int P = 2;
    while (P < n) P <<= 1;
    for (int i = n + threadIdx.x; i < P; i += blockDim.x) s[i] = 0;   // padding sorts last
    __syncthreads();
    bitonic_desc_u64(s, P);
    const int keepn = n < KP ? n : KP;
    for (int i = threadIdx.x; i < keepn; i += blockDim.x) keep[(size_t)q * KP + i] = unpack_value(s[i]);
    if (threadIdx.x == 0) {
        keepcnt[q] = keepn;
        if (n >= KP) thr[q] = __uint_as_float(unpack_value(s[KP - 1]).x);
    }
}

// ---------------------------------------------------------------------------------------------
// fp64 ranking key (smaller is better), defined on the exact query q (fp64 from the table values) and the tail row:
//   DistMult  q = h r,            key = -acc,  acc = fma(q_j, t_j, acc)
//   TransE    q = h + r,          key =  acc,  x = q_j - t_j, acc = fma(x, x, acc)
//   ComplEx   q = h * r (complex),  key = -acc,  acc = acc + (q_re t_re + q_im t_im) per complex coordinate
//   RotatE    q = h * e^{ir},       key =  acc,  acc = acc + (x_re^2 + x_im^2), x = q - t
//   TransH    u = w / max(|w|, 1e-12), q' = (h - (u.h) u) + r (both fp64, made once per query by the preparation
//             kernel), A = sum fma(u_j, t_j, .), key = acc, x = fma(A, u_j, q'_j - t_j), acc = fma(x, x, acc)
// every operation rounded on its own (no contraction), in this order: the same sequence of IEEE operations as
// the direct loops of Table 2 written in C give.  RotatE goes through cos / sin of the phase in fp64, whose last
// bit is the math library's.
// ---------------------------------------------------------------------------------------------
constexpr int TK_MAXD = 512;

__device__ __forceinline__ bool topk_mult(int scorer) { return scorer == KGE_DISTMULT || scorer == KGE_COMPLEX; }
__device__ __forceinline__ bool topk_cplx(int scorer) { return scorer == KGE_COMPLEX || scorer == KGE_ROTATE; }

// component j of the exact query (complex scorers: j < d/2 real parts, then imaginary parts)
template <bool BF16>
__device__ double query_f64(const KgeModelDev &m, int64_t hoff, int64_t roff, int j) {
    if (m.scorer == KGE_DISTMULT) return __dmul_rn((double)El<BF16>::ld(m.ent, hoff + j), (double)El<BF16>::ld(m.rel, roff + j));
    if (m.scorer == KGE_TRANSE) return __dadd_rn((double)El<BF16>::ld(m.ent, hoff + j), (double)El<BF16>::ld(m.rel, roff + j));
    const int c = m.dim >> 1, jr = j < c ? j : j - c;
    const double hre = (double)El<BF16>::ld(m.ent, hoff + jr), him = (double)El<BF16>::ld(m.ent, hoff + jr + c);
    double rre, rim;
    if (m.scorer == KGE_COMPLEX) { rre = (double)El<BF16>::ld(m.rel, roff + jr); rim = (double)El<BF16>::ld(m.rel, roff + jr + c); }
    else { const double ph = (double)El<BF16>::ld(m.rel, roff + jr); rre = cos(ph); rim = sin(ph); }
    return j < c ? __dsub_rn(__dmul_rn(hre, rre), __dmul_rn(him, rim)) : __dadd_rn(__dmul_rn(hre, rim), __dmul_rn(him, rre));
}

// one step of the key's accumulation: real scorers one column, complex scorers one complex coordinate
__device__ __forceinline__ double key_step(int scorer, double acc, double q0, double t0, double q1, double t1) {
    switch (scorer) {
    case KGE_DISTMULT: return fma(q0, t0, acc);
    case KGE_TRANSE: { const double x = __dsub_rn(q0, t0); return fma(x, x, acc); }
    case KGE_COMPLEX: return __dadd_rn(acc, __dadd_rn(__dmul_rn(q0, t0), __dmul_rn(q1, t1)));
    default: { const double xr = __dsub_rn(q0, t0), xi = __dsub_rn(q1, t1);
               return __dadd_rn(acc, __dadd_rn(__dmul_rn(xr, xr), __dmul_rn(xi, xi))); }
    }
}

// key of one tail row against the exact query qv[0 .. d)
template <bool BF16>
__device__ double canonical_key(int scorer, int d, const double *qv, const void *ent, int64_t toff) {
    double acc = 0.0;
    if (topk_cplx(scorer)) {
        const int c = d >> 1;
        for (int j = 0; j < c; ++j)
            acc = key_step(scorer, acc, qv[j], (double)El<BF16>::ld(ent, toff + j), qv[j + c], (double)El<BF16>::ld(ent, toff + j + c));
    } else {
        for (int j = 0; j < d; ++j) acc = key_step(scorer, acc, qv[j], (double)El<BF16>::ld(ent, toff + j), 0.0, 0.0);
    }
    return topk_mult(scorer) ? -acc : acc;
}

// TransH key of one tail row against q' = qv[0 .. d) and the unit normal wv[0 .. d)
template <bool BF16>
__device__ double canonical_key_th(int d, const double *qv, const double *wv, const void *ent, int64_t toff) {
    double A = 0.0, acc = 0.0;
    for (int j = 0; j < d; ++j) A = fma(wv[j], (double)El<BF16>::ld(ent, toff + j), A);
    for (int j = 0; j < d; ++j) {
        const double x = fma(A, wv[j], __dsub_rn(qv[j], (double)El<BF16>::ld(ent, toff + j)));
        acc = fma(x, x, acc);
    }
    return acc;
}

// One wave re-scores 64 survivors of one query, lane = survivor, so that the 64 sequential fp64 chains run in
// lockstep.  The candidate rows arrive through the LDS in chunks of 64 columns (complex scorers: 32 real parts
// followed by the 32 imaginary parts of the same coordinates): coalesced row reads on the way in, conflict-free
// column reads (row stride odd in dwords) on the way out; the exact query components of a chunk are computed once
// per wave.  The key is the one of canonical_key, step by step.
template <bool BF16>
__global__ __launch_bounds__(256) void topk_rescore_kernel(KgeModelDev m, const int32_t *h, const int32_t *r, int Q,
                                                           int64_t cand_lo, const int32_t *cnt, const uint2 *buf, int KP,
                                                           double *keyd, const double *qx) {
    constexpr int DW = BF16 ? 32 : 64;                  // dwords per row chunk of 64 columns
    constexpr int E = BF16 ? 2 : 1;                     // columns per dword
    __shared__ uint32_t rows[4][64 * (DW + 1)];
    __shared__ double qd[4][64], wd[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int groups = KP / 64;
    const int64_t task = (int64_t)blockIdx.x * 4 + wave;
    const int q = (int)(task / groups), s0 = (int)(task % groups) * 64;
    if (q >= Q) return;
    const int n = cnt[q];
    if (s0 >= n) return;
    const bool valid = s0 + lane < n;
    const int64_t cand = cand_lo + buf[(size_t)q * KP + (valid ? s0 + lane : s0)].y;
    const int d = m.dim, half = d >> 1;
    const bool cplx = topk_cplx(m.scorer), th = m.scorer == KGE_TRANSH;
    const double *qxq = th ? qx + (size_t)q * 2 * d : nullptr;     // TransH: q' then the unit normal, fp64
    const int span = cplx ? 32 : 64, total = cplx ? half : d;      // key steps per chunk, in all
    const int64_t hoff = (int64_t)h[q] * m.ent_ld, roff = (int64_t)r[q] * m.rel_ld;
    uint32_t *mine = rows[wave];
    auto elem = [&](const uint32_t *row, int e) -> double {        // staged element e of a row
        if constexpr (BF16) return (double)__uint_as_float((e & 1) ? (row[e >> 1] & 0xffff0000u) : (row[e >> 1] << 16));
        else return (double)__uint_as_float(row[e]);
    };
    double acc = 0.0, A = 0.0;
    // (TransH walks the row twice: first A = u . t, then the squared distance)
    for (int pass = th ? 0 : 1; pass < 2; ++pass)
    for (int c0 = 0; c0 < total; c0 += span) {
        const int steps = total - c0 < span ? total - c0 : span;
        // staged element e <-> table column: real scorers c0 + e; complex: c0 + e (e < 32), d/2 + c0 + e - 32 (else)
        auto column = [&](int e) { return cplx ? (e < 32 ? c0 + e : half + c0 + e - 32) : c0 + e; };
        auto live = [&](int e) { return (cplx ? (e & 31) : e) < steps; };
        if (live(lane)) {
            if (th) { qd[wave][lane] = qxq[c0 + lane]; wd[wave][lane] = qxq[d + c0 + lane]; }
            else qd[wave][lane] = query_f64<BF16>(m, hoff, roff, column(lane));
        }
        constexpr int RPI = 64 / DW;                    // rows per wave-wide load
        const int sub = lane / DW, dw = lane % DW;
        for (int rr = 0; rr < 64; rr += RPI) {
            const int64_t c = __shfl(cand, rr + sub);
            uint32_t v = 0u;
            if (live(dw * E))
                v = *(const uint32_t *)((const char *)m.ent + (c * m.ent_ld + column(dw * E)) * (BF16 ? 2 : 4));
            mine[(rr + sub) * (DW + 1) + dw] = v;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const uint32_t *row = mine + lane * (DW + 1);
        if (th) {
            if (pass == 0) for (int j = 0; j < steps; ++j) A = fma(wd[wave][j], elem(row, j), A);
            else for (int j = 0; j < steps; ++j) {
                const double x = fma(A, wd[wave][j], __dsub_rn(qd[wave][j], elem(row, j)));
                acc = fma(x, x, acc);
            }
        } else if (cplx) {
            for (int j = 0; j < steps; ++j) acc = key_step(m.scorer, acc, qd[wave][j], elem(row, j), qd[wave][32 + j], elem(row, 32 + j));
        } else {
            for (int j = 0; j < steps; ++j) acc = key_step(m.scorer, acc, qd[wave][j], elem(row, j), 0.0, 0.0);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    if (valid) keyd[(size_t)q * KP + s0 + lane] = topk_mult(m.scorer) ? -acc : acc;
}

struct QInfo { double qn; float eps_a, eps_b; float eps_w, c; };   // |q~|^2 (fp64), rounding-bound coefficients; TransH: |dw|, c

// final ordering, safety check, outputs
template <bool BF16>
__global__ void topk_final_kernel(KgeModelDev m, const int32_t *h, const int32_t *r, int Q, int64_t cand_lo,
                                  int64_t ncand, const int32_t *cnt, const uint2 *buf, int KP, int KPP,
                                  const double *keyd, const float *thr, const QInfo *qinfo, const float *tmax2,
                                  int K, int32_t *out_idx, float *out_score, const int32_t *true_t,
                                  const uint32_t *rankcnt, int64_t *out_rank, int32_t *flag) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    double *key = (double *)lds;
    int *idx = (int *)(lds + (size_t)KPP * 8);
    const int q = blockIdx.x;
    if (q >= Q) return;
    const int n = cnt[q];
    for (int i = threadIdx.x; i < KPP; i += blockDim.x) {
        key[i] = i < n ? keyd[(size_t)q * KP + i] : INFINITY;
        idx[i] = i < n ? (int)buf[(size_t)q * KP + i].y : 0x7FFFFFFF;
    }
    __syncthreads();
    bitonic_asc_pair(key, idx, KPP);
    const bool dm = topk_mult(m.scorer);
    for (int i = threadIdx.x; i < K; i += blockDim.x) {
        const bool ok = i < n;
        out_idx[(size_t)q * K + i] = ok ? (int32_t)(cand_lo + idx[i]) : -1;
        out_score[(size_t)q * K + i] = ok ? (dm ? (float)(-key[i]) : (float)(-sqrt(key[i]))) : -INFINITY;
    }
    if (threadIdx.x == 0) {
        // Everything that was discarded has a matrix-core value <= theta (the KP-th best value).  Its
        // exact value is at most theta + eps; the list is safe if that stays strictly below the exact
        // value of the K-th entry.  eps bounds the rounding of the query to the table type and the
        // fp32 accumulation:  DistMult (|dq| + d 2^-23 |q~|) Tmax;  TransE 2|dq|(|q~|+Tmax) + |dq|^2 +
        // d 2^-22 (|q~|+Tmax)^2, with Tmax the largest candidate norm; ComplEx and RotatE are the same two forms on
        // their own query (h * r, h * e^{ir}), whose fp32 evaluation error is part of dq.
        if (n >= KP && ncand > KP && K <= n) {
            const QInfo qi = qinfo[q];
            const double Tm = sqrt((double)*tmax2);
            double eps, exactK;
            if (dm) { eps = ((double)qi.eps_a + (double)qi.eps_b) * Tm; exactK = -key[K - 1]; }
            else if (m.scorer == KGE_TRANSH) {
                // value 2 q~.t - |t|^2 + (A~ - c)^2 against -key + |q~|^2 + c^2: the TransE terms for q~ (the
                // distance is taken to t_perp, no longer than t), then x = A - c: A~ is off by the rounding of the
                // normal to the table type (dw) and its fp32 accumulation, c (fp32 of u . q') by |dq| against u . q~.
                const double s = sqrt(qi.qn) + Tm, dq = qi.eps_a, dw = qi.eps_w, c = fabs((double)qi.c);
                const double wn = 1.0 + dw;                                            // |w~| <= |u| + |dw|
                const double dc = dq + 6e-8 * c;
                const double dx = (dw + (double)m.dim * 1.1920929e-07 * wn) * Tm + dc;
                const double xm = wn * Tm * 1.0001 + c;                                // |A~ - c| at most
                eps = 2.0 * dq * s + dq * dq + (double)qi.eps_b * s * s               // q~ for q', fp32 sums
                      + dx * (2.0 * xm + dx) + 4.8e-7 * (xm * xm + s * s)              // x~^2 for x^2, its fp32 evaluation
                      + dc * (2.0 * c + dc);                                           // c^2 for (u . q~)^2
                exactK = -key[K - 1] + qi.qn + (double)qi.c * (double)qi.c;
            } else {
                const double s = sqrt(qi.qn) + Tm;
                eps = 2.0 * qi.eps_a * s + (double)qi.eps_a * qi.eps_a + (double)qi.eps_b * s * s;
                exactK = -key[K - 1] + qi.qn;
            }
            eps = eps * 1.01 + 1e-30;
            if (!((double)thr[q] + eps < exactK)) flag[q] = 1;
        }
        if (out_rank) {
            const int tt = true_t[q];
            int64_t rank = 1 + (int64_t)rankcnt[q];
            bool in_range = tt >= cand_lo && tt < cand_lo + ncand;
            int pos = -1;
            const int lim = K < n ? K : n;
            for (int i = 0; i < lim; ++i) if (cand_lo + idx[i] == tt) { pos = i; break; }
            if (pos >= 0) rank = pos + 1;                    // exact: position in the fp64 ordering
            else if (in_range && rank <= lim) rank = lim + 1; // it is not in the exact list, so it ranks below it
            out_rank[q] = rank;
        }
    }
}

// exhaustive fp64 re-rank of one flagged query per workgroup
template <bool BF16>
__global__ void topk_exact_kernel(KgeModelDev m, const int32_t *h, const int32_t *r, int Q, int64_t cand_lo,
                                  int64_t ncand, int K, int32_t *out_idx, float *out_score, const int32_t *true_t,
                                  int64_t *out_rank, const int32_t *flag, const double *qx) {
    constexpr int CAPX = 2048;
    __shared__ double key[CAPX];
    __shared__ int idx[CAPX];
    __shared__ int count;
    __shared__ double tau;
    __shared__ unsigned long long above;
    const int q = blockIdx.x;
    if (q >= Q || !flag[q]) return;
    const int64_t hoff = (int64_t)h[q] * m.ent_ld, roff = (int64_t)r[q] * m.rel_ld;
    __shared__ double qv[TK_MAXD], wv[TK_MAXD];
    const bool th = m.scorer == KGE_TRANSH;
    for (int j = threadIdx.x; j < m.dim; j += blockDim.x) {
        if (th) { qv[j] = qx[(size_t)q * 2 * m.dim + j]; wv[j] = qx[(size_t)q * 2 * m.dim + m.dim + j]; }
        else qv[j] = query_f64<BF16>(m, hoff, roff, j);
    }
    auto key_of = [&](int64_t toff) {
        return th ? canonical_key_th<BF16>(m.dim, qv, wv, m.ent, toff) : canonical_key<BF16>(m.scorer, m.dim, qv, m.ent, toff);
    };
    if (threadIdx.x == 0) { count = 0; tau = INFINITY; above = 0ull; }
    for (int i = threadIdx.x; i < CAPX; i += blockDim.x) { key[i] = INFINITY; idx[i] = 0x7FFFFFFF; }
    __syncthreads();
    double tkey = 0.0; int tt = -1;
    if (true_t) { tt = true_t[q]; tkey = key_of((int64_t)tt * m.ent_ld); }
    unsigned long long mine = 0;
    for (int64_t c0 = 0; c0 < ncand; c0 += blockDim.x) {
        const int64_t c = c0 + threadIdx.x;
        if (c < ncand) {
            const double kc = key_of((cand_lo + c) * m.ent_ld);
            if (true_t && (kc < tkey || (kc == tkey && cand_lo + c < tt))) ++mine;
            if (kc <= tau) { const int s = atomicAdd(&count, 1); key[s] = kc; idx[s] = (int)c; }   // s < CAPX by the compaction below
        }
        __syncthreads();
        // every thread reads the counter between two barriers, so that no wave can start the next round's appends before
        // a slower one has taken the same decision
        const bool compact = count > CAPX - (int)blockDim.x;   // next round could overflow: compact to the K best
        __syncthreads();
        if (compact) {
            bitonic_asc_pair(key, idx, CAPX);
            if (threadIdx.x == 0) { count = K; tau = key[K - 1]; }
            __syncthreads();
            for (int i = K + threadIdx.x; i < CAPX; i += blockDim.x) { key[i] = INFINITY; idx[i] = 0x7FFFFFFF; }
            __syncthreads();
        }
    }
    bitonic_asc_pair(key, idx, CAPX);
    const bool dm = topk_mult(m.scorer);
    for (int i = threadIdx.x; i < K; i += blockDim.x) {
        const bool ok = idx[i] != 0x7FFFFFFF;
        out_idx[(size_t)q * K + i] = ok ? (int32_t)(cand_lo + idx[i]) : -1;
        out_score[(size_t)q * K + i] = ok ? (dm ? (float)(-key[i]) : (float)(-sqrt(key[i]))) : -INFINITY;
    }
    if (true_t) {
        atomicAdd(&above, mine);
        __syncthreads();
        if (threadIdx.x == 0) out_rank[q] = 1 + (int64_t)above;
    }
}

// ---------------------------------------------------------------------------------------------
// preparation
// ---------------------------------------------------------------------------------------------
// one wave per query: Q row in the table type, value of the held-out tail, rounding-bound coefficients
template <bool BF16>
__global__ void topk_prep_kernel(KgeModelDev m, const int32_t *h, const int32_t *r, const int32_t *true_t, int Q,
                                 int Qp, int dp, void *Qm, float *vt, QInfo *qinfo, float *thr, int32_t *cnt,
                                 int32_t *flag, uint32_t *rankcnt) {
    const int lane = threadIdx.x & 63;
    const int q = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (q >= Qp) return;
    if (q >= Q) {
        for (int j = lane; j < dp; j += 64) El<BF16>::st(Qm, (int64_t)q * dp + j, 0.f);
        if (lane == 0) { vt[q] = INFINITY; thr[q] = INFINITY; cnt[q] = 0; flag[q] = 0; rankcnt[q] = 0; }
        return;
    }
    KgeRowCtx<BF16> cx;
    kge_build_query<BF16>(m, h[q], r[q], lane, cx);
    const int d = m.dim;
    const bool mult = topk_mult(m.scorer);
    const int64_t hoff = (int64_t)h[q] * m.ent_ld, roff = (int64_t)r[q] * m.rel_ld;
    double qn = 0.0, dq2 = 0.0;
    float vtl = 0.f, tnl = 0.f;
    const int64_t toff = true_t ? (int64_t)true_t[q] * m.ent_ld : 0;
#pragma unroll
    for (int k = 0; k < KGE_MAXJ; ++k) {
        const int j = lane + 64 * k;
        const float qr = El<BF16>::rnd(cx.q[k]);
        // (TransE: stored doubled - exact - so that the scan's contraction yields 2 q.t directly)
        if (j < dp) El<BF16>::st(Qm, (int64_t)q * dp + j, mult ? cx.q[k] : 2.f * cx.q[k]);
        if (j >= d) continue;
        const double dq = (double)qr - query_f64<BF16>(m, hoff, roff, j);     // against the exact query component
        qn += (double)qr * (double)qr; dq2 += dq * dq;
        if (true_t) { const float tv = El<BF16>::ld(m.ent, toff + j); vtl += qr * tv; tnl += tv * tv; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        qn += __shfl_xor(qn, o); dq2 += __shfl_xor(dq2, o); vtl += __shfl_xor(vtl, o); tnl += __shfl_xor(tnl, o);
    }
    if (lane == 0) {
        QInfo qi;
        qi.qn = qn;
        qi.eps_a = (float)(sqrt(dq2) * 1.0001);
        qi.eps_b = mult ? (float)(d * 1.1920929e-07 * sqrt(qn) * 1.0001)                       // d 2^-23 |q~|
                                            : (float)((d + 2) * 2.3841858e-07);                  // (d+2) 2^-22: d products and the -|t|^2 start value
        qi.eps_w = 0.f; qi.c = 0.f;
        qinfo[q] = qi;
        vt[q] = true_t ? (mult ? vtl : 2.f * vtl - tnl) : INFINITY;
        thr[q] = -INFINITY; cnt[q] = 0; flag[q] = 0; rankcnt[q] = 0;
    }
}

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// TransH, one wave per query: unit normal u and q' = (h - (u.h) u) + r in fp64 (kept for the re-scoring), their
// roundings to the table type (q~ stored doubled, like TransE's), c = u . q', the value of the held-out tail
// and the rounding-bound coefficients.
template <bool BF16>
__global__ void topk_prep_th_kernel(KgeModelDev m, const int32_t *h, const int32_t *r, const int32_t *true_t, int Q,
                                    int Qp, int dp, void *Qm, void *Wm, float *cq, double *qx, float *vt, QInfo *qinfo,
                                    float *thr, int32_t *cnt, int32_t *flag, uint32_t *rankcnt) {
    const int lane = threadIdx.x & 63;
    const int q = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (q >= Qp) return;
    if (q >= Q) {
        for (int j = lane; j < dp; j += 64) { El<BF16>::st(Qm, (int64_t)q * dp + j, 0.f); El<BF16>::st(Wm, (int64_t)q * dp + j, 0.f); }
        if (lane == 0) { cq[q] = 0.f; vt[q] = INFINITY; thr[q] = INFINITY; cnt[q] = 0; flag[q] = 0; rankcnt[q] = 0; }
        return;
    }
    const int d = m.dim;
    const int64_t hoff = (int64_t)h[q] * m.ent_ld, roff = (int64_t)r[q] * m.rel_ld, woff = (int64_t)r[q] * m.relw_ld;
    double hv[KGE_MAXJ], rv[KGE_MAXJ], wv[KGE_MAXJ];
    double nn = 0.0;
#pragma unroll
    for (int k = 0; k < KGE_MAXJ; ++k) {
        const int j = lane + 64 * k;
        const bool ok = j < d;
        hv[k] = ok ? (double)El<BF16>::ld(m.ent, hoff + j) : 0.0;
        rv[k] = ok ? (double)El<BF16>::ld(m.rel, roff + j) : 0.0;
        wv[k] = ok ? (double)El<BF16>::ld(m.relw, woff + j) : 0.0;
        nn += wv[k] * wv[k];
    }
    nn = wave_sum_f64(nn);
    const double nrm = fmax(sqrt(nn), 1e-12);
    double wh = 0.0;
#pragma unroll
    for (int k = 0; k < KGE_MAXJ; ++k) { wv[k] = wv[k] / nrm; wh += wv[k] * hv[k]; }
    wh = wave_sum_f64(wh);
    double ce = 0.0, qn = 0.0, dq2 = 0.0, dw2 = 0.0;
    float qt = 0.f, tnl = 0.f, wt = 0.f;
    const int64_t toff = true_t ? (int64_t)true_t[q] * m.ent_ld : 0;
    double *qxq = qx + (size_t)q * 2 * d;
#pragma unroll
    for (int k = 0; k < KGE_MAXJ; ++k) {
        const int j = lane + 64 * k;
        const double qe = (hv[k] - wh * wv[k]) + rv[k];
        const float qr = El<BF16>::rnd((float)qe), wr = El<BF16>::rnd((float)wv[k]);
        if (j < dp) { El<BF16>::st(Qm, (int64_t)q * dp + j, 2.f * qr); El<BF16>::st(Wm, (int64_t)q * dp + j, wr); }
        if (j >= d) continue;
        qxq[j] = qe; qxq[d + j] = wv[k];
        ce += wv[k] * qe; qn += (double)qr * (double)qr;
        dq2 += ((double)qr - qe) * ((double)qr - qe); dw2 += ((double)wr - wv[k]) * ((double)wr - wv[k]);
        if (true_t) { const float tv = El<BF16>::ld(m.ent, toff + j); qt += qr * tv; tnl += tv * tv; wt += wr * tv; }
    }
    ce = wave_sum_f64(ce); qn = wave_sum_f64(qn); dq2 = wave_sum_f64(dq2); dw2 = wave_sum_f64(dw2);
    qt = kge_wave_sum(qt); tnl = kge_wave_sum(tnl); wt = kge_wave_sum(wt);
    if (lane == 0) {
        const float c = (float)ce;
        QInfo qi;
        qi.qn = qn;
        qi.eps_a = (float)(sqrt(dq2) * 1.0001);
        qi.eps_b = (float)((d + 2) * 2.3841858e-07);
        qi.eps_w = (float)(sqrt(dw2) * 1.0001);
        qi.c = c;
        qinfo[q] = qi;
        cq[q] = c;
        vt[q] = true_t ? fmaf(wt - c, wt - c, 2.f * qt - tnl) : INFINITY;
        thr[q] = -INFINITY; cnt[q] = 0; flag[q] = 0; rankcnt[q] = 0;
    }
}

// squared norms of the candidate rows (stored negated: the scan starts its accumulators from them) and their maximum, one
// atomic per wave.  Fast path (rows of 16-byte
// aligned power-of-two length): a lane reads 16 bytes, a wave 64 / LPR rows per step, four steps in flight.
template <bool BF16>
__global__ void topk_tnorm_kernel(const char *ent, int64_t stride, int d, int64_t ncand, int64_t npad, float *tn,
                                  uint32_t *tmax_bits) {
    const int lane = threadIdx.x & 63;
    const int64_t wid = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int64_t nw = (int64_t)gridDim.x * (blockDim.x >> 6);
    float mx = 0.f;
    const int rowb = d * (BF16 ? 2 : 4), lpr = rowb / 16;           // lanes per row
    const bool fast = rowb % 16 == 0 && lpr <= 64 && (lpr & (lpr - 1)) == 0 && stride % 16 == 0 && ((uintptr_t)ent & 15) == 0;
    if (fast) {
        const int rpw = 64 / lpr, sub = lane / lpr, li = lane % lpr;    // rows per wave step
        constexpr int U = 4;
        for (int64_t c0 = wid * rpw * U; c0 < npad; c0 += nw * rpw * U) {
            kge_u32x4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t c = c0 + u * rpw + sub;
                v[u] = kge_u32x4{0u, 0u, 0u, 0u};
                if (c < ncand) v[u] = *(const kge_u32x4 *)(ent + c * stride + li * 16);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float s = 0.f;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    if constexpr (BF16) {
                        const float a0 = __uint_as_float(v[u][k] << 16), a1 = __uint_as_float(v[u][k] & 0xffff0000u);
                        s += a0 * a0; s += a1 * a1;
                    } else { const float a0 = __uint_as_float(v[u][k]); s += a0 * a0; }
                }
                for (int o = lpr >> 1; o > 0; o >>= 1) s += __shfl_xor(s, o);
                const int64_t c = c0 + u * rpw + sub;
                if (li == 0 && c < npad) tn[c] = -s;
                mx = fmaxf(mx, s);
            }
        }
    } else {
        for (int64_t c = wid; c < npad; c += nw) {
            float s = 0.f;
            if (c < ncand) for (int j = lane; j < d; j += 64) { const float v = El<BF16>::ld(ent + c * stride, j); s += v * v; }
            s = kge_wave_sum(s);
            if (lane == 0) tn[c] = -s;
            mx = fmaxf(mx, s);
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    if (lane == 0) atomicMax(tmax_bits, __float_as_uint(mx));    // mx >= 0: bit order = value order
}

__global__ void topk_fill_empty_kernel(int32_t *out_idx, float *out_score, int64_t n, int64_t *out_rank, int Q) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) { out_idx[i] = -1; out_score[i] = -INFINITY; }
    if (out_rank && i < Q) out_rank[i] = 1;
}

__global__ void topk_zero_kernel(uint32_t *p, uint32_t *z) { if (threadIdx.x == 0) *p = 0u; if (threadIdx.x < 64) z[threadIdx.x] = 0u; }

struct TopkPlan {
    bool bf16, th; int es, rb, dp, ob, own, dim; int Qp; int KP, KPP, nseg; int64_t npad;
};

TopkPlan make_plan(const kge_model_t &m, int64_t Q, int64_t ncand, int K) {
    TopkPlan p{};
    p.bf16 = m.dtype == KGE_BF16; p.es = p.bf16 ? 2 : 4;
    p.rb = m.dim * p.es <= 512 ? 512 : 1024; p.dp = p.rb / p.es;
    p.th = m.scorer == KGE_TRANSH; p.dim = m.dim;
    p.ob = p.rb == 512 ? 2 : 1; p.own = p.th ? 128 : 128 * p.ob;          // TransH: the second row block holds the normals
    p.Qp = (int)kge_round_up(Q, p.own);
    p.KP = (int)kge_round_up(2 * K + 56, 64);
    p.KPP = 1; while (p.KPP < p.KP) p.KPP <<= 1;
    { int w = 1024 / (p.Qp / p.own); p.nseg = w < 32 ? 32 : (w > 256 ? 256 : w); }
    p.npad = kge_round_up(ncand > 0 ? ncand : 1, TK_ST);
    return p;
}

struct TopkWs {
    void *Qm; float *vt, *thr, *tn; QInfo *qinfo; int32_t *cnt, *flag, *redo; uint32_t *rankcnt, *tmax; uint2 *keep, *seg; int32_t *segcnt; double *keyd; uint32_t *zeros;
    void *Wm; float *cq; double *qx;                    // TransH only
};

size_t topk_carve(const TopkPlan &p, void *ws, TopkWs &w) {
    char *b = (char *)ws; size_t off = 0;
    auto take = [&](size_t bytes) { void *q = b ? b + off : nullptr; off += (bytes + 255) / 256 * 256; return q; };
    w.Qm = take((size_t)p.Qp * p.rb);
    w.vt = (float *)take((size_t)p.Qp * 4); w.thr = (float *)take((size_t)p.Qp * 4);
    w.qinfo = (QInfo *)take((size_t)p.Qp * sizeof(QInfo));
    w.cnt = (int32_t *)take((size_t)p.Qp * 4); w.flag = (int32_t *)take((size_t)p.Qp * 4);
    w.redo = (int32_t *)take((size_t)p.Qp * 4);
    w.rankcnt = (uint32_t *)take((size_t)p.Qp * 4); w.tmax = (uint32_t *)take(256); w.zeros = (uint32_t *)take(256);
    w.tn = (float *)take((size_t)p.npad * 4);
    w.keep = (uint2 *)take((size_t)p.Qp * p.KP * 8);
    w.seg = (uint2 *)take((size_t)p.Qp * p.nseg * 2 * TK_HALF * 8);
    w.segcnt = (int32_t *)take((size_t)p.Qp * p.nseg * 2 * 4);
    w.keyd = (double *)take((size_t)p.Qp * p.KP * 8);
    w.Wm = nullptr; w.cq = nullptr; w.qx = nullptr;
    if (p.th) {
        w.Wm = take((size_t)p.Qp * p.rb); w.cq = (float *)take((size_t)p.Qp * 4);
        w.qx = (double *)take((size_t)p.Qp * 2 * p.dim * 8);
    }
    return off + 256;
}

template <bool BF16, int RB, int KIND, int OB, bool TH = false>
int launch_scan(const TopkArgs &a, int own_tiles, int nsplit, hipStream_t st) {
    constexpr int NSTAGE = RB == 512 ? 4 : 3;
    constexpr int LDS = NSTAGE * TK_ST * RB + (NSTAGE + 1) * 4 * 256;
    static KgeLdsLimit lds_limit;
    if (lds_limit.set((const void *)topk_scan_kernel<BF16, RB, KIND, OB, TH>, LDS) != KGE_OK) return KGE_E_HIP;
    hipLaunchKernelGGL((topk_scan_kernel<BF16, RB, KIND, OB, TH>), dim3(own_tiles * ((nsplit + 7) / 8 * 8)), dim3(256), LDS, st, a);
    return kge_launch_status();
}

}  // namespace

size_t kge_topk_ws(const kge_model_t &model, int64_t Q, int64_t ncand, int K) {
    if (Q < 0 || ncand < 0 || K < 1 || K > 256) return 0;
    TopkPlan p = make_plan(model, Q, ncand, K);
    TopkWs w;
    return topk_carve(p, nullptr, w);
}

int kge_run_topk(const kge_model_t &model, const int32_t *h, const int32_t *r, int64_t Q, int64_t lo, int64_t hi,
                 int K, int32_t *out_idx, float *out_score, const int32_t *true_t, int64_t *out_rank, void *ws,
                 size_t ws_bytes, hipStream_t st) {
    (void)ws_bytes;
    const int64_t ncand = hi - lo;
    if (ncand == 0) {
        const int64_t n = Q * K;
        hipLaunchKernelGGL(topk_fill_empty_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, out_idx, out_score, n,
                           out_rank, (int)Q);
        return kge_launch_status();
    }
    const TopkPlan p = make_plan(model, Q, ncand, K);
    TopkWs w;
    topk_carve(p, ws, w);
    KgeModelDev md;
    md.scorer = model.scorer; md.bf16 = p.bf16; md.dim = model.dim; md.rel_dim = model.rel_dim; md.p1 = 0;
    md.ent = model.ent; md.rel = model.rel; md.relw = model.relw;
    md.ent_ld = model.ent_ld; md.rel_ld = model.rel_ld; md.relw_ld = model.relw_ld;
    const char *cand0 = (const char *)model.ent + lo * model.ent_ld * p.es;
    const int64_t stride = model.ent_ld * p.es;
    if (stride * TK_ST >= (1ll << 32)) return KGE_E_UNSUPPORTED;     // the scan advances its sources by a 32-bit step per tile
    const int kind = (model.scorer == KGE_DISTMULT || model.scorer == KGE_COMPLEX) ? KGE_KIND_MULT : KGE_KIND_DIST;

    hipLaunchKernelGGL(topk_zero_kernel, dim3(1), dim3(64), 0, st, w.tmax, w.zeros);
    if (p.th) {
        if (p.bf16) hipLaunchKernelGGL(topk_prep_th_kernel<true>, dim3((p.Qp + 3) / 4), dim3(256), 0, st, md, h, r, true_t, (int)Q, p.Qp, p.dp, w.Qm, w.Wm, w.cq, w.qx, w.vt, w.qinfo, w.thr, w.cnt, w.flag, w.rankcnt);
        else hipLaunchKernelGGL(topk_prep_th_kernel<false>, dim3((p.Qp + 3) / 4), dim3(256), 0, st, md, h, r, true_t, (int)Q, p.Qp, p.dp, w.Qm, w.Wm, w.cq, w.qx, w.vt, w.qinfo, w.thr, w.cnt, w.flag, w.rankcnt);
    }
    if (p.bf16) {
        if (!p.th) hipLaunchKernelGGL(topk_prep_kernel<true>, dim3((p.Qp + 3) / 4), dim3(256), 0, st, md, h, r, true_t, (int)Q, p.Qp, p.dp, w.Qm, w.vt, w.qinfo, w.thr, w.cnt, w.flag, w.rankcnt);
        hipLaunchKernelGGL(topk_tnorm_kernel<true>, dim3((unsigned)(p.npad / 4 < 8192 ? (p.npad + 3) / 4 : 8192)), dim3(256), 0, st, cand0, stride, model.dim, ncand, p.npad, w.tn, w.tmax);
    } else {
        if (!p.th) hipLaunchKernelGGL(topk_prep_kernel<false>, dim3((p.Qp + 3) / 4), dim3(256), 0, st, md, h, r, true_t, (int)Q, p.Qp, p.dp, w.Qm, w.vt, w.qinfo, w.thr, w.cnt, w.flag, w.rankcnt);
        hipLaunchKernelGGL(topk_tnorm_kernel<false>, dim3((unsigned)(p.npad / 4 < 8192 ? (p.npad + 3) / 4 : 8192)), dim3(256), 0, st, cand0, stride, model.dim, ncand, p.npad, w.tn, w.tmax);
    }
    if (hipGetLastError() != hipSuccess) return KGE_E_HIP;

    TopkArgs base{};
    base.Qmat = w.Qm; base.Wmat = w.Wm; base.cq = w.cq; base.ent = cand0; base.ent_stride = stride; base.valid_bytes = model.dim * p.es;
    base.ncand = ncand; base.cand_lo = lo; base.tn = w.tn; base.thr = w.thr; base.vt = w.vt; base.true_t = true_t;
    base.seg = w.seg; base.segcnt = w.segcnt; base.nseg = p.nseg; base.rankcnt = w.rankcnt; base.nq = (int)Q; base.zeros = w.zeros;
    const int own_tiles = p.Qp / p.own;
    const int64_t total_tiles = p.npad / TK_ST;
    // Growing chunks: thresholds are refreshed between chunks.  The first chunk appends everything (64
    // candidates per split and lane half fill a private area exactly); afterwards a chunk is 3x what has
    // been seen, so a query with a well-mixed candidate order appends about 3 KP entries per chunk,
    // spread over nsplit x 2 private areas of TK_HALF entries.
    int64_t seen = 0;
    const int compact_lds = TK_SORTCAP * 8;
    static KgeLdsLimit compact_limit;
    if (compact_limit.set((const void *)topk_compact_kernel, compact_lds) != KGE_OK) return KGE_E_HIP;
    while (seen < total_tiles) {
        int64_t tiles = seen == 0 ? (p.nseg * (TK_HALF / TK_ST) < 128 ? p.nseg * (TK_HALF / TK_ST) : 128) : 3 * seen;
        if (tiles > total_tiles - seen) tiles = total_tiles - seen;
        TopkArgs c = base;
        c.tile_lo = seen; c.tile_hi = seen + tiles; c.own_tiles = own_tiles;
        int want = p.nseg;                                    // one split per private area
        if (want > tiles) want = (int)tiles;
        c.tiles_per_wg = (int)((tiles + want - 1) / want);
        const int nsplit = (int)((tiles + c.tiles_per_wg - 1) / c.tiles_per_wg);
        int rc;
        {
            KgeProfScope prof(KGE_PROF_TOPK_SCAN, st);
            if (p.th) rc = p.bf16 ? launch_scan<true, 512, KGE_KIND_DIST, 2, true>(c, own_tiles, nsplit, st)
                                  : launch_scan<false, 512, KGE_KIND_DIST, 2, true>(c, own_tiles, nsplit, st);
            else if (p.bf16 && p.rb == 512) rc = kind == KGE_KIND_MULT ? launch_scan<true, 512, KGE_KIND_MULT, 2>(c, own_tiles, nsplit, st) : launch_scan<true, 512, KGE_KIND_DIST, 2>(c, own_tiles, nsplit, st);
            else if (p.bf16) rc = kind == KGE_KIND_MULT ? launch_scan<true, 1024, KGE_KIND_MULT, 1>(c, own_tiles, nsplit, st) : launch_scan<true, 1024, KGE_KIND_DIST, 1>(c, own_tiles, nsplit, st);
            else if (p.rb == 512) rc = kind == KGE_KIND_MULT ? launch_scan<false, 512, KGE_KIND_MULT, 2>(c, own_tiles, nsplit, st) : launch_scan<false, 512, KGE_KIND_DIST, 2>(c, own_tiles, nsplit, st);
            else rc = kind == KGE_KIND_MULT ? launch_scan<false, 1024, KGE_KIND_MULT, 1>(c, own_tiles, nsplit, st) : launch_scan<false, 1024, KGE_KIND_DIST, 1>(c, own_tiles, nsplit, st);
        }
        if (rc != KGE_OK) return rc;
        seen += tiles;
        const int areas_of = (nsplit + 7) / 8 * 8 < p.nseg ? (nsplit + 7) / 8 * 8 : p.nseg;
        hipLaunchKernelGGL(topk_compact_kernel, dim3((unsigned)Q), dim3(256), TK_SORTCAP_SMALL * 8, st, w.keep, w.cnt, w.seg, w.segcnt,
                           p.nseg, areas_of, p.KP, w.thr, w.flag, (int)Q, TK_SORTCAP_SMALL, w.redo, 0);
        hipLaunchKernelGGL(topk_compact_kernel, dim3((unsigned)Q), dim3(256), compact_lds, st, w.keep, w.cnt, w.seg, w.segcnt,
                           p.nseg, areas_of, p.KP, w.thr, w.flag, (int)Q, TK_SORTCAP, w.redo, 1);
    }
    const int64_t nres = Q * p.KP;
    const int final_lds = p.KPP * 12;
    if (p.bf16) {
        hipLaunchKernelGGL(topk_rescore_kernel<true>, dim3((unsigned)((nres / 64 + 3) / 4)), dim3(256), 0, st, md, h, r, (int)Q, lo, w.cnt, w.keep, p.KP, w.keyd, w.qx);
        hipLaunchKernelGGL(topk_final_kernel<true>, dim3((unsigned)Q), dim3(256), final_lds, st, md, h, r, (int)Q, lo, ncand, w.cnt, w.keep, p.KP, p.KPP, w.keyd, w.thr, w.qinfo, (const float *)w.tmax, K, out_idx, out_score, true_t, w.rankcnt, out_rank, w.flag);
        hipLaunchKernelGGL(topk_exact_kernel<true>, dim3((unsigned)Q), dim3(256), 0, st, md, h, r, (int)Q, lo, ncand, K, out_idx, out_score, true_t, out_rank, w.flag, w.qx);
    } else {
        hipLaunchKernelGGL(topk_rescore_kernel<false>, dim3((unsigned)((nres / 64 + 3) / 4)), dim3(256), 0, st, md, h, r, (int)Q, lo, w.cnt, w.keep, p.KP, w.keyd, w.qx);
        hipLaunchKernelGGL(topk_final_kernel<false>, dim3((unsigned)Q), dim3(256), final_lds, st, md, h, r, (int)Q, lo, ncand, w.cnt, w.keep, p.KP, p.KPP, w.keyd, w.thr, w.qinfo, (const float *)w.tmax, K, out_idx, out_score, true_t, w.rankcnt, out_rank, w.flag);
        hipLaunchKernelGGL(topk_exact_kernel<false>, dim3((unsigned)Q), dim3(256), 0, st, md, h, r, (int)Q, lo, ncand, K, out_idx, out_score, true_t, out_rank, w.flag, w.qx);
    }
    return kge_launch_status();
}
