// The score block of kge_score (Table 2 against the shared negatives of eq. (negsamples)) for fp32 tables on the fp16
// matrix pipe.  The fp32 MFMA of gfx950 runs at 1/16 of the 16-bit rate, so the gather kernels also write every fp32
// row, scaled by a power of two s that brings its largest magnitude into [2^10, 2^11), as TWO fp16 planes:
// s x = x1 + x2, x1 = fp16(s x), x2 = fp16(s x - x1) (two 11-bit significands: the residual is below 2^-22 s |x| for
// every element whose second piece is a normal number, i.e. above 2^-17 of the row's maximum; smaller elements
// carry an absolute error below 2^-35 of the maximum).  q . t is accumulated in fp32 from the three plane products
// q1.t1 + q1.t2 + q2.t1 and multiplied by 1 / (s_q s_t), exact powers of two (what is dropped, q2.t2 and the residuals,
// is below 3 x 2^-22 |q| |t|): three 16-bit MFMAs replace sixteen fp32-rate ones.
//
// A workgroup (4 waves, one per SIMD) owns 128 negatives as B-operands in registers and streams the queries in tiles of
// 32 rows x 2 planes through an LDS ring of three stages filled by asynchronous copies (rows of 2 dp bytes, 16-byte
// chunks swizzled by row % 16).  Epilogue: the bilinear scorers store the contraction; the distance scorers (TransE,
// RotatE; TransH has a kernel of its own below, it needs a second contraction) take |q|^2 + |t|^2 - 2 q.t, redo
// entries where that cancels by direct differences of the fp32 rows, and store -sqrt.
#include "block_kernel.hpp"
#include "prep_kernels.h"

// W32 null: one contraction, Qp holds the two planes of the queries; else TransH, Qp holds four (q', then the unit normal)
int kge_launch_score_h2(int kind, int dp, const void *Qp, const void *Tp, const float *t_inv, const float *Q32, const float *T32,
                        const float *W32, const KgeRowInfo *rowinfo, const float *tn, int B, int N, int Bp, int Np, float *S_out,
                        hipStream_t st);

namespace {

constexpr int H2_ST = 32, H2_NSTAGE = 3;
constexpr int H2_NSTAGE_ONE = 2;                     // one-contraction kernel: two workgroups share a compute unit, two stages each

typedef _Float16 kge_f16x8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ kge_f32x16 h2_mma(kge_f32x16 acc, uint4 a, uint4 b) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(kge_f16x8, a), __builtin_bit_cast(kge_f16x8, b), acc, 0, 0, 0);
}

struct ScoreH2Args {
    const char *Qp, *Tp;                               // fp16 planes [2 (4)][Bp][DP], [2][Np][DP]
    const float *t_inv;                                // 1 / scale of the negatives' rows [Np]
    const float *Q32, *T32;                            // the fp32 rows [Bp][DP], [Np][DP] (direct recomputation)
    const float *W32;                                  // TransH: the unit normals [Bp][DP]
    const KgeRowInfo *rowinfo;                         // |q|^2 of the queries (TransH: w.q', |w|^2), K = 1 / scale of the row
    const float *tn;                                   // |t|^2 of the negatives
    int B, N, Bp, Np, own_tiles, nsplit, tiles_per_split, str_tiles, xcd_per;
    float *S_out;                                      // [B][N]
};

// workgroups that stream the same queries share a die (workgroup ids go round the 8 dies: with 8 or more splits a die
// takes the splits congruent to it; with fewer, a split takes 8 / splits dies and the own tiles are dealt over them)
__device__ __forceinline__ bool h2_place(const ScoreH2Args &a, int &own_tile, int &t0, int &t1) {
    const int xcd = blockIdx.x & 7, kk = blockIdx.x >> 3;
    int split;
    if (a.xcd_per == 1) { own_tile = kk % a.own_tiles; split = xcd + 8 * (kk / a.own_tiles); }
    else { split = xcd / a.xcd_per; own_tile = kk * a.xcd_per + xcd % a.xcd_per; }
    if (own_tile >= a.own_tiles || split >= a.nsplit) return false;
    t0 = split * a.tiles_per_split;
    t1 = min(a.str_tiles, t0 + a.tiles_per_split);
    return t0 < t1;
}

template <int DP, int KIND>
__global__ __attribute__((amdgpu_flat_work_group_size(256, 256), amdgpu_waves_per_eu(2, 2)))
void score_h2_kernel(const ScoreH2Args a) {
    constexpr int RB = DP * 2, KS = DP / 16;           // bytes of a plane row, k-steps of 16
    constexpr int PLANE = H2_ST * RB, STAGE = 2 * PLANE;
    constexpr int CPW = STAGE / 1024 / 4;              // 1 KB copies per wave and tile
    constexpr int LPW = CPW + 1;                       // plus the row information
    constexpr int NSTAGE = H2_NSTAGE_ONE, AHEAD = NSTAGE - 1;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
    char *side_ring = lds + NSTAGE * STAGE;         // [stage][wave][64 lanes x 16 bytes]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 31, g = lane >> 5;
    int own_tile, t0, t1;
    if (!h2_place(a, own_tile, t0, t1)) return;
    const int oidx = own_tile * 128 + wave * 32 + lr;  // this lane's negative

    uint4 own[2][KS];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const char *src = a.Tp + ((size_t)p * a.Np + oidx) * RB + g * 16;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) own[p][ks] = *(const uint4 *)(src + ks * 32);
    }
    float o_tn = a.tn[oidx], o_ti = a.t_inv[oidx];

    // ---- staging: copy jj of this wave covers bytes [(wave CPW + jj) KB, + 1 KB) of the stage (two planes of 32 rows) ----
    int64_t x_off[CPW];
#pragma unroll
    for (int jj = 0; jj < CPW; ++jj) {
        const int byte = (wave * CPW + jj) * 1024 + lane * 16;
        const int p = byte / PLANE, within = byte % PLANE, r = within / RB, pos = (within % RB) / 16;
        x_off[jj] = (int64_t)p * a.Bp * RB + r * RB + ((pos ^ (r & 15)) * 16);
    }
    auto issue = [&](int tile, int slot) {
        tile = tile < t1 ? tile : t1 - 1;               // past the end: a harmless repeat keeps vmcnt uniform
        const uint32_t sbase = lds0 + (slot % NSTAGE) * STAGE;
        const char *src = a.Qp + (size_t)tile * H2_ST * RB;
#pragma unroll
        for (int jj = 0; jj < CPW; ++jj)
            kge_async_copy16(src + x_off[jj], __builtin_amdgcn_readfirstlane(sbase + (wave * CPW + jj) * 1024));
        kge_async_copy16(a.rowinfo + tile * H2_ST + lr,
                         __builtin_amdgcn_readfirstlane(lds0 + NSTAGE * STAGE + ((slot % NSTAGE) * 4 + wave) * 1024));
    };
    int frag_off[8];                                    // chunk 2 ks + g of row lr at position chunk ^ (lr & 15)
#pragma unroll
    for (int b = 0; b < 8; ++b) frag_off[b] = lr * RB + 16 * ((2 * b + g) ^ (lr & 15));

#pragma unroll
    for (int s2 = 0; s2 < AHEAD; ++s2) issue(t0 + s2, s2);
    // the own operand must have arrived before the loop (a wait inside it would drain the ring)
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(own[p][ks].x), "+v"(own[p][ks].y), "+v"(own[p][ks].z), "+v"(own[p][ks].w));
    asm volatile("" : "+v"(o_tn), "+v"(o_ti));

    for (int t = t0; t < t1; ++t) {
        const int slot = t - t0;
        kge_wait_vmcnt<(AHEAD - 1) * LPW>();            // tile t has landed (this wave's part); later tiles may be in flight
        __syncthreads();
        issue(t + AHEAD, slot + AHEAD);                 // into the stage that tile t - 1 vacated
        const char *stage = lds + (slot % NSTAGE) * STAGE;
        const char *side = side_ring + ((slot % NSTAGE) * 4 + wave) * 1024;
        kge_f32x16 acc0, acc1;
#pragma unroll
        for (int i = 0; i < 16; ++i) { acc0[i] = 0.f; acc1[i] = 0.f; }
        // the fragments of a k-step (one per plane) are requested two k-steps ahead of their MFMAs; the scheduling
        // barriers keep that order (the wave is alone on its SIMD: nothing else hides the LDS latency)
        uint4 q[KS][2];
        auto load_ks = [&](int ks) {
            const int fo = frag_off[ks & 7] + 256 * (ks >> 3);
#pragma unroll
            for (int p = 0; p < 2; ++p) q[ks][p] = *(const uint4 *)(stage + p * PLANE + fo);
        };
        load_ks(0); load_ks(1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (ks + 2 < KS) load_ks(ks + 2);
            __builtin_amdgcn_sched_barrier(0);
            acc0 = h2_mma(acc0, q[ks][1], own[0][ks]);
            acc1 = h2_mma(acc1, q[ks][0], own[1][ks]);
            acc0 = h2_mma(acc0, q[ks][0], own[0][ks]);
            __builtin_amdgcn_sched_barrier(0);
        }
        // register i holds stream row 8 (i / 4) + 4 g + i % 4 of the tile, own column lr
        float sv[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int sl = 8 * (i >> 2) + 4 * g + (i & 3);
            sv[i] = (acc0[i] + acc1[i]) * (*(const float *)(side + sl * 16 + 8) * o_ti);
        }
        if constexpr (KIND != KGE_KIND_MULT) {
            float thr[16];
            bool cancel = false;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int sl = 8 * (i >> 2) + 4 * g + (i & 3);
                const float qn = *(const float *)(side + sl * 16);
                sv[i] = fmaf(-2.f, sv[i], qn + o_tn);
                thr[i] = 1e-3f * (qn + o_tn);
                cancel = cancel || sv[i] < thr[i];
            }
            if (__any(cancel)) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    if (sv[i] < thr[i]) {
                        const int b = t * H2_ST + 8 * (i >> 2) + 4 * g + (i & 3);
                        sv[i] = kge_direct_d2<false, false>(a.Q32 + (size_t)b * DP, a.T32 + (size_t)oidx * DP, nullptr, DP);
                    }
                    asm volatile("" ::: "memory");      // keeps the branch from being turned into selects
                }
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float dd = fmaxf(sv[i], 0.f);
                sv[i] = dd > 0.f ? -dd * __builtin_amdgcn_rsqf(dd) : 0.f;   // -sqrt(d2)
            }
        }
        if (oidx < a.N) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int b = t * H2_ST + 8 * (i >> 2) + 4 * g + (i & 3);
                if (b < a.B) a.S_out[(size_t)b * a.N + oidx] = sv[i];
            }
        }
    }
    kge_wait_vmcnt<0>();                                // no copy may be in flight when the LDS is released
}

// TransH (two contractions per pair: q'.t and w.t, Table 2 with the expansion |q' - t + (w.t) w|^2 = |q'|^2 + |t|^2
// - 2 q'.t + A (2 w.q' - A (2 - |w|^2)), A = w.t): the stream carries the two planes of q' AND of w (the unit normals
// all with the scale KGE_PLANE_UNIT_SCALE), a stage of the ring holds a 256-byte piece of the rows (128 dimensions of
// four planes of 32 queries, 32 KB) and a tile takes DP / 128 stages; the accumulators live across a tile's stages.
template <int DP>
__global__ __attribute__((amdgpu_flat_work_group_size(256, 256), amdgpu_waves_per_eu(1, 1)))
void score_h2_transh_kernel(const ScoreH2Args a) {
    constexpr int RB = DP * 2, HB = 256, NH = RB / HB, KH = 8;        // bytes of a plane row, of a piece; pieces; k-steps per piece
    constexpr int PLANE = H2_ST * HB, STAGE = 4 * PLANE;
    constexpr int CPW = STAGE / 1024 / 4;
    constexpr int LPW = CPW + 1;
    static_assert(RB % HB == 0 && STAGE % 4096 == 0, "whole pieces, whole copies per wave");
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
    char *side_ring = lds + H2_NSTAGE * STAGE;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 31, g = lane >> 5;
    int own_tile, t0, t1;
    if (!h2_place(a, own_tile, t0, t1)) return;
    const int oidx = own_tile * 128 + wave * 32 + lr;

    uint4 own[2][NH * KH];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const char *src = a.Tp + ((size_t)p * a.Np + oidx) * RB + g * 16;
#pragma unroll
        for (int ks = 0; ks < NH * KH; ++ks) own[p][ks] = *(const uint4 *)(src + ks * 32);
    }
    float o_tn = a.tn[oidx], o_ti = a.t_inv[oidx];

    // copy jj of this wave covers bytes [(wave CPW + jj) KB, + 1 KB) of the stage: four planes of 32 row pieces
    int64_t x_off[CPW];
#pragma unroll
    for (int jj = 0; jj < CPW; ++jj) {
        const int byte = (wave * CPW + jj) * 1024 + lane * 16;
        const int p = byte / PLANE, within = byte % PLANE, r = within / HB, pos = (within % HB) / 16;
        x_off[jj] = (int64_t)p * a.Bp * RB + r * RB + ((pos ^ (r & 15)) * 16);
    }
    const int n_stage = (t1 - t0) * NH;
    auto issue = [&](int sidx) {                        // stage sidx of this workgroup: piece sidx % NH of tile t0 + sidx / NH
        const int sc = sidx < n_stage ? sidx : n_stage - 1;     // past the end: a harmless repeat keeps vmcnt uniform
        const int tile = t0 + sc / NH, hf = sc % NH;
        const uint32_t sbase = lds0 + (sidx % H2_NSTAGE) * STAGE;
        const char *src = a.Qp + (size_t)tile * H2_ST * RB + hf * HB;
#pragma unroll
        for (int jj = 0; jj < CPW; ++jj)
            kge_async_copy16(src + x_off[jj], __builtin_amdgcn_readfirstlane(sbase + (wave * CPW + jj) * 1024));
        kge_async_copy16(a.rowinfo + tile * H2_ST + lr,
                         __builtin_amdgcn_readfirstlane(lds0 + H2_NSTAGE * STAGE + ((sidx % H2_NSTAGE) * 4 + wave) * 1024));
    };
    int frag_off[KH];
#pragma unroll
    for (int b = 0; b < KH; ++b) frag_off[b] = lr * HB + 16 * ((2 * b + g) ^ (lr & 15));

    issue(0); issue(1);
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int ks = 0; ks < NH * KH; ++ks) asm volatile("" : "+v"(own[p][ks].x), "+v"(own[p][ks].y), "+v"(own[p][ks].z), "+v"(own[p][ks].w));
    asm volatile("" : "+v"(o_tn), "+v"(o_ti));

    for (int t = t0; t < t1; ++t) {
        kge_f32x16 aq0, aq1, aw0, aw1;
#pragma unroll
        for (int i = 0; i < 16; ++i) { aq0[i] = 0.f; aq1[i] = 0.f; aw0[i] = 0.f; aw1[i] = 0.f; }
        const char *side = nullptr;
#pragma unroll
        for (int hf = 0; hf < NH; ++hf) {
            const int sidx = (t - t0) * NH + hf;
            kge_wait_vmcnt<LPW>();                      // stage sidx has landed (this wave's part); the next may be in flight
            __syncthreads();
            issue(sidx + 2);                            // into the stage that sidx - 1 vacated
            const char *stage = lds + (sidx % H2_NSTAGE) * STAGE;
            side = side_ring + ((sidx % H2_NSTAGE) * 4 + wave) * 1024;
            uint4 q[KH][2], w[KH][2];
            auto load_ks = [&](int ks) {
#pragma unroll
                for (int p = 0; p < 2; ++p) {
                    q[ks][p] = *(const uint4 *)(stage + p * PLANE + frag_off[ks]);
                    w[ks][p] = *(const uint4 *)(stage + (2 + p) * PLANE + frag_off[ks]);
                }
            };
            load_ks(0); load_ks(1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = 0; ks < KH; ++ks) {
                if (ks + 2 < KH) load_ks(ks + 2);
                __builtin_amdgcn_sched_barrier(0);
                const int ko = hf * KH + ks;
                aq0 = h2_mma(aq0, q[ks][1], own[0][ko]);
                aq1 = h2_mma(aq1, q[ks][0], own[1][ko]);
                aw0 = h2_mma(aw0, w[ks][1], own[0][ko]);
                aw1 = h2_mma(aw1, w[ks][0], own[1][ko]);
                aq0 = h2_mma(aq0, q[ks][0], own[0][ko]);
                aw0 = h2_mma(aw0, w[ks][0], own[0][ko]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // register i holds stream row 8 (i / 4) + 4 g + i % 4 of the tile, own column lr; the row information of the
        // tile came with each of its stages: the last one's copy is read
        float d2[16], thr[16];
        bool cancel = false;
        const float w_ti = o_ti * (1.f / KGE_PLANE_UNIT_SCALE);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int sl = 8 * (i >> 2) + 4 * g + (i & 3);
            const float4 ri = *(const float4 *)(side + sl * 16);        // |q'|^2, w.q', 1 / scale of q', |w|^2
            const float A = (aw0[i] + aw1[i]) * w_ti;
            d2[i] = fmaf(-2.f, (aq0[i] + aq1[i]) * (ri.z * o_ti), ri.x + o_tn);
            d2[i] += A * (2.f * ri.y - A * (2.f - ri.w));
            thr[i] = 1e-3f * (ri.x + o_tn);
            cancel = cancel || d2[i] < thr[i];
        }
        if (__any(cancel)) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if (d2[i] < thr[i]) {
                    const int b = t * H2_ST + 8 * (i >> 2) + 4 * g + (i & 3);
                    d2[i] = kge_direct_d2<false, true>(a.Q32 + (size_t)b * DP, a.T32 + (size_t)oidx * DP, a.W32 + (size_t)b * DP, DP);
                }
                asm volatile("" ::: "memory");          // keeps the branch from being turned into selects
            }
        }
        if (oidx < a.N) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int b = t * H2_ST + 8 * (i >> 2) + 4 * g + (i & 3);
                const float dd = fmaxf(d2[i], 0.f);
                if (b < a.B) a.S_out[(size_t)b * a.N + oidx] = dd > 0.f ? -dd * __builtin_amdgcn_rsqf(dd) : 0.f;   // -sqrt(d2)
            }
        }
    }
    kge_wait_vmcnt<0>();                                // no copy may be in flight when the LDS is released
}

template <typename K>
int launch_h2(K kern, int lds_bytes, KgeLdsLimit &lds_limit, const ScoreH2Args &a, hipStream_t st) {
    if (lds_limit.set((const void *)kern, lds_bytes) != KGE_OK) return KGE_E_HIP;
    ScoreH2Args b = a;
    int groups;
    if (a.nsplit >= 8) { b.xcd_per = 1; groups = a.own_tiles * ((a.nsplit + 7) / 8); }
    else {
        int s2 = 1;
        while (s2 < a.nsplit) s2 <<= 1;
        b.xcd_per = 8 / s2;
        groups = (a.own_tiles + b.xcd_per - 1) / b.xcd_per;
    }
    hipLaunchKernelGGL(kern, dim3(8 * groups), dim3(256), lds_bytes, st, b);
    return kge_launch_status();
}

template <int DP>
int launch_transh(const ScoreH2Args &a, hipStream_t st) {
    constexpr int LDS = H2_NSTAGE * (4 * H2_ST * 256) + H2_NSTAGE * 4 * 1024;
    static_assert(LDS <= 160 * 1024, "LDS budget");
    static KgeLdsLimit lds_limit;
    return launch_h2(score_h2_transh_kernel<DP>, LDS, lds_limit, a, st);
}

template <int DP, int KIND>
int launch_one(const ScoreH2Args &a, hipStream_t st) {
    constexpr int LDS = H2_NSTAGE_ONE * (2 * H2_ST * DP * 2) + H2_NSTAGE_ONE * 4 * 1024;
    static_assert(2 * LDS <= 160 * 1024, "LDS budget of two workgroups");
    static KgeLdsLimit lds_limit;
    return launch_h2(score_h2_kernel<DP, KIND>, LDS, lds_limit, a, st);
}

}  // namespace

int kge_launch_score_h2(int kind, int dp, const void *Qp, const void *Tp, const float *t_inv, const float *Q32, const float *T32,
                        const float *W32, const KgeRowInfo *rowinfo, const float *tn, int B, int N, int Bp, int Np, float *S_out,
                        hipStream_t st) {
    if (!t_inv || (W32 && kind != KGE_KIND_DIST)) return KGE_E_INVALID_ARG;
    if (Bp % H2_ST || Np % 128 || (dp != 128 && dp != 256)) return KGE_E_INVALID_ARG;
    if (Bp == 0 || Np == 0) return KGE_OK;
    ScoreH2Args a{};
    a.Qp = (const char *)Qp; a.Tp = (const char *)Tp; a.t_inv = t_inv; a.Q32 = Q32; a.T32 = T32; a.W32 = W32;
    a.rowinfo = rowinfo; a.tn = tn; a.B = B; a.N = N; a.Bp = Bp; a.Np = Np; a.S_out = S_out;
    a.own_tiles = Np / 128; a.str_tiles = Bp / H2_ST;
    const int wgs = W32 ? 256 : 512;                            // one workgroup per compute unit (TransH), or two
    int want = (wgs + a.own_tiles - 1) / a.own_tiles;
    if (want > a.str_tiles) want = a.str_tiles;
    if (want < 1) want = 1;
    a.tiles_per_split = (a.str_tiles + want - 1) / want;
    a.nsplit = (a.str_tiles + a.tiles_per_split - 1) / a.tiles_per_split;
    KgeProfScope prof(KGE_PROF_BLOCK_SCORE, st);
    if (W32) return dp == 256 ? launch_transh<256>(a, st) : launch_transh<128>(a, st);
    if (dp == 256) return kind == KGE_KIND_MULT ? launch_one<256, KGE_KIND_MULT>(a, st) : launch_one<256, KGE_KIND_DIST>(a, st);
    return kind == KGE_KIND_MULT ? launch_one<128, KGE_KIND_MULT>(a, st) : launch_one<128, KGE_KIND_DIST>(a, st);
}
