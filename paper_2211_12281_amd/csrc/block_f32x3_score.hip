// The score block of kge_score (Table 2 against the shared negatives of eq. (negsamples)) for fp32 tables on the bf16
// matrix pipe.  The fp32 MFMA of gfx950 runs at 1/16 of the bf16 rate, so every fp32 operand is split into three bf16
// planes by the gather kernels, x = x1 + x2 + x3 with x1 = bf16(x), x2 = bf16(x - x1), x3 = bf16(x - x1 - x2) (the three 8-bit significands
// cover the 24 bits of the float: the residual is below 2^-24 |x|), and q . t is accumulated in fp32 from the six
// plane products of weight >= 2^-16: q1.t1 + q1.t2 + q2.t1 + q1.t3 + q2.t2 + q3.t1 (what is dropped is below
// 3 x 2^-24 |q| |t|, the size of the rounding of an fp32 contraction).  Six bf16 MFMAs replace sixteen fp32-rate ones.
//
// A workgroup (4 waves, one per SIMD: the own fragments of three planes take 192 registers) owns 128 negatives as
// B-operands in registers and streams the queries in tiles of 32 rows x 3 planes through an LDS ring of three stages
// filled by asynchronous copies (rows of 2 dp bytes, 16-byte chunks swizzled by row % 16).  Epilogue: the bilinear
// scorers store the contraction; the distance scorers (TransE, RotatE; TransH has a kernel of its own below, it needs a
// second contraction) take |q|^2 + |t|^2 - 2 q.t, redo entries where that cancels by direct differences of the fp32 rows, and
// store -sqrt.
#include "block_kernel.hpp"

// W32 null: one contraction, Qp holds the three planes of the queries; else TransH, Qp holds six (q', then the unit normal)
int kge_launch_score3(int kind, int dp, const void *Qp, const void *Tp, const float *Q32, const float *T32, const float *W32,
                      const KgeRowInfo *rowinfo, const float *tn, int B, int N, int Bp, int Np, float *S_out, hipStream_t st);

namespace {

constexpr int S3_ST = 32, S3_NSTAGE = 3;

struct Score3Args {
    const char *Qp, *Tp;                               // bf16 planes [3][Bp][DP], [3][Np][DP]
    const float *Q32, *T32;                            // the fp32 rows [Bp][DP], [Np][DP] (direct recomputation)
    const float *W32;                                  // TransH: the unit normals [Bp][DP]; Qp then holds SIX planes (q', then w)
    const KgeRowInfo *rowinfo;                         // |q|^2 of the queries
    const float *tn;                                   // |t|^2 of the negatives
    int B, N, Bp, Np, own_tiles, nsplit, tiles_per_split, str_tiles, xcd_per;
    float *S_out;                                      // [B][N]
};

template <int DP, int KIND>
__global__ __attribute__((amdgpu_flat_work_group_size(256, 256), amdgpu_waves_per_eu(1, 1)))
void score3_kernel(const Score3Args a) {
    constexpr int RB = DP * 2, KS = DP / 16;           // bytes of a plane row, k-steps of 16
    constexpr int PLANE = S3_ST * RB, STAGE = 3 * PLANE;
    constexpr int CPW = STAGE / 1024 / 4;              // 1 KB copies per wave and tile
    constexpr int LPW = CPW + 1;                       // plus the row information
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
    char *side_ring = lds + S3_NSTAGE * STAGE;         // [stage][wave][64 lanes x 16 bytes]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 31, g = lane >> 5;
    // workgroups that stream the same queries share a die
    const int xcd = blockIdx.x & 7, kk = blockIdx.x >> 3;
    // (workgroup ids go round the 8 dies: with 8 or more splits a die takes the splits congruent to it; with fewer, a
    // split takes 8 / splits dies and the own tiles are dealt over them)
    int own_tile, split;
    if (a.xcd_per == 1) { own_tile = kk % a.own_tiles; split = xcd + 8 * (kk / a.own_tiles); }
    else { split = xcd / a.xcd_per; own_tile = kk * a.xcd_per + xcd % a.xcd_per; }
    if (own_tile >= a.own_tiles || split >= a.nsplit) return;
    const int t0 = split * a.tiles_per_split;
    const int t1 = min(a.str_tiles, t0 + a.tiles_per_split);
    if (t0 >= t1) return;
    const int oidx = own_tile * 128 + wave * 32 + lr;  // this lane's negative

    uint4 own[3][KS];
#pragma unroll
    for (int p = 0; p < 3; ++p) {
        const char *src = a.Tp + ((size_t)p * a.Np + oidx) * RB + g * 16;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) own[p][ks] = *(const uint4 *)(src + ks * 32);
    }
    float o_tn = a.tn[oidx];

    // ---- staging: copy jj of this wave covers bytes [(wave CPW + jj) KB, + 1 KB) of the stage (three planes of 32 rows) ----
    int64_t x_off[CPW];
#pragma unroll
    for (int jj = 0; jj < CPW; ++jj) {
        const int byte = (wave * CPW + jj) * 1024 + lane * 16;
        const int p = byte / PLANE, within = byte % PLANE, r = within / RB, pos = (within % RB) / 16;
        x_off[jj] = (int64_t)p * a.Bp * RB + r * RB + ((pos ^ (r & 15)) * 16);
    }
    auto issue = [&](int tile, int slot) {
        tile = tile < t1 ? tile : t1 - 1;               // past the end: a harmless repeat keeps vmcnt uniform
        const uint32_t sbase = lds0 + (slot % S3_NSTAGE) * STAGE;
        const char *src = a.Qp + (size_t)tile * S3_ST * RB;
#pragma unroll
        for (int jj = 0; jj < CPW; ++jj)
            kge_async_copy16(src + x_off[jj], __builtin_amdgcn_readfirstlane(sbase + (wave * CPW + jj) * 1024));
        kge_async_copy16(a.rowinfo + tile * S3_ST + lr,
                         __builtin_amdgcn_readfirstlane(lds0 + S3_NSTAGE * STAGE + ((slot % S3_NSTAGE) * 4 + wave) * 1024));
    };
    int frag_off[8];                                    // chunk 2 ks + g of row lr at position chunk ^ (lr & 15)
#pragma unroll
    for (int b = 0; b < 8; ++b) frag_off[b] = lr * RB + 16 * ((2 * b + g) ^ (lr & 15));

    issue(t0, 0); issue(t0 + 1, 1);
    // the own operand must have arrived before the loop (a wait inside it would drain the ring)
#pragma unroll
    for (int p = 0; p < 3; ++p)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(own[p][ks].x), "+v"(own[p][ks].y), "+v"(own[p][ks].z), "+v"(own[p][ks].w));
    asm volatile("" : "+v"(o_tn));

    for (int t = t0; t < t1; ++t) {
        const int slot = t - t0;
        kge_wait_vmcnt<LPW>();                          // tile t has landed (this wave's part); tile t + 1 may be in flight
        __syncthreads();
        issue(t + 2, slot + 2);                         // into the stage that tile t - 1 vacated
        const char *stage = lds + (slot % S3_NSTAGE) * STAGE;
        const char *side = side_ring + ((slot % S3_NSTAGE) * 4 + wave) * 1024;
        kge_f32x16 acc0, acc1;
#pragma unroll
        for (int i = 0; i < 16; ++i) { acc0[i] = 0.f; acc1[i] = 0.f; }
        // the fragments of a k-step (one per plane) are requested two k-steps ahead of their MFMAs; the scheduling
        // barriers keep that order (the wave is alone on its SIMD: nothing else hides the LDS latency)
        uint4 q[KS][3];
        auto load_ks = [&](int ks) {
            const int fo = frag_off[ks & 7] + 256 * (ks >> 3);
#pragma unroll
            for (int p = 0; p < 3; ++p) q[ks][p] = *(const uint4 *)(stage + p * PLANE + fo);
        };
        load_ks(0); load_ks(1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (ks + 2 < KS) load_ks(ks + 2);
            __builtin_amdgcn_sched_barrier(0);
            acc0 = kge_mma16<true>(acc0, q[ks][2], own[0][ks]);     // small terms first
            acc1 = kge_mma16<true>(acc1, q[ks][0], own[2][ks]);
            acc0 = kge_mma16<true>(acc0, q[ks][1], own[1][ks]);
            acc1 = kge_mma16<true>(acc1, q[ks][1], own[0][ks]);
            acc0 = kge_mma16<true>(acc0, q[ks][0], own[1][ks]);
            acc1 = kge_mma16<true>(acc1, q[ks][0], own[0][ks]);
            __builtin_amdgcn_sched_barrier(0);
        }
        // register i holds stream row 8 (i / 4) + 4 g + i % 4 of the tile, own column lr
        float sv[16];
        if constexpr (KIND == KGE_KIND_MULT) {
#pragma unroll
            for (int i = 0; i < 16; ++i) sv[i] = acc0[i] + acc1[i];
        } else {
            float d2[16], thr[16];
            bool cancel = false;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int sl = 8 * (i >> 2) + 4 * g + (i & 3);
                const float qn = *(const float *)(side + sl * 16);
                d2[i] = fmaf(-2.f, acc0[i] + acc1[i], qn + o_tn);
                thr[i] = 1e-3f * (qn + o_tn);
                cancel = cancel || d2[i] < thr[i];
            }
            if (__any(cancel)) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    if (d2[i] < thr[i]) {
                        const int b = t * S3_ST + 8 * (i >> 2) + 4 * g + (i & 3);
                        d2[i] = kge_direct_d2<false, false>(a.Q32 + (size_t)b * DP, a.T32 + (size_t)oidx * DP, nullptr, DP);
                    }
                    asm volatile("" ::: "memory");      // keeps the branch from being turned into selects
                }
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float dd = fmaxf(d2[i], 0.f);
                sv[i] = dd > 0.f ? -dd * __builtin_amdgcn_rsqf(dd) : 0.f;   // -sqrt(d2)
            }
        }
        if (oidx < a.N) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int b = t * S3_ST + 8 * (i >> 2) + 4 * g + (i & 3);
                if (b < a.B) a.S_out[(size_t)b * a.N + oidx] = sv[i];
            }
        }
    }
    kge_wait_vmcnt<0>();                                // no copy may be in flight when the LDS is released
}

// TransH (two contractions per pair: q'.t and w.t, Table 2 with the expansion |q' - t + (w.t) w|^2 = |q'|^2 + |t|^2
// - 2 q'.t + A (2 w.q' - A (2 - |w|^2)), A = w.t): the stream carries the three planes of q' AND of w, so a stage of
// the ring holds a 256-byte piece of the rows (128 dimensions of six planes of 32 queries, 48 KB) and a tile takes
// DP / 128 stages; the accumulators live across the stages of a tile.
template <int DP>
__global__ __attribute__((amdgpu_flat_work_group_size(256, 256), amdgpu_waves_per_eu(1, 1)))
void score3h_kernel(const Score3Args a) {
    constexpr int RB = DP * 2, HB = 256, NH = RB / HB, KH = 8;        // bytes of a plane row, of a piece; pieces; k-steps per piece
    constexpr int PLANE = S3_ST * HB, STAGE = 6 * PLANE;
    constexpr int CPW = STAGE / 1024 / 4;
    constexpr int LPW = CPW + 1;
    static_assert(RB % HB == 0 && STAGE % 4096 == 0, "whole pieces, whole copies per wave");
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
    char *side_ring = lds + S3_NSTAGE * STAGE;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 31, g = lane >> 5;
    const int xcd = blockIdx.x & 7, kk = blockIdx.x >> 3;
    int own_tile, split;
    if (a.xcd_per == 1) { own_tile = kk % a.own_tiles; split = xcd + 8 * (kk / a.own_tiles); }
    else { split = xcd / a.xcd_per; own_tile = kk * a.xcd_per + xcd % a.xcd_per; }
    if (own_tile >= a.own_tiles || split >= a.nsplit) return;
    const int t0 = split * a.tiles_per_split;
    const int t1 = min(a.str_tiles, t0 + a.tiles_per_split);
    if (t0 >= t1) return;
    const int oidx = own_tile * 128 + wave * 32 + lr;

    uint4 own[3][NH * KH];
#pragma unroll
    for (int p = 0; p < 3; ++p) {
        const char *src = a.Tp + ((size_t)p * a.Np + oidx) * RB + g * 16;
#pragma unroll
        for (int ks = 0; ks < NH * KH; ++ks) own[p][ks] = *(const uint4 *)(src + ks * 32);
    }
    float o_tn = a.tn[oidx];

    // copy jj of this wave covers bytes [(wave CPW + jj) KB, + 1 KB) of the stage: six planes of 32 row pieces
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
        const uint32_t sbase = lds0 + (sidx % S3_NSTAGE) * STAGE;
        const char *src = a.Qp + (size_t)tile * S3_ST * RB + hf * HB;
#pragma unroll
        for (int jj = 0; jj < CPW; ++jj)
            kge_async_copy16(src + x_off[jj], __builtin_amdgcn_readfirstlane(sbase + (wave * CPW + jj) * 1024));
        kge_async_copy16(a.rowinfo + tile * S3_ST + lr,
                         __builtin_amdgcn_readfirstlane(lds0 + S3_NSTAGE * STAGE + ((sidx % S3_NSTAGE) * 4 + wave) * 1024));
    };
    int frag_off[KH];
#pragma unroll
    for (int b = 0; b < KH; ++b) frag_off[b] = lr * HB + 16 * ((2 * b + g) ^ (lr & 15));

    issue(0); issue(1);
#pragma unroll
    for (int p = 0; p < 3; ++p)
#pragma unroll
        for (int ks = 0; ks < NH * KH; ++ks) asm volatile("" : "+v"(own[p][ks].x), "+v"(own[p][ks].y), "+v"(own[p][ks].z), "+v"(own[p][ks].w));
    asm volatile("" : "+v"(o_tn));

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
            const char *stage = lds + (sidx % S3_NSTAGE) * STAGE;
            side = side_ring + ((sidx % S3_NSTAGE) * 4 + wave) * 1024;
            uint4 q[KH][3], w[KH][3];
            auto load_ks = [&](int ks) {
#pragma unroll
                for (int p = 0; p < 3; ++p) {
                    q[ks][p] = *(const uint4 *)(stage + p * PLANE + frag_off[ks]);
                    w[ks][p] = *(const uint4 *)(stage + (3 + p) * PLANE + frag_off[ks]);
                }
            };
            load_ks(0); load_ks(1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = 0; ks < KH; ++ks) {
                if (ks + 2 < KH) load_ks(ks + 2);
                __builtin_amdgcn_sched_barrier(0);
                const int ko = hf * KH + ks;
                aq0 = kge_mma16<true>(aq0, q[ks][2], own[0][ko]);       // small terms first
                aq1 = kge_mma16<true>(aq1, q[ks][0], own[2][ko]);
                aw0 = kge_mma16<true>(aw0, w[ks][2], own[0][ko]);
                aw1 = kge_mma16<true>(aw1, w[ks][0], own[2][ko]);
                aq0 = kge_mma16<true>(aq0, q[ks][1], own[1][ko]);
                aq1 = kge_mma16<true>(aq1, q[ks][1], own[0][ko]);
                aw0 = kge_mma16<true>(aw0, w[ks][1], own[1][ko]);
                aw1 = kge_mma16<true>(aw1, w[ks][1], own[0][ko]);
                aq0 = kge_mma16<true>(aq0, q[ks][0], own[1][ko]);
                aq1 = kge_mma16<true>(aq1, q[ks][0], own[0][ko]);
                aw0 = kge_mma16<true>(aw0, w[ks][0], own[1][ko]);
                aw1 = kge_mma16<true>(aw1, w[ks][0], own[0][ko]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // register i holds stream row 8 (i / 4) + 4 g + i % 4 of the tile, own column lr; the row information of the
        // tile came with each of its stages: the last one's copy is read
        float d2[16], thr[16];
        bool cancel = false;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int sl = 8 * (i >> 2) + 4 * g + (i & 3);
            const float4 ri = *(const float4 *)(side + sl * 16);        // |q'|^2, w.q', -, |w|^2
            const float A = aw0[i] + aw1[i];
            d2[i] = fmaf(-2.f, aq0[i] + aq1[i], ri.x + o_tn);
            d2[i] += A * (2.f * ri.y - A * (2.f - ri.w));
            thr[i] = 1e-3f * (ri.x + o_tn);
            cancel = cancel || d2[i] < thr[i];
        }
        if (__any(cancel)) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if (d2[i] < thr[i]) {
                    const int b = t * S3_ST + 8 * (i >> 2) + 4 * g + (i & 3);
                    d2[i] = kge_direct_d2<false, true>(a.Q32 + (size_t)b * DP, a.T32 + (size_t)oidx * DP, a.W32 + (size_t)b * DP, DP);
                }
                asm volatile("" ::: "memory");          // keeps the branch from being turned into selects
            }
        }
        if (oidx < a.N) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int b = t * S3_ST + 8 * (i >> 2) + 4 * g + (i & 3);
                const float dd = fmaxf(d2[i], 0.f);
                if (b < a.B) a.S_out[(size_t)b * a.N + oidx] = dd > 0.f ? -dd * __builtin_amdgcn_rsqf(dd) : 0.f;   // -sqrt(d2)
            }
        }
    }
    kge_wait_vmcnt<0>();                                // no copy may be in flight when the LDS is released
}

template <typename K>
int launch3_grid(K kern, int lds_bytes, bool &attr_set, const Score3Args &a, hipStream_t st) {
    if (!attr_set) {
        if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes) != hipSuccess)
            return KGE_E_HIP;
        attr_set = true;
    }
    Score3Args b = a;
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
int launch3h(const Score3Args &a, hipStream_t st) {
    constexpr int LDS = S3_NSTAGE * (6 * S3_ST * 256) + S3_NSTAGE * 4 * 1024;
    static_assert(LDS <= 160 * 1024, "LDS budget");
    static bool attr_set = false;
    return launch3_grid(score3h_kernel<DP>, LDS, attr_set, a, st);
}

template <int DP, int KIND>
int launch3(const Score3Args &a, hipStream_t st) {
    constexpr int LDS = S3_NSTAGE * (3 * S3_ST * DP * 2) + S3_NSTAGE * 4 * 1024;
    static_assert(LDS <= 160 * 1024, "LDS budget");
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute((const void *)score3_kernel<DP, KIND>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS) != hipSuccess)
            return KGE_E_HIP;
        attr_set = true;
    }
    Score3Args b = a;
    int groups;
    if (a.nsplit >= 8) { b.xcd_per = 1; groups = a.own_tiles * ((a.nsplit + 7) / 8); }
    else {
        int s2 = 1;
        while (s2 < a.nsplit) s2 <<= 1;
        b.xcd_per = 8 / s2;
        groups = (a.own_tiles + b.xcd_per - 1) / b.xcd_per;
    }
    hipLaunchKernelGGL((score3_kernel<DP, KIND>), dim3(8 * groups), dim3(256), LDS, st, b);
    return kge_launch_status();
}

}  // namespace

int kge_launch_score3(int kind, int dp, const void *Qp, const void *Tp, const float *Q32, const float *T32, const float *W32,
                      const KgeRowInfo *rowinfo, const float *tn, int B, int N, int Bp, int Np, float *S_out, hipStream_t st) {
    if (W32 && kind != KGE_KIND_DIST) return KGE_E_INVALID_ARG;
    if (Bp % S3_ST || Np % 128 || (dp != 128 && dp != 256)) return KGE_E_INVALID_ARG;
    if (Bp == 0 || Np == 0) return KGE_OK;
    Score3Args a{};
    a.Qp = (const char *)Qp; a.Tp = (const char *)Tp; a.Q32 = Q32; a.T32 = T32; a.rowinfo = rowinfo; a.tn = tn;
    a.B = B; a.N = N; a.Bp = Bp; a.Np = Np; a.S_out = S_out; a.W32 = W32;
    a.own_tiles = Np / 128; a.str_tiles = Bp / S3_ST;
    int want = (256 + a.own_tiles - 1) / a.own_tiles;           // about one workgroup per compute unit (one fits: 156 KB of LDS)
    if (want > a.str_tiles) want = a.str_tiles;
    if (want < 1) want = 1;
    a.tiles_per_split = (a.str_tiles + want - 1) / want;
    a.nsplit = (a.str_tiles + a.tiles_per_split - 1) / a.tiles_per_split;
    KgeProfScope prof(KGE_PROF_BLOCK_SCORE, st);
    if (W32) return dp == 256 ? launch3h<256>(a, st) : launch3h<128>(a, st);
    if (dp == 256) return kind == KGE_KIND_MULT ? launch3<256, KGE_KIND_MULT>(a, st) : launch3<256, KGE_KIND_DIST>(a, st);
    return kind == KGE_KIND_MULT ? launch3<128, KGE_KIND_MULT>(a, st) : launch3<128, KGE_KIND_DIST>(a, st);
}
