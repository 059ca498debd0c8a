// The shared-negative block kernel (gfx950, wave64, MFMA 32x32).
//
// The micro-batch's queries Q [B, d] (built from h and r) meet ONE block of negative tails
// T [N, d] shared by all of them (arXiv 2211.12281, Section 4 "Training", eq. (negsamples)), so the
// B x N scores of Table 2 are a dense contraction Q T^t followed by an elementwise map; the loss of
// Section 3.1 needs row reductions of that block, and its backward pass two more contractions
// (G T and G^t Q).  The block itself never goes to memory: it is recomputed tile by tile.
//
// One template serves all passes.  A workgroup (4 waves) OWNS 128 rows of one operand, held in
// registers as MFMA B-fragments for the whole launch, and STREAMS the other operand through an LDS
// ring of 2-4 stages in tiles of 32 rows.  The ring is filled by asynchronous global->LDS copies
// (no registers, several tiles in flight); rows are stored unpadded with their 16-byte chunks
// XOR-swizzled so that the fragment reads of 8 consecutive rows hit 8 different bank groups.
// Workgroups that stream the same rows are placed on the same XCD (shared L2).  Per tile and wave:
//   phase 1   acc[32 stream x 32 own] = X_tile . own^t          (contraction over d)
//   epilogue  score / loss weights / gradient coefficients, element by element
//   phase 2   out^t[d x 32 own] += Xt_tile[d x 32 stream] . coef[stream x own]
//             (contraction over the stream index; the coefficients go from the accumulator
//             registers straight into the B-operand, the transposed tile Xt supplies the A-fragments)
// In both phases an own row lives in ONE lane pair (l, l+32), so every per-row quantity (running
// maximum, sums, rescaling factors) is a per-lane scalar.
//
//   MODE_SCORE  own = negatives, stream = queries : writes the scores S[b, n]
//   MODE_FWD    own = queries,   stream = negatives: one pass gives the loss statistics of each row
//               (running max / sum of the softmax weights, weighted loss terms) AND the
//               unnormalised gradient of the queries, rescaled online when the running max moves
//   MODE_GRADT  own = negatives, stream = queries : gradient of the negatives, needs the per-row
//               constants that MODE_FWD's statistics produce
//
// Accumulator layout of v_mfma_f32_32x32x*: lane l holds column (l & 31) and, in register i,
// row 8*(i/4) + 4*(l/32) + (i%4).
#pragma once
#include "kge_internal.h"
#include <type_traits>

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 kge_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float kge_f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float kge_f32x4;
typedef uint32_t kge_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t kge_u32x2 __attribute__((ext_vector_type(2)));

constexpr float KGE_LOG2E = 1.4426950408889634f;
constexpr float KGE_LN2 = 0.6931471805599453f;
constexpr float KGE_TAU = 8.f;     // log2 headroom of the softmax weights over their reference exponent

template <bool BF16> struct KgeElem;
template <> struct KgeElem<true>  { using type = __bf16; static constexpr int size = 2; };
template <> struct KgeElem<false> { using type = float;  static constexpr int size = 4; };

// acc += A(16 bytes per lane) . B(16 bytes per lane): one 32x32x16 bf16 MFMA, or four 32x32x2 fp32
template <bool BF16>
__device__ __forceinline__ kge_f32x16 kge_mma16(kge_f32x16 acc, uint4 a, uint4 b) {
    if constexpr (BF16) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(kge_bf16x8, a),
                                                       __builtin_bit_cast(kge_bf16x8, b), acc, 0, 0, 0);
    } else {
        kge_f32x4 fa = __builtin_bit_cast(kge_f32x4, a), fb = __builtin_bit_cast(kge_f32x4, b);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[0], fb[0], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[1], fb[1], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[2], fb[2], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[3], fb[3], acc, 0, 0, 0);
        return acc;
    }
}

__device__ __forceinline__ uint32_t kge_pack_bf16x2(float lo, float hi) {
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf2;
    bf2 v = { (__bf16)lo, (__bf16)hi };          // round-to-nearest-even, lo in bits 0..15
    return __builtin_bit_cast(uint32_t, v);
}

// fp32 operands on the bf16 matrix pipe.  The fp32 MFMA of gfx950 runs at 1/16 of the bf16 rate, so the fp32 passes
// whose registers allow it (KgeBlockCfg::X3) split every operand value into THREE bf16 pieces, x = x0 + x1 + x2 with x0 = bf16(x), x1 = bf16(x - x0),
// x2 = bf16(x - x0 - x1) (round to nearest; 8 significand bits each, |x1| <= 2^-9 |x|, |x2| <= 2^-18 |x|; the bf16
// exponent range is that of fp32, so no scaling is needed), and accumulate the six products of total order <= 2 in
// fp32: a.b = a0 b0 + a0 b1 + a1 b0 + a1 b1 + a0 b2 + a2 b0 + O(2^-26 |a| |b|).  Six 32x32x16 bf16 MFMAs (192 cycles)
// replace the eight 32x32x2 fp32 ones (512 cycles) of sixteen k-steps.
// Eight values of a lane (two 16-byte fragments: slot j of lane half g of both operands is one contraction index,
// whatever its number) become three bf16 fragments.
struct KgeP3 { uint4 p[3]; };
__device__ __forceinline__ KgeP3 kge_split3(uint4 a, uint4 b) {
    const uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    uint32_t q[3][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float x0 = __uint_as_float(w[2 * i]), x1 = __uint_as_float(w[2 * i + 1]);
#pragma unroll
        for (int pl = 0; pl < 3; ++pl) {
            const uint32_t pk = kge_pack_bf16x2(x0, x1);
            q[pl][i] = pk;
            if (pl < 2) { x0 -= __uint_as_float(pk << 16); x1 -= __uint_as_float(pk & 0xffff0000u); }
        }
    }
    KgeP3 r;
#pragma unroll
    for (int pl = 0; pl < 3; ++pl) r.p[pl] = make_uint4(q[pl][0], q[pl][1], q[pl][2], q[pl][3]);
    return r;
}
// acc += A . B over the sixteen contraction indices of two fragment pairs (smallest terms first)
__device__ __forceinline__ kge_f32x16 kge_mma3(kge_f32x16 acc, const KgeP3 &A, const KgeP3 &B) {
    auto mm = [](kge_f32x16 c, uint4 x, uint4 y) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(kge_bf16x8, x), __builtin_bit_cast(kge_bf16x8, y), c, 0, 0, 0);
    };
    acc = mm(acc, A.p[0], B.p[2]);
    acc = mm(acc, A.p[2], B.p[0]);
    acc = mm(acc, A.p[1], B.p[1]);
    acc = mm(acc, A.p[0], B.p[1]);
    acc = mm(acc, A.p[1], B.p[0]);
    acc = mm(acc, A.p[0], B.p[0]);
    return acc;
}

// Asynchronous global -> LDS copies: lane l of a wave-wide instruction writes its 16 (4) bytes to LDS
// byte address m0 + 16 l (4 l).  Completion is tracked by vmcnt; the compiler does not see these
// loads, so the waits are explicit.
__device__ __forceinline__ void kge_async_copy16(const void *g, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(g) : "memory");
}
__device__ __forceinline__ void kge_async_copy4(const void *g, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_addr), "v"(g) : "memory");
}
template <int N> __device__ __forceinline__ void kge_wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

__device__ __forceinline__ float kge_elem_to_float(float x) { return x; }
__device__ __forceinline__ float kge_elem_to_float(__bf16 x) { return (float)x; }
__device__ __forceinline__ float kge_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float kge_log2(float x) { return __builtin_amdgcn_logf(x); }

// Squared distance of one (query, tail) pair by direct differences; the fallback for block entries
// whose norm-expansion form cancels.  TransH: u = q - t + (w.t) w.
template <bool BF16, bool TRANSH>
__device__ __noinline__ float kge_direct_d2(const void *qv, const void *tv, const void *wv, int dp) {
    using E = typename KgeElem<BF16>::type;
    const E *q = (const E *)qv, *t = (const E *)tv, *w = (const E *)wv;
    float A = 0.f;
    if constexpr (TRANSH)
        for (int j = 0; j < dp; ++j) A += kge_elem_to_float(w[j]) * kge_elem_to_float(t[j]);
    float acc = 0.f;
    for (int j = 0; j < dp; ++j) {
        float x = kge_elem_to_float(q[j]) - kge_elem_to_float(t[j]);
        if constexpr (TRANSH) x += A * kge_elem_to_float(w[j]);
        acc += x * x;
    }
    return acc;
}

template <bool BF16, int RB, int MODE, bool TRANSH, int KIND, int DSPLIT>
struct KgeBlockCfg {
    static constexpr bool OWN_ROW = MODE == KGE_MODE_FWD;
    static constexpr int OW = kge_block_ow(BF16, RB, TRANSH, MODE, KIND);   // 32-row own fragments per wave
    static constexpr int OWN_TILE = 128 * OW;              // own rows of a workgroup
    static constexpr int ES = KgeElem<BF16>::size;
    static constexpr int DP = RB / ES;                     // padded dim
    static constexpr int KS = RB / 32;                     // 32-byte k-steps of phase 1
    static constexpr int ST = KGE_STREAM_TILE;
    static constexpr int NB = DP / 32;                     // 32-column output blocks of phase 2
    static constexpr int NBH = NB / DSPLIT;                // ... handled by one z-slice
    static constexpr int X_BYTES = ST * RB;                // [ST rows][RB bytes], chunk c of row r at c ^ (r & 7)
    static constexpr int XT_ROWB = ST * ES;                // one transposed row: ST stream entries (64 or 128 bytes)
    static constexpr int XT_BYTES = DP * XT_ROWB;
    static constexpr bool HAS_X2 = TRANSH && !OWN_ROW;     // second streamed operand (normals)
    static constexpr bool HAS_XT = MODE != KGE_MODE_SCORE;
    static constexpr int NX = HAS_X2 ? 2 : 1;
    static constexpr int STAGE_BYTES = X_BYTES * NX + (HAS_XT ? XT_BYTES * NX : 0);
    static constexpr int SIDE_SLOT = OWN_ROW ? 4 * 256 : 4 * 1024;   // per-wave copies of the tile's side info
    // Workgroups per compute unit (= waves per SIMD): two where a workgroup's registers fit in 256, so that
    // the MFMA, LDS and vector phases of one workgroup run under those of the other.
    // fp32 training passes that contract bf16 pieces (kge_split3 / kge_mma3): the own operand's pieces take 1.5 times the
    // registers of its fp32 fragments, which the pass over the queries has only for rows of up to 512 bytes (measured, rows
    // of 1,024 bytes: pass over the negatives 550 -> 461 us, pass over the queries 589 -> 727 us with 170-320 bytes of
    // scratch).  The score block of this kernel stays on the fp32 instructions: kge_score on fp32 tables runs
    // block_f32h2_score.hip, and this one is what that is compared with.
    static constexpr bool X3 = !BF16 && ((MODE == KGE_MODE_FWD && RB <= 512) || MODE == KGE_MODE_GRADT);
    static constexpr int OCC = kge_block_occ(BF16, RB, TRANSH, MODE);
    static constexpr int LDS_MAX = 160 * 1024 / OCC;
    static constexpr int NSTAGE_RAW = (LDS_MAX - SIDE_SLOT) / (STAGE_BYTES + SIDE_SLOT);   // n stages + (n+1) side slots fit
    static constexpr int NSTAGE = NSTAGE_RAW > 4 ? 4 : NSTAGE_RAW;
    static constexpr int SIDE_SLOTS = NSTAGE + 1;
    static constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES + SIDE_SLOTS * SIDE_SLOT;
    static constexpr int X_IPW = X_BYTES / 1024 / 4;       // 1 KB wave-wide copies per wave and tile
    static constexpr int XT_IPW = XT_BYTES / 1024 / 4;
    static constexpr int LPW = X_IPW * NX + (HAS_XT ? XT_IPW * NX : 0) + 1;
    static_assert(NSTAGE >= 2, "two stages must fit");
    static_assert(X_BYTES % 4096 == 0 && XT_BYTES % 4096 == 0, "tile copies must divide over four waves");
    static_assert((NSTAGE - 2) * LPW < 64, "vmcnt range");
    static_assert(OW == 1 || !TRANSH, "two own fragments per wave leave no registers for the TransH operands");
    static_assert(KS % 8 == 0, "phase 1 works in groups of four fragments, split in two halves");
};

template <bool BF16, int RB, int MODE, bool TRANSH, int KIND, int LOSS, int DSPLIT>
__global__ __attribute__((amdgpu_flat_work_group_size(256, 256),
                          amdgpu_waves_per_eu(kge_block_occ(BF16, RB, TRANSH, MODE), kge_block_occ(BF16, RB, TRANSH, MODE))))
void kge_block_kernel(const KgeBlockArgs a) {
    using C = KgeBlockCfg<BF16, RB, MODE, TRANSH, KIND, DSPLIT>;
    constexpr bool OWN_ROW = C::OWN_ROW;
    constexpr bool PHASE2 = MODE != KGE_MODE_SCORE;
    constexpr int OW = C::OW;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
    char *side_ring = lds + C::NSTAGE * C::STAGE_BYTES;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 31, g = lane >> 5;
    // Workgroups go to the 8 XCDs round-robin: the workgroups that stream the same rows (same split)
    // get ids with the same residue mod 8 and share that XCD's L2.
    // With fewer than 8 splits, each split's own-tiles are dealt to 8 / nsplit XCDs.
    const int xcd = blockIdx.x & 7, kk = blockIdx.x >> 3;
    int own_tile, split;
    if (a.xcd_per == 1) { own_tile = kk % a.own_tiles; split = xcd + 8 * (kk / a.own_tiles); }
    else { split = xcd / a.xcd_per; own_tile = kk * a.xcd_per + xcd % a.xcd_per; }
    if (own_tile >= a.own_tiles) return;
    const int own_base = own_tile * C::OWN_TILE;
    const int dblk0 = blockIdx.y * C::NBH;
    const int oidx0 = own_base + wave * 32 * OW + lr;     // own row of fragment h: oidx0 + 32 h
    const int t0 = split * a.tiles_per_split;
    const int t1 = min(a.str_tiles, t0 + a.tiles_per_split);
    const int str_limit = OWN_ROW ? a.N : a.B;            // valid stream rows
    if (split >= a.nsplit) return;

    // ---- own operand fragments: 16 bytes per lane per 32-byte k-step --------------------------
    uint4 own[OW][C::KS];
    uint4 ownw[(TRANSH && OWN_ROW) ? C::KS : 1];
    float o_qn[OW], o_c[OW], o_wn[OW], o_tn[OW];          // own-side scalars
#pragma unroll
    for (int h = 0; h < OW; ++h) {
        const int oidx = oidx0 + 32 * h;
        const char *p = (const char *)a.own + (size_t)oidx * RB + g * 16;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) own[h][ks] = *(const uint4 *)(p + ks * 32);
        if constexpr (TRANSH && OWN_ROW) {
            const char *pw = (const char *)a.own2 + (size_t)oidx * RB + g * 16;
#pragma unroll
            for (int ks = 0; ks < C::KS; ++ks) ownw[ks] = *(const uint4 *)(pw + ks * 32);
        }
        o_qn[h] = 0.f; o_c[h] = 0.f; o_wn[h] = 1.f; o_tn[h] = 0.f;
        if constexpr (OWN_ROW) {
            KgeRowInfo ri = a.rowinfo[oidx];
            o_qn[h] = ri.qn; o_c[h] = ri.c; o_wn[h] = ri.wn;
        } else {
            o_tn[h] = a.tn[oidx];
        }
    }

    // ---- accumulators of the launch ------------------------------------------------------------
    kge_f32x16 acc2[OW][PHASE2 ? C::NBH : 1];
    kge_f32x16 acc2b[(PHASE2 && TRANSH && OWN_ROW) ? C::NBH : 1];
    if constexpr (PHASE2) {
#pragma unroll
        for (int b = 0; b < C::NBH; ++b) {
#pragma unroll
            for (int h = 0; h < OW; ++h)
                for (int i = 0; i < 16; ++i) acc2[h][b][i] = 0.f;
            if constexpr (TRANSH && OWN_ROW) for (int i = 0; i < 16; ++i) acc2b[b][i] = 0.f;
        }
    }
    float sum1[OW], sum2[OW], sum3[OW];                   // sums of the coefficients over the stream index
    float st_m[OW], st_l[OW], st_acc[OW];                 // FWD: running max (log2 domain) / sum / weighted loss
#pragma unroll
    for (int h = 0; h < OW; ++h) { sum1[h] = sum2[h] = sum3[h] = 0.f; st_m[h] = -INFINITY; st_l[h] = st_acc[h] = 0.f; }

    // ---- asynchronous staging of one stream tile --------------------------------------------------
    // X tile: instruction jj of this wave covers LDS bytes [(wave*X_IPW + jj) KB, +1 KB) of the tile; the
    // lane's 16 bytes are position (byte % RB)/16 of row byte/RB and must hold source chunk pos ^ (row & 7).
    int x_off[C::X_IPW];                                   // source byte offset inside the tile
#pragma unroll
    for (int jj = 0; jj < C::X_IPW; ++jj) {
        const int byte = (wave * C::X_IPW + jj) * 1024 + lane * 16;
        const int r = byte / RB, pos = (byte % RB) / 16;
        x_off[jj] = r * RB + ((pos ^ (r & 7)) * 16);
    }
    // Xt tile: rows of XT_ROWB bytes (dcol-major).  bf16: 64-byte rows, two rows per 128-byte line, chunk
    // slot ((row&1)*4 + c) ^ ((row>>1)&7) within the line; fp32: 128-byte rows, chunk c at c ^ (row & 7).
    int64_t xt_off[C::HAS_XT ? C::XT_IPW : 1];             // source byte offset relative to the tile's first column
    if constexpr (C::HAS_XT) {
#pragma unroll
        for (int jj = 0; jj < C::XT_IPW; ++jj) {
            const int byte = (wave * C::XT_IPW + jj) * 1024 + lane * 16;
            const int line = byte >> 7, slot = (byte >> 4) & 7;
            int row, c;
            if constexpr (BF16) { const int sslot = slot ^ (line & 7); row = 2 * line + (sslot >> 2); c = sslot & 3; }
            else { row = line; c = slot ^ (row & 7); }
            xt_off[jj] = (int64_t)row * a.strT_ld * C::ES + c * 16;
        }
    }
    auto issue = [&](int tile, int slot) {
        tile = tile < t1 ? tile : t1 - 1;                  // past the end: a harmless repeat keeps vmcnt uniform
        const uint32_t sbase = lds0 + (slot % C::NSTAGE) * C::STAGE_BYTES;
        const char *src = (const char *)a.str + (size_t)tile * C::ST * RB;
#pragma unroll
        for (int jj = 0; jj < C::X_IPW; ++jj)
            kge_async_copy16(src + x_off[jj], __builtin_amdgcn_readfirstlane(sbase + (wave * C::X_IPW + jj) * 1024));
        if constexpr (C::HAS_X2) {
            const char *src2 = (const char *)a.str2 + (size_t)tile * C::ST * RB;
#pragma unroll
            for (int jj = 0; jj < C::X_IPW; ++jj)
                kge_async_copy16(src2 + x_off[jj], __builtin_amdgcn_readfirstlane(sbase + C::X_BYTES + (wave * C::X_IPW + jj) * 1024));
        }
        if constexpr (C::HAS_XT) {
            const char *srct = (const char *)a.strT + (size_t)tile * C::ST * C::ES;
#pragma unroll
            for (int jj = 0; jj < C::XT_IPW; ++jj)
                kge_async_copy16(srct + xt_off[jj], __builtin_amdgcn_readfirstlane(sbase + C::X_BYTES * C::NX + (wave * C::XT_IPW + jj) * 1024));
            if constexpr (C::HAS_X2) {
                const char *srct2 = (const char *)a.strT2 + (size_t)tile * C::ST * C::ES;
#pragma unroll
                for (int jj = 0; jj < C::XT_IPW; ++jj)
                    kge_async_copy16(srct2 + xt_off[jj], __builtin_amdgcn_readfirstlane(sbase + C::X_BYTES * C::NX + C::XT_BYTES + (wave * C::XT_IPW + jj) * 1024));
            }
        }
        // side info of the tile's 32 stream rows, one private copy per wave
        const uint32_t sside = lds0 + C::NSTAGE * C::STAGE_BYTES + (slot % C::SIDE_SLOTS) * C::SIDE_SLOT;
        if constexpr (OWN_ROW) kge_async_copy4(a.tn + tile * C::ST + lr, __builtin_amdgcn_readfirstlane(sside + wave * 256));
        else kge_async_copy16(a.rowinfo + tile * C::ST + lr, __builtin_amdgcn_readfirstlane(sside + wave * 1024));
    };
    // fragment addresses inside a stage: chunk (2 ks + g) of row lr sits at position chunk ^ (lr & 7)
    int frag_off[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) frag_off[b] = lr * RB + 16 * (((2 * b) ^ (lr & 6)) | (g ^ (lr & 1)));

#pragma unroll
    for (int s2 = 0; s2 < C::NSTAGE - 1; ++s2) issue(t0 + s2, s2);
    // Pin the own operand as loaded before the loop.  Otherwise the compiler defers its waits for these
    // ordinary loads to their first uses inside the hot loop, and such a wait (which counts every memory
    // operation in flight) would also drain the asynchronous copies of the coming tiles on every iteration.
#pragma unroll
    for (int h = 0; h < OW; ++h) {
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            asm volatile("" : "+v"(own[h][ks].x), "+v"(own[h][ks].y), "+v"(own[h][ks].z), "+v"(own[h][ks].w));
            if constexpr (TRANSH && OWN_ROW)
                asm volatile("" : "+v"(ownw[ks].x), "+v"(ownw[ks].y), "+v"(ownw[ks].z), "+v"(ownw[ks].w));
        }
        asm volatile("" : "+v"(o_qn[h]), "+v"(o_c[h]), "+v"(o_wn[h]), "+v"(o_tn[h]));
    }

    // the own operand as bf16 pieces, two k-steps per entry (the fp32 fragments are not used again)
    constexpr bool X3 = C::X3;
    KgeP3 ownp[X3 ? OW : 1][X3 ? C::KS / 2 : 1], ownwp[(X3 && TRANSH && OWN_ROW) ? C::KS / 2 : 1];
    if constexpr (X3) {
#pragma unroll
        for (int h = 0; h < OW; ++h)
#pragma unroll
            for (int k2 = 0; k2 < C::KS / 2; ++k2) ownp[h][k2] = kge_split3(own[h][2 * k2], own[h][2 * k2 + 1]);
        if constexpr (TRANSH && OWN_ROW) {
#pragma unroll
            for (int k2 = 0; k2 < C::KS / 2; ++k2) ownwp[k2] = kge_split3(ownw[2 * k2], ownw[2 * k2 + 1]);
        }
    }

    // ---- state of the tile in work (set by the loops below, used by the pieces) -------------------
    int tile = t0;
    const char *base = lds, *side = side_ring;
    int sbase = 0;                                        // stream index of register i: sbase + 8*(i/4) + (i%4)
    bool tile_full = true;
    const float xscale = (LOSS == KGE_LOGSIGMOID ? a.adv_temp : 1.f) * KGE_LOG2E;
    auto set_tile = [&](int t) {
        tile = t;
        const int slot = t - t0;
        base = lds + (slot % C::NSTAGE) * C::STAGE_BYTES;
        side = side_ring + (slot % C::SIDE_SLOTS) * C::SIDE_SLOT + wave * (OWN_ROW ? 256 : 1024);
        sbase = t * C::ST + 4 * g;
        tile_full = t * C::ST + C::ST <= str_limit;
    };
    kge_f32x16 acc[OW], accw;                              // phase-1 accumulators: [stream, own]
    uint4 bf[OW][2], bf2[2];                               // bf16 B-operands of phase 2
    float coefs[(BF16 || X3) ? 1 : 16], coefs2[(BF16 || X3) ? 1 : 16];   // fp32 B-operands of phase 2 (OW == 1) ...
    KgeP3 coefp[2], coefp2[2];                             // ... or their bf16 pieces

    // ---- phase 1: acc[h][stream, own] = X_tile . own^t; a fragment read from the LDS feeds all own fragments
    constexpr bool HASW = TRANSH && !OWN_ROW;
    constexpr int G1 = HASW ? 2 : 4, NG1 = C::KS / G1;      // fragments per group, groups
    uint4 av[C::KS], aw[HASW ? C::KS : 1];
    auto ld1 = [&](const char *stage, int grp) {
#pragma unroll
        for (int k = 0; k < G1; ++k) {
            const int ks = grp * G1 + k;
            av[ks] = *(const uint4 *)(stage + frag_off[ks & 3] + 128 * (ks >> 2));
            if constexpr (HASW) aw[ks] = *(const uint4 *)(stage + C::X_BYTES + frag_off[ks & 3] + 128 * (ks >> 2));
        }
    };
    auto zero1 = [&]() {
#pragma unroll
        for (int h = 0; h < OW; ++h) for (int i = 0; i < 16; ++i) acc[h][i] = 0.f;
        for (int i = 0; i < 16; ++i) accw[i] = 0.f;
    };
    auto mma1 = [&](int grp) {
#pragma unroll
        for (int k = 0; k < G1; ++k) {
            const int ks = grp * G1 + k;
            if constexpr (!X3) {
#pragma unroll
                for (int h = 0; h < OW; ++h) acc[h] = kge_mma16<BF16>(acc[h], av[ks], own[h][ks]);
                if constexpr (TRANSH && OWN_ROW) accw = kge_mma16<BF16>(accw, av[ks], ownw[ks]);
                if constexpr (HASW) accw = kge_mma16<BF16>(accw, aw[ks], own[0][ks]);
            } else if ((k & 1) == 0) {                      // bf16 pieces: two k-steps at a time (G1 is even)
                const KgeP3 x = kge_split3(av[ks], av[ks + 1]);
#pragma unroll
                for (int h = 0; h < OW; ++h) acc[h] = kge_mma3(acc[h], x, ownp[h][ks >> 1]);
                if constexpr (TRANSH && OWN_ROW) accw = kge_mma3(accw, x, ownwp[ks >> 1]);
                if constexpr (HASW) accw = kge_mma3(accw, kge_split3(aw[ks], aw[ks + 1]), ownp[0][ks >> 1]);
            }
        }
    };
    // ---- phase 2: out^t[d, own] += Xt_tile[d, stream] . coef[stream, own] ---------------------------
    constexpr int G2 = BF16 ? (HASW ? 1 : 2) : 1;          // blocks per group
    constexpr int NG2 = PHASE2 ? C::NBH / G2 : 0;
    constexpr int F2 = BF16 ? 2 : 4;                       // 16-byte fragments per block
    uint4 av2[PHASE2 ? C::NBH : 1][F2], aw2[(PHASE2 && HASW) ? C::NBH : 1][F2];
    auto ld2 = [&](const char *stage, int grp) {
        const char *xt = stage + C::X_BYTES * C::NX;
#pragma unroll
        for (int bb = 0; bb < G2; ++bb) {
            const int blk = grp * G2 + bb;
            const int row = (dblk0 + blk) * 32 + lr;
#pragma unroll
            for (int f = 0; f < F2; ++f) {
                const char *p;
                if constexpr (BF16) {
                    // The transposed operand keeps, inside every group of 16 stream entries, the 8 entries of
                    // one lane half contiguous (the producer swaps bits 2 and 3 of the column), so the
                    // A-fragment of (block, f) is ONE 16-byte chunk: chunk 2 f + g of row dcol, at its slot.
                    const int sslot = (((row & 1) << 2) | (2 * f + g)) ^ ((row >> 1) & 7);
                    p = xt + (row >> 1) * 128 + sslot * 16;
                } else {
                    p = xt + row * 128 + ((2 * f + g) ^ (row & 7)) * 16;
                }
                av2[blk][f] = *(const uint4 *)p;
                if constexpr (HASW) aw2[blk][f] = *(const uint4 *)(p + C::XT_BYTES);
            }
        }
    };
    auto mma2 = [&](int grp) {
#pragma unroll
        for (int bb = 0; bb < G2; ++bb) {
            const int blk = grp * G2 + bb;
            if constexpr (BF16) {
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
#pragma unroll
                    for (int h = 0; h < OW; ++h) acc2[h][blk] = kge_mma16<true>(acc2[h][blk], av2[blk][s2], bf[h][s2]);
                    if constexpr (TRANSH && OWN_ROW) acc2b[blk] = kge_mma16<true>(acc2b[blk], av2[blk][s2], bf2[s2]);
                    if constexpr (HASW) acc2[0][blk] = kge_mma16<true>(acc2[0][blk], aw2[blk][s2], bf2[s2]);
                }
            } else if constexpr (!X3) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const kge_f32x4 fa = __builtin_bit_cast(kge_f32x4, av2[blk][j]);
                    kge_f32x4 fw;
                    if constexpr (HASW) fw = __builtin_bit_cast(kge_f32x4, aw2[blk][j]);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        acc2[0][blk] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[r], coefs[4 * j + r], acc2[0][blk], 0, 0, 0);
                        if constexpr (TRANSH && OWN_ROW)
                            acc2b[blk] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[r], coefs2[4 * j + r], acc2b[blk], 0, 0, 0);
                        if constexpr (HASW)
                            acc2[0][blk] = __builtin_amdgcn_mfma_f32_32x32x2f32(fw[r], coefs2[4 * j + r], acc2[0][blk], 0, 0, 0);
                    }
                }
            } else {
#pragma unroll
                for (int j2 = 0; j2 < 2; ++j2) {            // stream entries 16 j2 .. + 15: fragments 2 j2 and 2 j2 + 1
                    const KgeP3 x = kge_split3(av2[blk][2 * j2], av2[blk][2 * j2 + 1]);
                    acc2[0][blk] = kge_mma3(acc2[0][blk], x, coefp[j2]);
                    if constexpr (TRANSH && OWN_ROW) acc2b[blk] = kge_mma3(acc2b[blk], x, coefp2[j2]);
                    if constexpr (HASW)
                        acc2[0][blk] = kge_mma3(acc2[0][blk], kge_split3(aw2[blk][2 * j2], aw2[blk][2 * j2 + 1]), coefp2[j2]);
                }
            }
        }
    };
    // ---- epilogue: scores / loss weights / gradient coefficients of the tile, element by element ----
    // scores of own fragment h against the tile (SCORE mode stores them), 1/distance, w.t
    auto scores = [&](int h, float (&sv)[16], float (&dv)[16], float (&Av)[16]) {
        const int oidx = oidx0 + 32 * h;
#pragma unroll
        for (int i = 0; i < 16; ++i) { dv[i] = 0.f; Av[i] = 0.f; }
        if constexpr (KIND == KGE_KIND_MULT) {
#pragma unroll
            for (int i = 0; i < 16; ++i) sv[i] = acc[h][i];
        } else {
            // squared distance by the norm expansion |q|^2 + |t|^2 - 2 q.t (TransH: plus the terms of the
            // projection); entries where it cancels (below 1e-3 of the norms) are redone by direct
            // differences in a rarely taken branch
            float d2[16], thr[16];
            bool cancel = false;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int sl = 8 * (i >> 2) + 4 * g + (i & 3);
                float qn, cc, wn, tnv;
                if constexpr (OWN_ROW) { qn = o_qn[h]; cc = o_c[h]; wn = o_wn[h]; tnv = *(const float *)(side + sl * 4); }
                else { float4 ri = *(const float4 *)(side + sl * 16); qn = ri.x; cc = ri.y; wn = ri.w; tnv = o_tn[h]; }
                d2[i] = fmaf(-2.f, acc[h][i], qn + tnv);
                if constexpr (TRANSH) { const float A = accw[i]; Av[i] = A; d2[i] += A * (2.f * cc - A * (2.f - wn)); }
                thr[i] = 1e-3f * (qn + tnv);
                cancel = cancel || d2[i] < thr[i];
            }
            if (__any(cancel)) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    if (d2[i] < thr[i]) {
                        const int sidx = tile * C::ST + 8 * (i >> 2) + 4 * g + (i & 3);
                        const int b = OWN_ROW ? oidx : sidx, n = OWN_ROW ? sidx : oidx;
                        const char *qb = (const char *)(OWN_ROW ? a.own : a.str) + (size_t)b * RB;
                        const char *tb = (const char *)(OWN_ROW ? a.str : a.own) + (size_t)n * RB;
                        const char *wb = TRANSH ? (const char *)(OWN_ROW ? a.own2 : a.str2) + (size_t)b * RB : nullptr;
                        d2[i] = kge_direct_d2<BF16, TRANSH>(qb, tb, wb, C::DP);
                    }
                    asm volatile("" ::: "memory");          // keeps the branch from being turned into selects
                }
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float dd = fmaxf(d2[i], 0.f);
                const float inv = dd > 0.f ? __builtin_amdgcn_rsqf(dd) : 0.f;
                dv[i] = inv;
                sv[i] = -dd * inv;                          // -sqrt(d2)
            }
        }
        if constexpr (MODE == KGE_MODE_SCORE) {
            if (oidx < a.N) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int b = sbase + 8 * (i >> 2) + (i & 3);
                    if (b < a.B) a.S_out[(size_t)b * a.N + oidx] = sv[i];
                }
            }
        }
    };
    // FWD: exponents of the softmax weights of own fragment h relative to its reference st_m (log2
    // domain; entries past the end of the stream operand get -inf: only the last tile has any, the
    // branch is wave-uniform), and their maximum over the tile.  Lanes l and l^32 hold the two halves
    // of the same own row and feed ONE contraction in phase 2, so they share the maximum.
    auto exponents = [&](int h, const float (&sv)[16], float (&x2)[16]) -> float {
        const float m_neg = st_m[h] > -INFINITY ? -st_m[h] : 0.f;
        float tm = -INFINITY;
#pragma unroll
        for (int i = 0; i < 16; ++i) x2[i] = fmaf(sv[i], xscale, m_neg);
        if (!tile_full) {
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (sbase + 8 * (i >> 2) + (i & 3) >= str_limit) x2[i] = -INFINITY;
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) tm = fmaxf(tm, x2[i]);
        return fmaxf(tm, __shfl_xor(tm, 32));
    };
    // the coefficients of phase 2 for own fragment h, packed as its B-operand
    auto weights = [&](int h, const float (&sv)[16], const float (&dv)[16], const float (&Av)[16], const float (&x2)[16]) {
        float coef[16], coef2[16];
        if constexpr (MODE == KGE_MODE_FWD) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float e = kge_exp2(x2[i]);                             // masked entries: exp2(-inf) = 0
                st_l[h] += e;
                float u = e;
                if constexpr (LOSS == KGE_LOGSIGMOID) {
                    // weight * sigma(gamma + s) for the gradient, weight * softplus(gamma + s) for the loss
                    const float y = a.gamma + sv[i];
                    const float t = kge_exp2(-fabsf(y) * KGE_LOG2E);
                    const float rcp = __builtin_amdgcn_rcpf(1.f + t);
                    const float sig = y >= 0.f ? rcp : t * rcp;
                    const float softplus = fmaxf(y, 0.f) + KGE_LN2 * kge_log2(1.f + t);
                    if (e > 0.f) st_acc[h] = fmaf(e, softplus, st_acc[h]);
                    u = e * sig;
                }
                const float c1 = KIND == KGE_KIND_DIST ? u * dv[i] : u;
                coef[i] = c1;
                if constexpr (KIND == KGE_KIND_DIST) sum1[h] += c1;  // only the distance scorers' chain rule needs it
                if constexpr (TRANSH) { coef2[i] = c1 * Av[i]; sum2[h] += coef2[i]; sum3[h] += coef2[i] * Av[i]; }
            }
        }
        if constexpr (MODE == KGE_MODE_GRADT) {
            // gradient coefficient of every (query, negative) pair from the finished row constants
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int sl = 8 * (i >> 2) + 4 * g + (i & 3);
                const float K2 = *(const float *)(side + sl * 16 + 8);       // -inf for padded queries
                float u = kge_exp2(fmaf(sv[i], xscale, K2));
                if constexpr (LOSS == KGE_LOGSIGMOID) {
                    const float y = a.gamma + sv[i];
                    const float t = kge_exp2(-fabsf(y) * KGE_LOG2E);
                    const float rcp = __builtin_amdgcn_rcpf(1.f + t);
                    u *= y >= 0.f ? rcp : t * rcp;
                }
                const float c1 = KIND == KGE_KIND_DIST ? u * dv[i] : u;
                coef[i] = c1;
                if constexpr (KIND == KGE_KIND_DIST) sum1[h] += c1;
                if constexpr (TRANSH) coef2[i] = c1 * Av[i];
            }
        }
        if constexpr (PHASE2) {
            if constexpr (BF16) {
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    bf[h][s2] = make_uint4(kge_pack_bf16x2(coef[8 * s2 + 0], coef[8 * s2 + 1]),
                                           kge_pack_bf16x2(coef[8 * s2 + 2], coef[8 * s2 + 3]),
                                           kge_pack_bf16x2(coef[8 * s2 + 4], coef[8 * s2 + 5]),
                                           kge_pack_bf16x2(coef[8 * s2 + 6], coef[8 * s2 + 7]));
                    if constexpr (TRANSH)
                        bf2[s2] = make_uint4(kge_pack_bf16x2(coef2[8 * s2 + 0], coef2[8 * s2 + 1]),
                                             kge_pack_bf16x2(coef2[8 * s2 + 2], coef2[8 * s2 + 3]),
                                             kge_pack_bf16x2(coef2[8 * s2 + 4], coef2[8 * s2 + 5]),
                                             kge_pack_bf16x2(coef2[8 * s2 + 6], coef2[8 * s2 + 7]));
                }
            } else if constexpr (!X3) {
#pragma unroll
                for (int i = 0; i < 16; ++i) { coefs[i] = coef[i]; if constexpr (TRANSH) coefs2[i] = coef2[i]; }
            } else {
                auto four = [](const float *c) { return make_uint4(__float_as_uint(c[0]), __float_as_uint(c[1]), __float_as_uint(c[2]), __float_as_uint(c[3])); };
#pragma unroll
                for (int j2 = 0; j2 < 2; ++j2) {
                    coefp[j2] = kge_split3(four(coef + 8 * j2), four(coef + 8 * j2 + 4));
                    if constexpr (TRANSH) coefp2[j2] = kge_split3(four(coef2 + 8 * j2), four(coef2 + 8 * j2 + 4));
                }
            }
        }
    };
    // The FWD pass keeps all weights relative to a per-row reference exponent st_m that is only
    // raised (and what the row has accumulated rescaled) when a tile's maximum exceeds it by more than
    // KGE_TAU: weights stay below 2^KGE_TAU, and the rescaling is a rarely taken branch of the loop.
    auto epilogue = [&]() {
#pragma unroll
        for (int h = 0; h < OW; ++h) {
            float sv[16], dv[16], Av[16], x2[16];
            scores(h, sv, dv, Av);
            if constexpr (MODE == KGE_MODE_FWD) {
                const float tm = exponents(h, sv, x2);
                const bool have = st_m[h] > -INFINITY;
                const bool trip = tm > (have ? KGE_TAU : -INFINITY);   // without a reference, any finite entry sets one
                if (__any(trip)) {
                    // the rows that tripped take the tile's maximum as their reference
                    const float m_new = trip ? (have ? tm + st_m[h] : tm) : st_m[h];
                    const float shift = trip ? -tm : 0.f;              // exponents relative to the new reference
                    const float r = trip ? (have ? kge_exp2(-tm) : 0.f) : 1.f;   // nothing accumulated yet without one
                    st_m[h] = m_new;
                    st_l[h] *= r; st_acc[h] *= r; sum1[h] *= r; sum2[h] *= r; sum3[h] *= r;
#pragma unroll
                    for (int b = 0; b < C::NBH; ++b) {
                        // one block at a time: the accumulators live in AGPRs and pass through VGPRs here; the
                        // empty statements keep this rarely executed code from being turned into selects
                        for (int i = 0; i < 16; ++i) acc2[h][b][i] *= r;
                        asm volatile("" ::: "memory");
                        if constexpr (TRANSH) { for (int i = 0; i < 16; ++i) acc2b[b][i] *= r; asm volatile("" ::: "memory"); }
                    }
#pragma unroll
                    for (int i = 0; i < 16; ++i) x2[i] += shift;       // masked entries stay at -inf
                }
            }
            weights(h, sv, dv, Av, x2);
        }
    };

    for (int t = t0; t < t1; ++t) {
        // tile t has landed when at most NSTAGE-2 younger tiles are still in flight; after the
        // barrier every wave has finished tile t-1, whose stage receives tile t + NSTAGE - 1
        kge_wait_vmcnt<(C::NSTAGE - 2) * C::LPW>();
        __syncthreads();
        issue(t + C::NSTAGE - 1, t - t0 + C::NSTAGE - 1);
        set_tile(t);
        // The fragments of a chunk are requested before its first MFMA (the whole phase where the registers
        // allow it).  Deeper software pipelining of the reads, enforced with scheduling barriers, was
        // measured and did not pay: inside a chunk the order is left to the compiler.
        zero1();
        constexpr int CH1 = OW > 1 ? 1 : (NG1 > 4 ? 4 : NG1);   // groups per chunk: at most 64 (16) registers in flight
#pragma unroll
        for (int c0 = 0; c0 < NG1; c0 += CH1) {
#pragma unroll
            for (int gq = c0; gq < c0 + CH1; ++gq) ld1(base, gq);
#pragma unroll
            for (int gq = c0; gq < c0 + CH1; ++gq) mma1(gq);
        }
        epilogue();
        if constexpr (PHASE2) {
            constexpr int CH2 = OW > 1 ? 1 : NG2;
#pragma unroll
            for (int c0 = 0; c0 < NG2; c0 += CH2) {
#pragma unroll
                for (int gq = c0; gq < c0 + CH2; ++gq) ld2(base, gq);
#pragma unroll
                for (int gq = c0; gq < c0 + CH2; ++gq) mma2(gq);
            }
        }
    }
    kge_wait_vmcnt<0>();                                  // no copy may be in flight when the LDS is released

    // ---- write-out ---------------------------------------------------------------------------------
    if constexpr (PHASE2) {
#pragma unroll
        for (int h = 0; h < OW; ++h) {
            const int oidx = oidx0 + 32 * h;
            // lanes l and l^32 hold the same own row over disjoint stream entries (same running max):
            // add their scalars.  The phase-2 accumulators already contain both halves.
            if constexpr (MODE == KGE_MODE_FWD) { st_l[h] += __shfl_xor(st_l[h], 32); st_acc[h] += __shfl_xor(st_acc[h], 32); }
            sum1[h] += __shfl_xor(sum1[h], 32); sum2[h] += __shfl_xor(sum2[h], 32); sum3[h] += __shfl_xor(sum3[h], 32);
            if (g == 0 && blockIdx.y == 0) {
                a.sum_part[(size_t)split * a.own_pad + oidx] = make_float4(sum1[h], sum2[h], sum3[h], 0.f);
                if constexpr (MODE == KGE_MODE_FWD)
                    a.stat_part[(size_t)split * a.own_pad + oidx] = make_float4(st_m[h], st_l[h], st_acc[h], 0.f);
            }
#pragma unroll
            for (int blk = 0; blk < C::NBH; ++blk) {
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const int dcol = (dblk0 + blk) * 32 + 8 * q4 + 4 * g;
                    const size_t o = ((size_t)split * a.own_pad + oidx) * C::DP + dcol;
                    *(float4 *)(a.acc_part + o) = make_float4(acc2[h][blk][4 * q4], acc2[h][blk][4 * q4 + 1], acc2[h][blk][4 * q4 + 2], acc2[h][blk][4 * q4 + 3]);
                    if constexpr (TRANSH && OWN_ROW)
                        *(float4 *)(a.acc_part2 + o) = make_float4(acc2b[blk][4 * q4], acc2b[blk][4 * q4 + 1], acc2b[blk][4 * q4 + 2], acc2b[blk][4 * q4 + 3]);
                }
            }
        }
    }
}

template <bool BF16, int RB, int MODE, bool TRANSH, int KIND, int LOSS, int DSPLIT>
int kge_block_launch(const KgeBlockArgs &a, int own_tiles, int nsplit, hipStream_t st) {
    using C = KgeBlockCfg<BF16, RB, MODE, TRANSH, KIND, DSPLIT>;
    auto kern = kge_block_kernel<BF16, RB, MODE, TRANSH, KIND, LOSS, DSPLIT>;
    static KgeLdsLimit lds_limit;
    if (lds_limit.set((const void *)kern, C::LDS_BYTES) != KGE_OK) return KGE_E_HIP;
    if ((int64_t)own_tiles * C::OWN_TILE != a.own_pad) return KGE_E_INVALID_ARG;   // the caller's geometry must match
    KgeBlockArgs b = a;
    b.own_tiles = own_tiles; b.nsplit = nsplit;
    int groups;                                            // workgroups per XCD
    if (nsplit >= 8) { b.xcd_per = 1; groups = own_tiles * ((nsplit + 7) / 8); }
    else {
        int s2 = 1;
        while (s2 < nsplit) s2 <<= 1;
        b.xcd_per = 8 / s2;
        groups = (own_tiles + b.xcd_per - 1) / b.xcd_per;
    }
    dim3 grid(8 * groups, MODE != KGE_MODE_SCORE ? DSPLIT : 1);
    hipLaunchKernelGGL(kern, grid, dim3(256), C::LDS_BYTES, st, b);
    return kge_launch_status();
}
