// extern "C" entry points: argument validation, workspace carving, kernel sequencing.
#include "prep_kernels.h"
#include <math.h>

int kge_run_sparse_adam(float *param, void *shadow, float *m, float *v, int64_t n_rows, int dim, int64_t ld,
                        const int32_t *idx, const float *grads, int64_t M, const kge_adam_cfg_t &cfg, void *ws,
                        size_t ws_bytes, hipStream_t st);
size_t kge_sparse_adam_ws(int64_t M, int dim);
int kge_static_scratch(void **ptr, size_t *bytes);
size_t kge_static_scratch_bytes();
int kge_run_sparse_adam_plan(int64_t n_rows, const int32_t *idx, int64_t M, void *ws, hipStream_t st);
int kge_run_sparse_adam_apply(float *param, void *shadow, float *m, float *v, int64_t n_rows, int dim, int64_t ld,
                              const float *grads, int64_t M, const kge_adam_cfg_t &cfg, void *ws, hipStream_t st);
int kge_run_sparse_adam_apply_tables(const kge_adam_table_t *tb, int n, const kge_adam_cfg_t &cfg, hipStream_t st);
int kge_run_sparse_adam_plan_tables(const kge_adam_plan_t *pl, int n, hipStream_t st, const KgeRowFinishQArgs *rf = nullptr);
int kge_run_topk(const kge_model_t &model, const int32_t *h, const int32_t *r, int64_t Q, int64_t lo, int64_t hi,
                 int K, int32_t *out_idx, float *out_score, const int32_t *true_t, int64_t *out_rank, void *ws,
                 size_t ws_bytes, hipStream_t st);
size_t kge_topk_ws(const kge_model_t &model, int64_t Q, int64_t ncand, int K);
int kge_launch_score_h2(int kind, int dp, const void *Qp, const void *Tp, const float *t_inv, const float *Q32, const float *T32,
                        const float *W32, const KgeRowInfo *rowinfo, const float *tn, int B, int N, int Bp, int Np, float *S_out,
                        hipStream_t st);
int kge_run_partition(const int32_t *h, const int32_t *t, int64_t n, int64_t part_size, int D, int64_t *offsets,
                      int64_t *order, void *ws, size_t ws_bytes, hipStream_t st);
size_t kge_partition_ws(int64_t n, int D);
size_t kge_sampler_ws(int64_t n);
int kge_validate_encoder(const kge_encoder_t *e);
size_t kge_encode_ws(const kge_encoder_t &e, int64_t B, int64_t N, bool bwd);
int kge_run_encode(const kge_encoder_t &e, const int32_t *h, const int32_t *t, int64_t B, const int32_t *neg, int64_t N,
                   uint64_t seed, uint64_t step, void *e_out, float *proj_out, float *reg_out, void *ws, hipStream_t st);
int kge_run_encode_bwd(const kge_encoder_t &e, const int32_t *h, const int32_t *t, int64_t B, const int32_t *neg, int64_t N,
                       uint64_t seed, uint64_t step, const float *proj, const float *de, float *g_es, float *g_mh, float *g_mt,
                       void *ws, hipStream_t st);
int kge_run_sampler_build(const int32_t *h, const int32_t *r, const int32_t *t, int64_t n, int64_t part_size, int D,
                          int64_t n_rel, int64_t *order, int64_t *rel_offsets, uint64_t *cdf, void *ws, hipStream_t st);
int kge_run_sample_triples(uint64_t seed, uint64_t step, uint32_t tag, int64_t bucket_lo, int64_t draws, int64_t per_bucket,
                           int64_t n_rel, const int64_t *rel_offsets, const uint64_t *cdf, const int64_t *order,
                           const int32_t *h, const int32_t *r, const int32_t *t, int64_t *out_pos, int32_t *out_h,
                           int32_t *out_r, int32_t *out_t, hipStream_t st);
int kge_run_negatives_sharded(uint64_t seed, uint64_t step, uint32_t tag, int64_t part_size, int64_t n_ent, int64_t per_shard,
                              int64_t n, int32_t *out, hipStream_t st);

int kge_run_ensemble(const int32_t *lists, int M, int64_t Q, int K, double p, int K_out, int32_t *out_idx, float *out_score,
                     hipStream_t st);

namespace {

struct Geometry {
    bool bf16, transh, l1;              // l1: the vector-pipe kernels with the score block in memory - distance scorers with the
                                        // 1-norm, and in training calls TransH rows over 512 bytes (2-norm; the matrix-core
                                        // kernels have no registers for two operands of that width)
    int pn;                             // ... the norm they compute
    int es, rb, dp, kind;
    int B, N, Bp, Np;
    int own_tiles_b, own_tiles_n, own_tiles_s;   // own tiles of the FWD pass (queries), the GRADT and the SCORE pass (negatives)
    int str_tiles_b, str_tiles_n;       // 32-row tiles
    int nsplit_q, tps_q;                // row-owner launches: splits over the negatives
    int nsplit_t, tps_t;                // GRADT launches: splits over the queries
    int nsplit_s, tps_s;                // SCORE launches: splits over the queries
    int dsplit_q, dsplit_t;
};

constexpr int TARGET_WGS = 256;         // one workgroup per compute unit

int validate_model(const kge_model_t *m) {
    if (!m) return KGE_E_INVALID_ARG;
    if (m->scorer < KGE_TRANSE || m->scorer > KGE_COMPLEX) return KGE_E_INVALID_ARG;
    if (m->dtype != KGE_F32 && m->dtype != KGE_BF16) return KGE_E_INVALID_ARG;
    const int es = m->dtype == KGE_BF16 ? 2 : 4;
    if (m->dim <= 0 || m->dim % (32 / es) != 0 || m->dim * es > 1024) return KGE_E_INVALID_ARG;
    const bool dist = m->scorer == KGE_TRANSE || m->scorer == KGE_TRANSH || m->scorer == KGE_ROTATE;
    if (dist && m->p_norm != 1 && m->p_norm != 2) return KGE_E_INVALID_ARG;
    const int k = m->scorer == KGE_ROTATE ? m->dim / 2 : m->dim;
    if (m->rel_dim != k) return KGE_E_INVALID_ARG;
    if (m->n_ent <= 0 || m->n_rel <= 0 || m->n_ent >= (1ll << 31) || m->n_rel >= (1ll << 31)) return KGE_E_INVALID_ARG;
    if (!m->ent || !m->rel || m->ent_ld < m->dim || m->rel_ld < k) return KGE_E_INVALID_ARG;
    if (m->scorer == KGE_TRANSH && (!m->relw || m->relw_ld < m->dim)) return KGE_E_INVALID_ARG;
    return KGE_OK;
}

Geometry make_geometry(const kge_model_t &m, int64_t B, int64_t N, bool train = false) {
    Geometry g{};
    g.bf16 = m.dtype == KGE_BF16;
    g.transh = m.scorer == KGE_TRANSH;
    g.es = g.bf16 ? 2 : 4;
    g.rb = m.dim * g.es <= 512 ? 512 : 1024;
    g.dp = g.rb / g.es;
    g.kind = (m.scorer == KGE_DISTMULT || m.scorer == KGE_COMPLEX) ? KGE_KIND_MULT : KGE_KIND_DIST;
    g.l1 = g.kind == KGE_KIND_DIST && (m.p_norm == 1 || (train && g.transh && g.rb > 512));
    g.pn = g.kind == KGE_KIND_DIST ? m.p_norm : 2;
    g.B = (int)B; g.N = (int)N;
    g.Bp = (int)kge_round_up(B, KGE_PAD); g.Np = (int)kge_round_up(N, KGE_PAD);
    g.own_tiles_b = g.Bp / (128 * kge_block_ow(g.bf16, g.rb, g.transh, KGE_MODE_FWD, g.kind));
    g.dsplit_q = (g.bf16 && (g.rb == 1024 || g.transh)) ? 2 : 1;
    g.dsplit_t = (g.bf16 && g.rb == 1024) ? 2 : 1;
    // (the two-role kernel of the pass over the negatives keeps one own fragment per wave)
    g.own_tiles_n = g.Np / (128 * (kge_gradt_pp_applies(g.bf16, g.rb, g.transh, g.dsplit_t) ? 1 : kge_block_ow(g.bf16, g.rb, g.transh, KGE_MODE_GRADT, g.kind)));
    g.own_tiles_s = g.Np / (128 * kge_block_ow(g.bf16, g.rb, g.transh, KGE_MODE_SCORE, g.kind));
    g.str_tiles_b = g.Bp / KGE_STREAM_TILE; g.str_tiles_n = g.Np / KGE_STREAM_TILE;
    // gran: stream tiles (of 32 rows) that a kernel consumes at a time; a split holds a multiple of it
    auto split = [](int own_tiles, int str_tiles, int &nsplit, int &tps, int occ, int gran) {
        if (own_tiles == 0 || str_tiles == 0) { nsplit = 0; tps = 0; return; }
        int want = (TARGET_WGS * occ + own_tiles - 1) / own_tiles;
        if (want > str_tiles) want = str_tiles;
        if (want < 1) want = 1;
        tps = ((str_tiles + want - 1) / want + gran - 1) / gran * gran;
        nsplit = (str_tiles + tps - 1) / tps;
    };
    const int gran = kge_sym_applies(g.bf16, g.rb, g.transh, g.dsplit_q) ? 2 : 1;
    // (where the forward pass keeps its weights for the pass over the negatives, a forward split holds whole own tiles of
    // that pass: 128 negatives = four stream tiles)
    split(g.own_tiles_b, g.str_tiles_n, g.nsplit_q, g.tps_q, kge_block_occ(g.bf16, g.rb, g.transh, KGE_MODE_FWD),
          kge_gradp_applies(g.bf16, g.rb, g.transh, g.dsplit_q, g.kind) ? 4 : gran);
    split(g.own_tiles_n, g.str_tiles_b, g.nsplit_t, g.tps_t, kge_block_occ(g.bf16, g.rb, g.transh, KGE_MODE_GRADT), gran);
    split(g.own_tiles_s, g.str_tiles_b, g.nsplit_s, g.tps_s, kge_block_occ(g.bf16, g.rb, g.transh, KGE_MODE_SCORE), 1);
    g.dsplit_q = (g.bf16 && (g.rb == 1024 || g.transh)) ? 2 : 1;
    g.dsplit_t = (g.bf16 && g.rb == 1024) ? 2 : 1;
    if (g.l1) {
        g.nsplit_q = kge_l1_nsplit(g.Bp, g.Np, g.dp, g.transh);
        g.nsplit_t = kge_l1_nsplit(g.Np, g.Bp, g.dp, g.transh);
    }
    return g;
}

// fp32 score blocks go through two fp16 planes on the 16-bit matrix pipe (block_f32h2_score.hip); other row sizes, and
// the comparison that kge_debug_select(KGE_DEBUG_SCORE_F32_MFMA, 1) asks for, use the fp32 matrix instructions
bool score_h2_applies(const Geometry &g) {
    return !kge_knob(KGE_KNOB_SCORE_F32_MFMA) && !g.bf16 && !g.l1 && (g.dp == 128 || g.dp == 256) && g.N > 0;
}

// bump allocator over the caller's workspace (256-byte granules); with base == nullptr it only sizes
struct Carver {
    char *base; size_t off = 0;
    explicit Carver(void *p) : base((char *)p) {}
    template <typename T> T *take(size_t count) {
        size_t bytes = (count * sizeof(T) + 255) / 256 * 256;
        T *p = base ? (T *)(base + off) : nullptr;
        off += bytes;
        return p;
    }
};

struct Buffers {
    void *Q, *W, *Q2, *T, *Qt, *Wt, *Tt;
    KgeRowInfo *rowinfo; float *tn, *pos, *lossb, *gpos;
    float4 *stat_part; float *accq, *accq2; float4 *sumq; float *acct; float4 *sumt;
    float *regv;                       // L3 norms of the gathered slots: [Bp heads][Bp tails][Np negatives]
    float *S, *Q32;                    // 1-norm scorers: the score block [Bp][Np], the queries unrounded [Bp][dp]
    float *W32, *A, *P;                // ... TransH: the unit normals unrounded, w^ . t and sign(x) . w^ per pair [Bp][Np]
    void *Qp2, *Tp2;                   // score-only calls on fp32 tables: two fp16 planes of the scaled Q (TransH: and of W) and T
    float *t_inv;                      // ... 1 / scale of the rows of T
    void *pstore, *Qs;                 // sampled softmax on the kernels of block_sym.hip / block_gradp.hip: the weights of the
                                       // forward pass [Bp x Np bf16, in records], the queries scaled per forward split [nsplit_q][Bp][dp]
    float *nbias;                      // training calls: 0 for each of the N negatives, -inf for the padding rows behind them
};

size_t carve(const Geometry &g, bool bwd, void *ws, Buffers &b) {
    Carver c(ws);
    const size_t es = g.es, rowsB = (size_t)g.Bp * g.dp, rowsN = (size_t)g.Np * g.dp;
    b.Q = c.take<char>(rowsB * es);
    b.W = g.transh ? c.take<char>(rowsB * es) : nullptr;
    b.T = c.take<char>(rowsN * es);
    b.rowinfo = c.take<KgeRowInfo>(g.Bp);
    b.tn = c.take<float>(g.Np);
    b.pos = c.take<float>(g.Bp);
    b.Q32 = g.l1 ? c.take<float>(rowsB) : nullptr;
    b.W32 = g.l1 && g.transh ? c.take<float>(rowsB) : nullptr;
    b.A = b.P = nullptr;
    b.Qp2 = b.Tp2 = nullptr; b.t_inv = nullptr;
    if (!bwd && score_h2_applies(g)) {
        b.Qp2 = c.take<char>((g.transh ? 4 : 2) * rowsB * 2); b.Tp2 = c.take<char>(2 * rowsN * 2); b.t_inv = c.take<float>(g.Np);
    }
    b.Q2 = nullptr; b.Qt = b.Wt = b.Tt = nullptr; b.lossb = b.gpos = nullptr; b.stat_part = nullptr;
    b.accq = b.accq2 = b.acct = nullptr; b.sumq = b.sumt = nullptr; b.regv = nullptr; b.S = nullptr; b.nbias = nullptr;
    if (bwd) {
        b.Q2 = g.transh && !g.l1 ? c.take<char>(rowsB * es) : nullptr;
        if (!g.l1) {
            b.Qt = c.take<char>(rowsB * es);
            b.Wt = g.transh ? c.take<char>(rowsB * es) : nullptr;
            b.Tt = c.take<char>(rowsN * es);
        } else {
            b.S = c.take<float>((size_t)g.Bp * g.Np);
            if (g.transh) { b.A = c.take<float>((size_t)g.Bp * g.Np); b.P = c.take<float>((size_t)g.Bp * g.Np); }
        }
        b.lossb = c.take<float>(g.Bp);
        b.gpos = c.take<float>(g.Bp);
        b.stat_part = c.take<float4>((size_t)g.nsplit_q * g.Bp);
        b.accq = c.take<float>((size_t)g.nsplit_q * rowsB);
        b.accq2 = g.transh ? c.take<float>((size_t)g.nsplit_q * rowsB) : nullptr;
        b.sumq = c.take<float4>((size_t)g.nsplit_q * g.Bp);
        b.acct = c.take<float>((size_t)g.nsplit_t * rowsN);
        b.sumt = c.take<float4>((size_t)g.nsplit_t * g.Np);
        b.regv = c.take<float>((size_t)2 * g.Bp + g.Np);
        b.nbias = c.take<float>(g.Np);
        b.pstore = b.Qs = nullptr;
        if (g.B > 0 && g.N > 0 && !g.l1 && kge_gradp_applies(g.bf16, g.rb, g.transh, g.dsplit_q, g.kind)) {
            b.pstore = c.take<char>((size_t)g.own_tiles_b * g.nsplit_q * (g.tps_q / 2) * 16384);
            b.Qs = c.take<char>((size_t)g.nsplit_q * rowsB * es);
        }
    }
    return c.off + 256;
}

KgeModelDev dev_model(const kge_model_t &m) {
    KgeModelDev d;
    d.scorer = m.scorer; d.bf16 = m.dtype == KGE_BF16; d.dim = m.dim; d.rel_dim = m.rel_dim;
    d.p1 = (m.scorer == KGE_TRANSE || m.scorer == KGE_TRANSH || m.scorer == KGE_ROTATE) && m.p_norm == 1;
    d.vec = d.p1;
    d.ent = m.ent; d.rel = m.rel; d.relw = m.relw;
    d.ent_ld = m.ent_ld; d.rel_ld = m.rel_ld; d.relw_ld = m.relw_ld;
    return d;
}

int launch_block(const Geometry &g, int mode, int loss, const KgeBlockArgs &a, int own_tiles, int nsplit, int dsplit,
                 hipStream_t st) {
    return kge_launch_block(g.bf16, g.rb, mode, g.transh, g.kind, loss, dsplit, a, own_tiles, nsplit, st);
}

// the update reads and writes four columns at a time: 16-byte aligned fp32 rows (ld % 4 == 0 is checked by the callers),
// 8-byte aligned bf16 shadow rows
bool adam_rows_aligned(const float *param_f32, const void *param_bf16, const float *m, const float *v, const float *grads) {
    return (((uintptr_t)param_f32 | (uintptr_t)m | (uintptr_t)v | (uintptr_t)grads) & 15) == 0 && ((uintptr_t)param_bf16 & 7) == 0;
}

void *align_ws(void *ws, size_t &bytes) {
    uintptr_t p = (uintptr_t)ws, q = (p + 255) & ~(uintptr_t)255;
    bytes = bytes >= (q - p) ? bytes - (q - p) : 0;
    return (void *)q;
}

}  // namespace

extern "C" {

const char *kge_status_string(int status) {
    switch (status) {
    case KGE_OK: return "ok";
    case KGE_E_INVALID_ARG: return "invalid argument";
    case KGE_E_UNSUPPORTED: return "unsupported configuration";
    case KGE_E_WORKSPACE_TOO_SMALL: return "workspace too small";
    case KGE_E_HIP: return "HIP runtime error";
    case KGE_E_STATIC_SCRATCH_TOO_SMALL: return "request exceeds the library's static scratch buffer";
    default: return "unknown status";
    }
}

size_t kge_workspace_bytes(int op, const kge_model_t *model, int64_t B, int64_t N, int64_t K) {
    if (B < 0 || N < 0) return 0;
    switch (op) {
    case KGE_OP_SCORE:
    case KGE_OP_LOSS_BWD: {
        if (validate_model(model) != KGE_OK || B >= (1ll << 30) || N >= (1ll << 30)) return 0;
        Geometry g = make_geometry(*model, B, N, op == KGE_OP_LOSS_BWD);
        Buffers b;
        return carve(g, op == KGE_OP_LOSS_BWD, nullptr, b);
    }
    case KGE_OP_SPARSE_ADAM: return N <= 4096 ? kge_sparse_adam_ws(B, (int)N) : 0;
    case KGE_OP_TOPK:
        if (validate_model(model) != KGE_OK || K < 1 || K > 256) return 0;
        return kge_topk_ws(*model, B, N, (int)K);
    case KGE_OP_PARTITION: return (N >= 1 && N <= 64) ? kge_partition_ws(B, (int)N) : 0;
    case KGE_OP_SAMPLER_BUILD: return (N >= 1 && N <= 64) ? kge_sampler_ws(B) : 0;
    default: return 0;
    }
}

int kge_sample_negatives(uint64_t seed, uint64_t step, uint32_t stream_tag, int64_t lo, int64_t hi, int64_t n,
                         int32_t *out_idx, void *hip_stream) {
    if (n < 0 || hi <= lo || lo < 0 || hi > (1ll << 31) || step >= (1ull << 32)) return KGE_E_INVALID_ARG;
    if (n == 0) return KGE_OK;
    if (!out_idx) return KGE_E_INVALID_ARG;
    return kge_run_negatives(seed, step, nullptr, stream_tag, lo, hi, n, out_idx, (hipStream_t)hip_stream);
}

int kge_sample_negatives_dev(uint64_t seed, const uint64_t *step_counter, uint64_t step_offset, uint32_t stream_tag, int64_t lo,
                             int64_t hi, int64_t n, int32_t *out_idx, void *hip_stream) {
    if (!step_counter || n < 0 || hi <= lo || lo < 0 || hi > (1ll << 31) || step_offset >= (1ull << 32)) return KGE_E_INVALID_ARG;
    if (n == 0) return KGE_OK;
    if (!out_idx) return KGE_E_INVALID_ARG;
    return kge_run_negatives(seed, step_offset, step_counter, stream_tag, lo, hi, n, out_idx, (hipStream_t)hip_stream);
}

int kge_step_counter_add(uint64_t *step_counter, uint64_t inc, void *hip_stream) {
    if (!step_counter) return KGE_E_INVALID_ARG;
    return kge_run_step_counter_add(step_counter, inc, (hipStream_t)hip_stream);
}

size_t kge_encode_workspace_bytes(int op, const kge_encoder_t *enc, int64_t B, int64_t N) {
    if ((op != KGE_OP_ENCODE && op != KGE_OP_ENCODE_BWD) || kge_validate_encoder(enc) != KGE_OK) return 0;
    if (B < 0 || N < 0 || 2 * B + N >= (1ll << 30)) return 0;
    return kge_encode_ws(*enc, B, N, op == KGE_OP_ENCODE_BWD);
}

int kge_encode(const kge_encoder_t *enc, const int32_t *h, const int32_t *t, int64_t B, const int32_t *neg, int64_t N,
               uint64_t seed, uint64_t step, void *e_out, float *proj_out, float *reg_out, void *ws, size_t ws_bytes,
               void *hip_stream) {
    int rc = kge_validate_encoder(enc);
    if (rc != KGE_OK) return rc;
    if (B < 0 || N < 0 || 2 * B + N >= (1ll << 30) || step >= (1ull << 32)) return KGE_E_INVALID_ARG;
    if (B > 0 && (!h || !t)) return KGE_E_INVALID_ARG;
    if (N > 0 && !neg) return KGE_E_INVALID_ARG;
    if (2 * B + N > 0 && (!e_out || !proj_out)) return KGE_E_INVALID_ARG;
    if (!ws) return KGE_E_WORKSPACE_TOO_SMALL;
    ws = align_ws(ws, ws_bytes);
    if (kge_encode_ws(*enc, B, N, false) - 256 > ws_bytes) return KGE_E_WORKSPACE_TOO_SMALL;
    return kge_run_encode(*enc, h, t, B, neg, N, seed, step, e_out, proj_out, reg_out, ws, (hipStream_t)hip_stream);
}

int kge_encode_bwd(const kge_encoder_t *enc, const int32_t *h, const int32_t *t, int64_t B, const int32_t *neg, int64_t N,
                   uint64_t seed, uint64_t step, const float *proj, const float *de, float *g_es, float *g_mh, float *g_mt,
                   void *ws, size_t ws_bytes, void *hip_stream) {
    int rc = kge_validate_encoder(enc);
    if (rc != KGE_OK) return rc;
    if (B < 0 || N < 0 || 2 * B + N >= (1ll << 30) || step >= (1ull << 32)) return KGE_E_INVALID_ARG;
    if (B > 0 && (!h || !t)) return KGE_E_INVALID_ARG;
    if (N > 0 && !neg) return KGE_E_INVALID_ARG;
    if (2 * B + N > 0 && (!proj || !de || !g_es)) return KGE_E_INVALID_ARG;
    if (!g_mh || !g_mt) return KGE_E_INVALID_ARG;
    if (!ws) return KGE_E_WORKSPACE_TOO_SMALL;
    ws = align_ws(ws, ws_bytes);
    if (kge_encode_ws(*enc, B, N, true) - 256 > ws_bytes) return KGE_E_WORKSPACE_TOO_SMALL;
    return kge_run_encode_bwd(*enc, h, t, B, neg, N, seed, step, proj, de, g_es, g_mh, g_mt, ws, (hipStream_t)hip_stream);
}

int kge_sampler_build(const int32_t *h, const int32_t *r, const int32_t *t, int64_t n, int64_t part_size, int32_t D,
                      int64_t n_rel, int64_t *order, int64_t *rel_offsets, uint64_t *cdf, void *ws, size_t ws_bytes,
                      void *hip_stream) {
    if (n < 0 || n >= (1ll << 31) || part_size <= 0 || D < 1 || D > 64 || n_rel < 1) return KGE_E_INVALID_ARG;
    if ((int64_t)D * D * n_rel >= (1ll << 31)) return KGE_E_INVALID_ARG;
    if (!rel_offsets || !cdf || (n > 0 && (!h || !r || !t || !order))) return KGE_E_INVALID_ARG;
    if (n > 0 && !ws) return KGE_E_WORKSPACE_TOO_SMALL;
    ws = align_ws(ws, ws_bytes);
    if (n > 0 && kge_sampler_ws(n) - 256 > ws_bytes) return KGE_E_WORKSPACE_TOO_SMALL;
    return kge_run_sampler_build(h, r, t, n, part_size, D, n_rel, order, rel_offsets, cdf, ws, (hipStream_t)hip_stream);
}

int kge_sample_triples(uint64_t seed, uint64_t step, uint32_t stream_tag, int64_t bucket_lo, int64_t n_buckets,
                       int64_t per_bucket, int32_t D, int64_t n_rel, const int64_t *rel_offsets, const uint64_t *cdf,
                       const int64_t *order, const int32_t *h, const int32_t *r, const int32_t *t, int64_t *out_pos,
                       int32_t *out_h, int32_t *out_r, int32_t *out_t, void *hip_stream) {
    if (D < 1 || D > 64 || n_rel < 1 || bucket_lo < 0 || n_buckets < 0 || per_bucket < 0 || step >= (1ull << 32))
        return KGE_E_INVALID_ARG;
    if (bucket_lo + n_buckets > (int64_t)D * D) return KGE_E_INVALID_ARG;
    const int64_t draws = n_buckets * per_bucket;
    if (draws == 0) return KGE_OK;
    if (draws >= (1ll << 31) || !rel_offsets || !cdf || !order) return KGE_E_INVALID_ARG;
    if (!out_pos && !out_h) return KGE_E_INVALID_ARG;
    if (out_h && (!out_r || !out_t || !h || !r || !t)) return KGE_E_INVALID_ARG;
    return kge_run_sample_triples(seed, step, stream_tag, bucket_lo, draws, per_bucket, n_rel, rel_offsets, cdf, order, h, r,
                                  t, out_pos, out_h, out_r, out_t, (hipStream_t)hip_stream);
}

int kge_sample_negatives_sharded(uint64_t seed, uint64_t step, uint32_t stream_tag, int64_t part_size, int64_t n_ent,
                                 int32_t D, int64_t per_shard, int32_t *out_idx, void *hip_stream) {
    if (D < 1 || D > 64 || part_size <= 0 || per_shard < 0 || n_ent <= 0 || n_ent > (1ll << 31) || step >= (1ull << 32))
        return KGE_E_INVALID_ARG;
    if ((int64_t)(D - 1) * part_size >= n_ent || (int64_t)D * part_size < n_ent) return KGE_E_INVALID_ARG;   // D non-empty shards
    const int64_t n = (int64_t)D * per_shard;
    if (n == 0) return KGE_OK;
    if (n >= (1ll << 31) || !out_idx) return KGE_E_INVALID_ARG;
    return kge_run_negatives_sharded(seed, step, stream_tag, part_size, n_ent, per_shard, n, out_idx, (hipStream_t)hip_stream);
}

int kge_score(const kge_model_t *model, const int32_t *h, const int32_t *r, const int32_t *t, int64_t B,
              const int32_t *neg, int64_t N, float *pos_out, float *neg_out, void *ws, size_t ws_bytes,
              void *hip_stream) {
    int rc = validate_model(model);
    if (rc != KGE_OK) return rc;
    if (B < 0 || N < 0 || B >= (1ll << 30) || N >= (1ll << 30)) return KGE_E_INVALID_ARG;
    if (B == 0) return KGE_OK;
    if (!h || !r || !t || (N > 0 && !neg)) return KGE_E_INVALID_ARG;
    if (!ws) return KGE_E_WORKSPACE_TOO_SMALL;
    hipStream_t st = (hipStream_t)hip_stream;
    const bool block = N > 0 && neg_out;
    Geometry g = make_geometry(*model, B, block ? N : 0);
    Buffers b;
    ws = align_ws(ws, ws_bytes);
    if (carve(g, false, nullptr, b) - 256 > ws_bytes) return KGE_E_WORKSPACE_TOO_SMALL;
    carve(g, false, ws, b);
    KgeModelDev md = dev_model(*model);
    // (queries and negatives from one launch when there is a block to score)
    if (block && g.Bp > 0)
        rc = kge_run_qbuild_tgather(md, h, r, t, g.B, g.Bp, g.dp, b.Q, b.W, nullptr, b.Q32, b.W32, b.rowinfo, b.pos, neg, g.N, g.Np,
                                    b.T, b.tn, st, pos_out, b.Qp2, b.Tp2, b.t_inv);
    else
        rc = kge_run_qbuild(md, h, r, t, g.B, g.Bp, g.dp, b.Q, b.W, nullptr, b.Q32, b.W32, b.rowinfo, b.pos, pos_out, st, b.Qp2);
    if (rc != KGE_OK || !block) return rc;
    if (g.l1 && g.transh)
        return kge_run_l1h_score(g.bf16, b.Q32, b.W32, b.T, g.B, g.N, g.Bp, g.Np, g.dp, neg_out, nullptr, nullptr, g.N, st);
    if (g.l1) return kge_run_l1_score(g.bf16, b.Q32, b.T, g.B, g.N, g.Bp, g.Np, g.dp, neg_out, g.N, st);
    if (score_h2_applies(g)) {
        return kge_launch_score_h2(g.kind, g.dp, b.Qp2, b.Tp2, b.t_inv, (const float *)b.Q, (const float *)b.T,
                                 g.transh ? (const float *)b.W : nullptr, b.rowinfo, b.tn, g.B, g.N,
                                 g.Bp, g.Np, neg_out, st);
    }
    KgeBlockArgs a{};
    a.own = b.T; a.str = b.Q; a.str2 = b.W; a.rowinfo = b.rowinfo; a.tn = b.tn;
    a.B = g.B; a.N = g.N; a.dp = g.dp; a.str_tiles = g.str_tiles_b; a.tiles_per_split = g.tps_s;
    a.kind = g.kind; a.S_out = neg_out; a.own_pad = g.Np;
    return launch_block(g, KGE_MODE_SCORE, 0, a, g.own_tiles_s, g.nsplit_s, 1, st);
}

// kge_loss_bwd and kge_loss_bwd_sampled (gen: the draw of the negatives, gen->out their ids' place; else neg holds them)
static int loss_bwd_impl(const kge_model_t *model, const kge_loss_cfg_t *cfg, const int32_t *h, const int32_t *r,
                         const int32_t *t, int64_t B, const int32_t *neg, const KgeNegGen *gen, int64_t N, float *loss_out,
                         float *g_ent, int32_t *g_ent_idx, float *g_rel, float *g_relw, int32_t *g_rel_idx, void *ws,
                         size_t ws_bytes, void *hip_stream, const kge_adam_plan_t *plans = nullptr, int n_plans = 0) {
    if (gen) neg = gen->out;
    int rc = validate_model(model);
    if (rc != KGE_OK) return rc;
    if (!cfg || (cfg->loss != KGE_LOGSIGMOID && cfg->loss != KGE_SAMPLED_SOFTMAX)) return KGE_E_INVALID_ARG;
    if (B < 0 || N < 0 || B >= (1ll << 30) || N >= (1ll << 30)) return KGE_E_INVALID_ARG;
    if (!(cfg->adv_temp >= 0.f) || !(cfg->reg_l3 >= 0.f)) return KGE_E_INVALID_ARG;
    if (cfg->loss == KGE_SAMPLED_SOFTMAX && N > 0 && cfg->n_ent_for_c < 2) return KGE_E_INVALID_ARG;
    if (!loss_out) return KGE_E_INVALID_ARG;
    if (B > 0 && (!h || !r || !t || !g_ent || !g_ent_idx || !g_rel || !g_rel_idx)) return KGE_E_INVALID_ARG;
    if (N > 0 && (!neg || !g_ent || !g_ent_idx)) return KGE_E_INVALID_ARG;
    if (model->scorer == KGE_TRANSH && B > 0 && !g_relw) return KGE_E_INVALID_ARG;
    Geometry g = make_geometry(*model, B, N, true);
    if (!ws) return KGE_E_WORKSPACE_TOO_SMALL;
    hipStream_t st = (hipStream_t)hip_stream;
    Buffers b;
    ws = align_ws(ws, ws_bytes);
    if (carve(g, true, nullptr, b) - 256 > ws_bytes) return KGE_E_WORKSPACE_TOO_SMALL;
    carve(g, true, ws, b);
    KgeModelDev md = dev_model(*model);
    md.vec = g.l1;
    const float scale = cfg->loss_scale > 0.f ? cfg->loss_scale : (B > 0 ? 1.f / (float)B : 1.f);
    const float c_corr = (cfg->loss == KGE_SAMPLED_SOFTMAX && N > 0)
                             ? (float)log((double)(cfg->n_ent_for_c - 1) / (double)N) : 0.f;
    const bool have_block = B > 0 && N > 0;
    // sampled softmax, bilinear scorers on bf16 rows of 512 bytes: the forward pass keeps its weights, the pass over the
    // negatives contracts them with the scaled queries instead of scoring every pair again
    const bool keep_weights = have_block && !g.l1 && cfg->loss == KGE_SAMPLED_SOFTMAX && b.pstore != nullptr;

    // (the kernels that need no transposed copy of the negatives get queries and negatives from ONE launch)
    const bool plain_gather = have_block && (g.l1 || kge_fwd_pp_applies(g.bf16, g.rb, g.transh, g.dsplit_q));
    // (negatives that the call draws itself: in that launch; where the rows are gathered otherwise, in a launch of their own)
    if (gen && N > 0 && !plain_gather) {
        rc = kge_run_negatives(((uint64_t)gen->seed_hi << 32) | gen->seed_lo, gen->step, gen->step_counter, gen->tag, gen->lo,
                               gen->lo + (int64_t)gen->range, N, gen->out, st);
        if (rc != KGE_OK) return rc;
    }
    if (plain_gather) {
        KgeProfScope prof(KGE_PROF_GATHER, st);
        rc = kge_run_qbuild_tgather(md, h, r, t, g.B, g.Bp, g.dp, b.Q, b.W, b.Q2, b.Q32, b.W32, b.rowinfo, b.pos,
                                    neg, g.N, g.Np, b.T, b.tn, st, nullptr, nullptr, nullptr, nullptr, b.nbias, gen);
    }
    else rc = kge_run_qbuild(md, h, r, t, g.B, g.Bp, g.dp, b.Q, b.W, b.Q2, b.Q32, b.W32, b.rowinfo, b.pos, nullptr, st);
    if (rc != KGE_OK) return rc;
    KgeBlockArgs a{};
    if (have_block && g.l1) {
        // 1-norm: the score block goes to memory, one row pass gives the loss statistics
        rc = g.transh ? kge_run_l1h_score(g.bf16, b.Q32, b.W32, b.T, g.B, g.N, g.Bp, g.Np, g.dp, b.S, b.A, b.P, g.Np, st, g.pn)
                      : kge_run_l1_score(g.bf16, b.Q32, b.T, g.B, g.N, g.Bp, g.Np, g.dp, b.S, g.Np, st);
        if (rc != KGE_OK) return rc;
        if ((rc = kge_run_l1_rowstat(b.S, g.Np, g.B, g.N, g.Bp, cfg->loss, cfg->gamma, cfg->adv_temp, b.stat_part, st)) != KGE_OK) return rc;
    } else if (have_block) {
        // (the two-role row-owner kernel transposes its tiles in the LDS and needs no transposed copy of the negatives)
        if (!plain_gather && (rc = kge_run_tgather_t(md, neg, g.N, g.Np, g.dp, b.T, b.Tt, b.tn, st)) != KGE_OK) return rc;
        // (nor does the two-role kernel of the pass over the negatives need transposed queries)
        if (!kge_gradt_pp_applies(g.bf16, g.rb, g.transh, g.dsplit_t) &&
            (rc = kge_run_transpose(g.transh ? b.Q2 : b.Q, b.Qt, g.Bp, g.dp, g.bf16, st)) != KGE_OK) return rc;
        if (g.transh && (rc = kge_run_transpose(b.W, b.Wt, g.Bp, g.dp, g.bf16, st)) != KGE_OK) return rc;
        // pass 1 (row owner): loss statistics of every row and the unnormalised gradient of the queries
        a.own = b.Q; a.own2 = b.W; a.str = b.T; a.strT = b.Tt; a.strT_ld = g.Np; a.rowinfo = b.rowinfo; a.tn = b.tn;
        a.B = g.B; a.N = g.N; a.dp = g.dp; a.str_tiles = g.str_tiles_n; a.tiles_per_split = g.tps_q;
        a.kind = g.kind; a.loss = cfg->loss; a.gamma = cfg->gamma; a.adv_temp = cfg->adv_temp; a.c_corr = c_corr;
        a.stat_part = b.stat_part; a.acc_part = b.accq; a.acc_part2 = b.accq2; a.sum_part = b.sumq; a.own_pad = g.Bp;
        a.str_bias = b.nbias;
        if (keep_weights) { a.pstore = b.pstore; a.ps_nsplit = g.nsplit_q; a.ps_rounds = g.tps_q / 2; a.part_bf16 = 1; }
        if ((rc = launch_block(g, KGE_MODE_FWD, cfg->loss, a, g.own_tiles_b, g.nsplit_q, g.dsplit_q, st)) != KGE_OK) return rc;
    }
    // (the plans of the sparse update that the caller asked for: their sorts need the ids alone and share the launch of the
    // rows' finish where there is one of that kind; otherwise they follow at the end)
    bool planned = false;
    if (keep_weights && plans) {
        const KgeRowFinishQArgs rf{b.stat_part, g.nsplit_q, g.Bp, g.B, g.N, cfg->loss, cfg->gamma, c_corr, scale, b.pos, b.rowinfo,
                                   b.lossb, b.gpos, (const uint16_t *)b.Q, (uint16_t *)b.Qs};
        rc = kge_run_sparse_adam_plan_tables(plans, n_plans, st, &rf);
        planned = true;
    } else if (keep_weights)
        rc = kge_run_rowfinish_qscale(b.stat_part, g.nsplit_q, g.Bp, g.B, g.N, cfg->loss, cfg->gamma, c_corr, scale, b.pos, b.rowinfo,
                                      b.lossb, b.gpos, b.Q, b.Qs, st);
    else
        rc = kge_run_rowfinish(b.stat_part, have_block ? (g.l1 ? 1 : g.nsplit_q) : 0, g.Bp, g.B, have_block ? g.N : 0, cfg->loss,
                               cfg->gamma, c_corr, scale, b.pos, b.rowinfo, b.lossb, b.gpos, have_block ? nullptr : loss_out, st);
    if (rc != KGE_OK) return rc;
    if (have_block && g.l1 && g.transh) {
        if ((rc = kge_run_l1h_grad(g.bf16, true, b.Q32, b.W32, b.T, b.S, b.A, b.P, g.Np, b.rowinfo, g.B, g.N, g.Bp, g.Np, g.dp,
                                   cfg->loss, cfg->gamma, cfg->adv_temp, g.nsplit_q, b.accq, b.accq2, st, g.pn)) != KGE_OK) return rc;
        if ((rc = kge_run_l1h_grad(g.bf16, false, b.Q32, b.W32, b.T, b.S, b.A, b.P, g.Np, b.rowinfo, g.B, g.N, g.Np, g.Bp, g.dp,
                                   cfg->loss, cfg->gamma, cfg->adv_temp, g.nsplit_t, b.acct, nullptr, st, g.pn)) != KGE_OK) return rc;
    } else if (have_block && g.l1) {
        // gradient rows of the queries and of the shared negatives from S and the finished row constants
        if ((rc = kge_run_l1_grad(g.bf16, true, b.Q32, b.T, b.S, g.Np, b.rowinfo, g.B, g.N, g.Bp, g.Np, g.dp, cfg->loss, cfg->gamma,
                                  cfg->adv_temp, g.nsplit_q, b.accq, st)) != KGE_OK) return rc;
        if ((rc = kge_run_l1_grad(g.bf16, false, b.T, b.Q32, b.S, g.Np, b.rowinfo, g.B, g.N, g.Np, g.Bp, g.dp, cfg->loss, cfg->gamma,
                                  cfg->adv_temp, g.nsplit_t, b.acct, st)) != KGE_OK) return rc;
    } else if (have_block) {
        // pass 2 (column owner): gradient of the shared negatives from the finished row constants
        KgeBlockArgs c = a;
        c.own = b.T; c.own2 = nullptr; c.str = b.Q; c.str2 = b.W; c.strT = b.Qt; c.strT2 = b.Wt; c.strT_ld = g.Bp;
        c.str_tiles = g.str_tiles_b; c.tiles_per_split = g.tps_t;
        c.acc_part = b.acct; c.acc_part2 = nullptr; c.sum_part = b.sumt; c.stat_part = nullptr; c.own_pad = g.Np;
        if (keep_weights) c.str2 = b.Qs; else c.pstore = nullptr;    // (str2: the scaled queries; the recomputing kernel behind streams the plain ones)
        if ((rc = launch_block(g, KGE_MODE_GRADT, cfg->loss, c, g.own_tiles_n, g.nsplit_t, g.dsplit_t, st)) != KGE_OK) return rc;
    }
    if (have_block) {
        // chain rule of the queries and finish of the negatives' gradient rows in ONE launch
        KgeProfScope prof(KGE_PROF_FINISH, st);
        rc = kge_run_chain_tfinish(md, h, r, t, g.B, g.Bp, g.dp, b.accq, b.accq2, b.sumq, b.stat_part, b.rowinfo, g.nsplit_q, b.gpos,
                                   g_ent, g_rel, g_relw, g_ent_idx, g_rel_idx, cfg->reg_l3, b.regv,
                                   b.acct, b.sumt, g.nsplit_t, g.Np, g.N, model->dim, g.kind == KGE_KIND_DIST && !g.l1, b.T, neg,
                                   g_ent + (size_t)2 * B * model->dim, g_ent_idx + 2 * B, b.regv + (size_t)2 * g.Bp,
                                   b.lossb, scale, loss_out, st, keep_weights);
        if (rc != KGE_OK) return rc;
    } else {
        if ((rc = kge_run_chain(md, h, r, t, g.B, g.Bp, g.dp, b.accq, b.accq2, b.sumq, b.stat_part, b.rowinfo, 0, b.gpos,
                                g_ent, g_rel, g_relw, g_ent_idx, g_rel_idx, cfg->reg_l3, b.regv, st)) != KGE_OK) return rc;
        if (N > 0) {
            // with B == 0 there are no partials: nsplit 0 writes zero rows (plus the regulariser of the rows, read from the table)
            rc = kge_run_tfinish(b.acct, b.sumt, 0, g.Np, g.N, g.dp, model->dim, 0, nullptr, g.bf16, neg,
                                 g_ent + (size_t)2 * B * model->dim, g_ent_idx + 2 * B, model->ent, model->ent_ld, cfg->reg_l3,
                                 b.regv + (size_t)2 * g.Bp, st);
            if (rc != KGE_OK) return rc;
        }
    }
    if (cfg->reg_l3 > 0.f && B + N > 0) rc = kge_run_reg_add(b.regv, g.B, g.Bp, g.N, cfg->reg_l3, loss_out, st);
    if (rc == KGE_OK && plans && !planned) rc = kge_run_sparse_adam_plan_tables(plans, n_plans, st);
    return rc;
}

int kge_loss_bwd(const kge_model_t *model, const kge_loss_cfg_t *cfg, const int32_t *h, const int32_t *r,
                 const int32_t *t, int64_t B, const int32_t *neg, int64_t N, float *loss_out, float *g_ent,
                 int32_t *g_ent_idx, float *g_rel, float *g_relw, int32_t *g_rel_idx, void *ws, size_t ws_bytes,
                 void *hip_stream) {
    return loss_bwd_impl(model, cfg, h, r, t, B, neg, nullptr, N, loss_out, g_ent, g_ent_idx, g_rel, g_relw, g_rel_idx, ws,
                         ws_bytes, hip_stream);
}

static int loss_bwd_sampled_impl(const kge_model_t *model, const kge_loss_cfg_t *cfg, const int32_t *h, const int32_t *r,
                                 const int32_t *t, int64_t B, const kge_neg_draw_t *draw, int32_t *neg_out, int64_t N,
                                 float *loss_out, float *g_ent, int32_t *g_ent_idx, float *g_rel, float *g_relw,
                                 int32_t *g_rel_idx, void *ws, size_t ws_bytes, const kge_adam_plan_t *plans, int32_t n_tables,
                                 void *hip_stream) {
    if (!draw || draw->hi <= draw->lo || draw->lo < 0 || draw->hi > (1ll << 31) || draw->step >= (1ull << 32) || draw->reserved != 0)
        return KGE_E_INVALID_ARG;
    if (N > 0 && !neg_out) return KGE_E_INVALID_ARG;
    const KgeNegGen gen{neg_out, (uint32_t)draw->seed, (uint32_t)(draw->seed >> 32), (uint32_t)draw->step, draw->stream_tag,
                        draw->step_counter, draw->lo, (uint64_t)(draw->hi - draw->lo)};
    return loss_bwd_impl(model, cfg, h, r, t, B, nullptr, &gen, N, loss_out, g_ent, g_ent_idx, g_rel, g_relw, g_rel_idx, ws,
                         ws_bytes, hip_stream, plans, n_tables);
}

int kge_loss_bwd_sampled(const kge_model_t *model, const kge_loss_cfg_t *cfg, const int32_t *h, const int32_t *r,
                         const int32_t *t, int64_t B, const kge_neg_draw_t *draw, int32_t *neg_out, int64_t N,
                         float *loss_out, float *g_ent, int32_t *g_ent_idx, float *g_rel, float *g_relw,
                         int32_t *g_rel_idx, void *ws, size_t ws_bytes, void *hip_stream) {
    return loss_bwd_sampled_impl(model, cfg, h, r, t, B, draw, neg_out, N, loss_out, g_ent, g_ent_idx, g_rel, g_relw, g_rel_idx,
                                 ws, ws_bytes, nullptr, 0, hip_stream);
}

// argument checks shared by kge_sparse_adam and kge_sparse_adam_static; KGE_OK with M == 0 means "nothing to do"
static int validate_sparse_adam(const float *param_f32, const void *param_bf16, const float *m, const float *v, int64_t n_rows,
                                int32_t dim, int64_t ld, const int32_t *idx, const float *grads, int64_t M,
                                const kge_adam_cfg_t *cfg) {
    if (!cfg || M < 0 || n_rows <= 0 || n_rows >= (1ll << 31) || dim <= 0 || dim % 4 != 0 || dim > 4096 || ld < dim || ld % 4 != 0)
        return KGE_E_INVALID_ARG;
    if (cfg->step < 1 || !(cfg->beta1 >= 0.f && cfg->beta1 < 1.f) || !(cfg->beta2 >= 0.f && cfg->beta2 < 1.f))
        return KGE_E_INVALID_ARG;
    if (M == 0) return KGE_OK;
    if (M >= (1ll << 31)) return KGE_E_INVALID_ARG;
    if (!param_f32 || !m || !v || !idx || !grads) return KGE_E_INVALID_ARG;
    if (!adam_rows_aligned(param_f32, param_bf16, m, v, grads)) return KGE_E_INVALID_ARG;
    return KGE_OK;
}

int kge_sparse_adam(float *param_f32, void *param_bf16, float *m, float *v, int64_t n_rows, int32_t dim,
                    int64_t ld, const int32_t *idx, const float *grads, int64_t M, const kge_adam_cfg_t *cfg,
                    void *ws, size_t ws_bytes, void *hip_stream) {
    const int rc = validate_sparse_adam(param_f32, param_bf16, m, v, n_rows, dim, ld, idx, grads, M, cfg);
    if (rc != KGE_OK || M == 0) return rc;
    if (!ws) return KGE_E_WORKSPACE_TOO_SMALL;
    ws = align_ws(ws, ws_bytes);
    if (kge_sparse_adam_ws(M, dim) - 256 > ws_bytes) return KGE_E_WORKSPACE_TOO_SMALL;
    return kge_run_sparse_adam(param_f32, param_bf16, m, v, n_rows, dim, ld, idx, grads, M, *cfg, ws, ws_bytes,
                               (hipStream_t)hip_stream);
}

size_t kge_sparse_adam_static_limit(void) { return kge_static_scratch_bytes(); }

int kge_sparse_adam_static(float *param_f32, void *param_bf16, float *m, float *v, int64_t n_rows, int32_t dim,
                           int64_t ld, const int32_t *idx, const float *grads, int64_t M, const kge_adam_cfg_t *cfg,
                           void *hip_stream) {
    const int rc = validate_sparse_adam(param_f32, param_bf16, m, v, n_rows, dim, ld, idx, grads, M, cfg);
    if (rc != KGE_OK || M == 0) return rc;
    if (kge_sparse_adam_ws(M, dim) > kge_static_scratch_bytes()) return KGE_E_STATIC_SCRATCH_TOO_SMALL;
    void *ws = nullptr; size_t ws_bytes = 0;
    const int rs = kge_static_scratch(&ws, &ws_bytes);
    if (rs != KGE_OK) return rs;
    return kge_run_sparse_adam(param_f32, param_bf16, m, v, n_rows, dim, ld, idx, grads, M, *cfg, ws, ws_bytes,
                               (hipStream_t)hip_stream);
}

int kge_sparse_adam_plan(int64_t n_rows, int32_t dim, const int32_t *idx, int64_t M, void *ws, size_t ws_bytes,
                         void *hip_stream) {
    if (M < 0 || n_rows <= 0 || n_rows >= (1ll << 31) || dim <= 0 || dim % 4 != 0 || dim > 4096) return KGE_E_INVALID_ARG;
    if (M == 0) return KGE_OK;
    if (M >= (1ll << 31) || !idx) return KGE_E_INVALID_ARG;
    if (!ws) return KGE_E_WORKSPACE_TOO_SMALL;
    ws = align_ws(ws, ws_bytes);
    if (kge_sparse_adam_ws(M, dim) - 256 > ws_bytes) return KGE_E_WORKSPACE_TOO_SMALL;
    return kge_run_sparse_adam_plan(n_rows, idx, M, ws, (hipStream_t)hip_stream);
}

int kge_sparse_adam_apply(float *param_f32, void *param_bf16, float *m, float *v, int64_t n_rows, int32_t dim,
                          int64_t ld, const float *grads, int64_t M, const kge_adam_cfg_t *cfg, void *ws,
                          size_t ws_bytes, void *hip_stream) {
    if (!cfg || M < 0 || n_rows <= 0 || n_rows >= (1ll << 31) || dim <= 0 || dim % 4 != 0 || dim > 4096 || ld < dim ||
        ld % 4 != 0)
        return KGE_E_INVALID_ARG;
    if (cfg->step < 1 || !(cfg->beta1 >= 0.f && cfg->beta1 < 1.f) || !(cfg->beta2 >= 0.f && cfg->beta2 < 1.f))
        return KGE_E_INVALID_ARG;
    if (M == 0) return KGE_OK;
    if (M >= (1ll << 31)) return KGE_E_INVALID_ARG;
    if (!param_f32 || !m || !v || !grads) return KGE_E_INVALID_ARG;
    if (!adam_rows_aligned(param_f32, param_bf16, m, v, grads)) return KGE_E_INVALID_ARG;
    if (!ws) return KGE_E_WORKSPACE_TOO_SMALL;
    ws = align_ws(ws, ws_bytes);
    if (kge_sparse_adam_ws(M, dim) - 256 > ws_bytes) return KGE_E_WORKSPACE_TOO_SMALL;
    return kge_run_sparse_adam_apply(param_f32, param_bf16, m, v, n_rows, dim, ld, grads, M, *cfg, ws,
                                     (hipStream_t)hip_stream);
}

static int validate_plans(const kge_adam_plan_t *plans, int32_t n_tables) {
    if (!plans || n_tables < 1 || n_tables > 4) return KGE_E_INVALID_ARG;
    for (int k = 0; k < n_tables; ++k) {
        const kge_adam_plan_t &t = plans[k];
        if (t.M < 0 || t.n_rows <= 0 || t.n_rows >= (1ll << 31) || t.dim <= 0 || t.dim % 4 != 0 || t.dim > 4096 || t.M >= (1ll << 31))
            return KGE_E_INVALID_ARG;
        if (t.M == 0) continue;
        if (!t.idx) return KGE_E_INVALID_ARG;
        if (!t.ws) return KGE_E_WORKSPACE_TOO_SMALL;
        size_t bytes = t.ws_bytes;
        void *ws = t.ws;
        ws = align_ws(ws, bytes);
        if (kge_sparse_adam_ws(t.M, t.dim) - 256 > bytes) return KGE_E_WORKSPACE_TOO_SMALL;
    }
    return KGE_OK;
}

int kge_sparse_adam_plan_tables(const kge_adam_plan_t *plans, int32_t n_tables, void *hip_stream) {
    const int rc = validate_plans(plans, n_tables);
    if (rc != KGE_OK) return rc;
    return kge_run_sparse_adam_plan_tables(plans, n_tables, (hipStream_t)hip_stream);
}

int kge_loss_bwd_sampled_planned(const kge_model_t *model, const kge_loss_cfg_t *cfg, const int32_t *h, const int32_t *r,
                                 const int32_t *t, int64_t B, const kge_neg_draw_t *draw, int32_t *neg_out, int64_t N,
                                 float *loss_out, float *g_ent, int32_t *g_ent_idx, float *g_rel, float *g_relw,
                                 int32_t *g_rel_idx, void *ws, size_t ws_bytes, const kge_adam_plan_t *plans,
                                 int32_t n_tables, void *hip_stream) {
    const int rc = validate_plans(plans, n_tables);
    if (rc != KGE_OK) return rc;
    for (int k = 0; k < n_tables; ++k)                      // (the sorts may run before these arrays are written)
        if (plans[k].M > 0 && (plans[k].idx == g_ent_idx || plans[k].idx == g_rel_idx)) return KGE_E_INVALID_ARG;
    return loss_bwd_sampled_impl(model, cfg, h, r, t, B, draw, neg_out, N, loss_out, g_ent, g_ent_idx, g_rel, g_relw, g_rel_idx,
                                 ws, ws_bytes, plans, n_tables, hip_stream);
}

int kge_sparse_adam_apply_tables(const kge_adam_table_t *tables, int32_t n_tables, const kge_adam_cfg_t *cfg, void *hip_stream) {
    if (!tables || !cfg || n_tables < 1 || n_tables > 4) return KGE_E_INVALID_ARG;
    if (cfg->step < 1 || !(cfg->beta1 >= 0.f && cfg->beta1 < 1.f) || !(cfg->beta2 >= 0.f && cfg->beta2 < 1.f))
        return KGE_E_INVALID_ARG;
    kge_adam_table_t live[4];
    int n = 0;
    for (int k = 0; k < n_tables; ++k) {
        const kge_adam_table_t &t = tables[k];
        if (t.M < 0 || t.n_rows <= 0 || t.n_rows >= (1ll << 31) || t.dim <= 0 || t.dim % 4 != 0 || t.dim > 4096 || t.ld < t.dim ||
            t.ld % 4 != 0 || t.M >= (1ll << 31))
            return KGE_E_INVALID_ARG;
        if (t.M == 0) continue;
        if (!t.param_f32 || !t.m || !t.v || !t.grads) return KGE_E_INVALID_ARG;
        if (!adam_rows_aligned(t.param_f32, t.param_bf16, t.m, t.v, t.grads)) return KGE_E_INVALID_ARG;
        if (!t.ws) return KGE_E_WORKSPACE_TOO_SMALL;
        size_t bytes = t.ws_bytes;
        void *ws = t.ws;
        ws = align_ws(ws, bytes);
        if (kge_sparse_adam_ws(t.M, t.dim) - 256 > bytes) return KGE_E_WORKSPACE_TOO_SMALL;
        live[n] = t; live[n].ws = ws; live[n].ws_bytes = bytes;
        ++n;
    }
    if (n == 0) return KGE_OK;
    return kge_run_sparse_adam_apply_tables(live, n, *cfg, (hipStream_t)hip_stream);
}

int kge_topk(const kge_model_t *model, const int32_t *h, const int32_t *r, int64_t Q, int64_t cand_lo,
             int64_t cand_hi, int32_t K, int32_t *out_idx, float *out_score, const int32_t *true_t,
             int64_t *out_rank, void *ws, size_t ws_bytes, void *hip_stream) {
    int rc = validate_model(model);
    if (rc != KGE_OK) return rc;
    if (Q < 0 || Q >= (1ll << 30) || cand_lo < 0 || cand_hi < cand_lo || cand_hi > model->n_ent) return KGE_E_INVALID_ARG;
    if (K < 1 || K > 256) return KGE_E_INVALID_ARG;
    if ((true_t == nullptr) != (out_rank == nullptr)) return KGE_E_INVALID_ARG;
    if (model->scorer == KGE_TRANSH && (int64_t)model->dim * (model->dtype == KGE_BF16 ? 2 : 4) > 512) return KGE_E_UNSUPPORTED;
    if ((model->scorer == KGE_TRANSE || model->scorer == KGE_ROTATE || model->scorer == KGE_TRANSH) && model->p_norm != 2)
        return KGE_E_UNSUPPORTED;
    // the scan copies candidate rows straight from the table in 16-byte pieces
    if (((uintptr_t)model->ent & 15) != 0 || (model->ent_ld * (model->dtype == KGE_BF16 ? 2 : 4)) % 16 != 0) return KGE_E_UNSUPPORTED;
    if (Q == 0) return KGE_OK;
    if (!h || !r || !out_idx || !out_score) return KGE_E_INVALID_ARG;
    if (!ws) return KGE_E_WORKSPACE_TOO_SMALL;
    ws = align_ws(ws, ws_bytes);
    if (kge_topk_ws(*model, Q, cand_hi - cand_lo, K) - 256 > ws_bytes) return KGE_E_WORKSPACE_TOO_SMALL;
    return kge_run_topk(*model, h, r, Q, cand_lo, cand_hi, K, out_idx, out_score, true_t, out_rank, ws, ws_bytes,
                        (hipStream_t)hip_stream);
}

int kge_ensemble(const int32_t *lists, int32_t M, int64_t Q, int32_t K, double p, int32_t K_out, int32_t *out_idx,
                 float *out_score, void *hip_stream) {
    if (M < 1 || K < 1 || Q < 0 || Q >= (1ll << 31) || K_out < 1 || K_out > 256 || !(p != 0.0) || !(p == p) || !(fabs(p) <= 64.0))
        return KGE_E_INVALID_ARG;
    if (Q == 0) return KGE_OK;
    if (!lists || !out_idx || !out_score) return KGE_E_INVALID_ARG;
    return kge_run_ensemble(lists, M, Q, K, p, K_out, out_idx, out_score, (hipStream_t)hip_stream);
}

int kge_partition_triples(const int32_t *h, const int32_t *t, int64_t n, int64_t part_size, int32_t D,
                          int64_t *bucket_offsets, int64_t *order, void *ws, size_t ws_bytes, void *hip_stream) {
    if (n < 0 || part_size <= 0 || D < 1 || D > 64 || !bucket_offsets) return KGE_E_INVALID_ARG;
    if (n > 0 && (!h || !t || !order)) return KGE_E_INVALID_ARG;
    if (!ws) return KGE_E_WORKSPACE_TOO_SMALL;
    ws = align_ws(ws, ws_bytes);
    if (kge_partition_ws(n, D) - 256 > ws_bytes) return KGE_E_WORKSPACE_TOO_SMALL;
    return kge_run_partition(h, t, n, part_size, D, bucket_offsets, order, ws, ws_bytes, (hipStream_t)hip_stream);
}

}  // extern "C"
