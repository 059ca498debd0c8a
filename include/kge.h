/*
 * kge.h -- C ABI of the MI355X (gfx950) knowledge-graph-embedding hot path.
 *
 * One GPU plays one BESS worker (arXiv 2211.12281, Section 4): it gathers the (h, r, t) embedding
 * rows of a micro-batch, scores every query against its positive tail and against ONE block of
 * negative tails shared by the whole micro-batch, evaluates the loss and its backward pass, and
 * applies a duplicate-aware sparse Adam update to the touched rows; for link prediction it scores
 * queries against a range of entity rows and returns the top-K.
 *
 * Conventions for every entry point
 *  - Structs (kge_model_t, kge_loss_cfg_t, kge_adam_cfg_t) are read on the HOST during the call.
 *    Every other pointer is a DEVICE pointer into memory owned by the caller; the library neither
 *    allocates nor frees device memory and keeps no state between calls (the optional profiling
 *    hooks at the end of this file aside).  Scratch space comes
 *    from the caller's workspace `ws` (size from kge_workspace_bytes(); 256-byte aligned).
 *  - Work is enqueued on `hip_stream` (a hipStream_t, may be NULL for the default stream) and the
 *    call returns without waiting for it.  Calls that share a workspace must be ordered on one
 *    stream.  The training calls (kge_sample_negatives*, kge_loss_bwd, kge_sparse_adam*) only launch
 *    kernels: no allocation, no synchronisation, no memset or copy node, so a stream that is being
 *    captured into a HIP graph may be passed; what changes from one replay to the next then comes
 *    from a counter in device memory (kge_step_counter_add below).
 *  - Return value: KGE_OK (0) or a negative KGE_E_* code.  Arguments are validated on the host
 *    before anything is launched; on error nothing has been enqueued.
 *  - Index VALUES are not range-checked on the device: ids outside [0, n_ent) / [0, n_rel) are
 *    undefined behaviour.  n_ent, n_rel < 2^31.
 *  - Table layout: row-major, row i of a table starts at element i*ld; dtype KGE_F32 (float) or
 *    KGE_BF16 (bfloat16 bit patterns).  `dim` (d) must be a multiple of 8 (fp32) or 16 (bf16);
 *    d*sizeof(element) <= 1024 bytes.  Complex-valued scorers (RotatE, ComplEx) store a row as
 *    [d/2 real parts | d/2 imaginary parts].  The relation row has rel_dim = d elements, except
 *    RotatE where it holds d/2 phases (Section 3.1, "Encoder": k = d/2 for RotatE, else d).
 *  - Scores follow Table 2 with p = 2:
 *      TransE   -||h + r - t||            TransH  -||(h - (w.h)w) + r - (t - (w.t)w)||, w = relw/||relw||
 *      RotatE   -||h o e^{ir} - t||       DistMult <r, h, t>       ComplEx  Re<r, h, conj t>
 */
#ifndef KGE_H_
#define KGE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { KGE_TRANSE = 0, KGE_TRANSH = 1, KGE_ROTATE = 2, KGE_DISTMULT = 3, KGE_COMPLEX = 4 } kge_scorer_t;
typedef enum { KGE_LOGSIGMOID = 0, KGE_SAMPLED_SOFTMAX = 1 } kge_loss_t;
typedef enum { KGE_F32 = 0, KGE_BF16 = 1 } kge_dtype_t;
typedef enum { KGE_OP_SCORE = 0, KGE_OP_LOSS_BWD = 1, KGE_OP_SPARSE_ADAM = 2, KGE_OP_TOPK = 3,
               KGE_OP_PARTITION = 4, KGE_OP_SAMPLER_BUILD = 5, KGE_OP_ENCODE = 6, KGE_OP_ENCODE_BWD = 7 } kge_op_t;

enum {
    KGE_OK = 0,
    KGE_E_INVALID_ARG = -1,         /* NULL where data is required, negative size, bad enum, bad dim */
    KGE_E_UNSUPPORTED = -2,         /* valid request this build has no kernel for (e.g. kge_topk with p_norm = 1) */
    KGE_E_WORKSPACE_TOO_SMALL = -3,
    KGE_E_HIP = -4,                 /* a HIP runtime call failed (launch error) */
    KGE_E_STATIC_SCRATCH_TOO_SMALL = -5   /* kge_sparse_adam_static: the request needs more than the built-in scratch buffer */
};

/* A model = scorer + tables (Section 3.1: shallow entity / relation embeddings; TransH adds w_r). */
typedef struct {
    int32_t scorer;      /* kge_scorer_t */
    int32_t p_norm;      /* distance scorers: 2, or 1 (Table 2: p in {1, 2}) for TransE and RotatE - RotatE then takes
                            the 1-norm in R^d, |Re| + |Im| per complex coordinate; the 1-norm has no contraction
                            form, its kernels run on the vector pipe and kge_loss_bwd keeps the B x N score block
                            in the workspace (TransH: three such blocks - the scores, w^ . t and sign(x) . w^ of
                            every pair, since the hyperplane term sits inside the absolute values).  kge_topk
                            with p_norm = 1: KGE_E_UNSUPPORTED.  Ignored by DistMult and ComplEx. */
    int32_t dtype;       /* kge_dtype_t of ent, rel, relw as the kernels read them */
    int32_t dim;         /* d */
    int32_t rel_dim;     /* d, or d/2 for RotatE */
    int32_t reserved;
    int64_t n_ent, n_rel;
    const void *ent;     /* [n_ent, ent_ld] */
    const void *rel;     /* [n_rel, rel_ld] */
    const void *relw;    /* [n_rel, relw_ld], TransH only (else NULL) */
    int64_t ent_ld, rel_ld, relw_ld;   /* row strides in elements */
} kge_model_t;

/* Loss of Section 3.1 ("Loss Functions"). */
typedef struct {
    int32_t loss;          /* kge_loss_t */
    float gamma;           /* margin of the log-sigmoid loss */
    float adv_temp;        /* a >= 0, temperature of the self-adversarial weights (StopGrad) */
    float loss_scale;      /* the micro-batch loss is loss_scale * sum_b L_b; <= 0 selects 1/B */
    int64_t n_ent_for_c;   /* |E| in the sampled-softmax correction c = log((|E|-1)/N) */
    float reg_l3;          /* lambda_S >= 0 of Section 3.1 "Regularisation": reg_l3 * Omega_S is added to the
                              loss (NOT scaled by loss_scale), Omega_S = sum over the 2B+N gathered entity slots
                              of the L3 norm (sum_j |x_j|^3)^(1/3) of the slot's embedding row; 0 = off */
    int32_t reserved;      /* 0 */
} kge_loss_cfg_t;

typedef struct {
    float lr, beta1, beta2, eps;
    int64_t step;          /* global 1-based step used in the bias corrections */
    const uint64_t *step_counter;   /* NULL, or a DEVICE counter (kge_step_counter_add): the kernels then use
                                       step + *step_counter, read when they run, so that a captured update
                                       can be replayed step after step */
} kge_adam_cfg_t;

/*
 * Shared negative ids (Section 4, "Training", eq. (negsamples): one set of corrupted tails per
 * micro-batch): out_idx[i], i < n, i.i.d. uniform in [lo, hi), with replacement, no filtering.
 * Counter-based Philox4x32-10: key = (seed_lo, seed_hi); block k = i/2 has counter
 * (k_lo, k_hi, step, stream_tag) and yields two ids from its words (w1:w0) and (w3:w2);
 * id = lo + floor(x * (hi - lo) / 2^64).  Bit-exact, no hidden state.  step < 2^32.
 * out_idx: device int32[n].  Per-partition draws (N/D ids from each shard E_j) are D calls with
 * the shard's [lo, hi).
 */
int kge_sample_negatives(uint64_t seed, uint64_t step, uint32_t stream_tag, int64_t lo, int64_t hi,
                         int64_t n, int32_t *out_idx, void *hip_stream);

/*
 * Steps replayed from a HIP graph.  A graph fixes every kernel argument when it is captured; of the training step
 * (Section 4, "Training": sample, gather, score, update) two numbers change from one step to the next - the step word of
 * the negatives' Philox counter and the step of Adam's bias corrections.  Both can be read from a uint64 in DEVICE
 * memory instead: kge_sample_negatives_dev uses step_offset + *step_counter (same ids as kge_sample_negatives with that
 * step; the caller keeps the sum below 2^32), kge_adam_cfg_t.step_counter does the same for the updates, and
 * kge_step_counter_add enqueues *step_counter += inc (one thread; typically the last node of the captured step).
 * The counter is the caller's memory; the caller sets its first value (e.g. with a copy before the first replay).
 */
int kge_step_counter_add(uint64_t *step_counter, uint64_t inc, void *hip_stream);
int kge_sample_negatives_dev(uint64_t seed, const uint64_t *step_counter, uint64_t step_offset, uint32_t stream_tag,
                             int64_t lo, int64_t hi, int64_t n, int32_t *out_idx, void *hip_stream);

/*
 * Scores of a micro-batch (Table 2; negative sharing per eq. (negsamples)):
 *   pos_out[b]       = f(h_b, r_b, t_b)           b < B          (float[B], or NULL)
 *   neg_out[b*N + n] = f(h_b, r_b, neg_n)         n < N          (float[B*N] row-major, or NULL)
 * h, r, t: int32[B]; neg: int32[N] (may be NULL when N = 0).  B = 0 or N = 0 are valid.
 * Arithmetic: bf16 tables -> bf16 matrix cores with fp32 accumulation (queries are rounded to bf16
 * after the query build).  fp32 tables -> the positive scores by direct fp32 sums; the block, for rows
 * padded to 128 or 256 dimensions (dim <= 256), from TWO fp16 pieces of every operand row scaled by a
 * power of two of its own (22 significand bits, three fp16 matrix products per fp32 one, fp32
 * accumulation; the error of a contraction stays below 3 x 2^-22 |q| |t| whatever the magnitude of the
 * tables), entries of a distance scorer whose norm expansion cancels being redone by direct fp32
 * differences.
 */
int kge_score(const kge_model_t *model, const int32_t *h, const int32_t *r, const int32_t *t,
              int64_t B, const int32_t *neg, int64_t N, float *pos_out, float *neg_out, void *ws,
              size_t ws_bytes, void *hip_stream);

/*
 * Forward + backward of one micro-batch (losses of Section 3.1; the shared negative block is
 * never written to memory):
 *   loss_out      float[1]           loss_scale * sum_b L_b + reg_l3 * Omega_S
 *   g_ent         float[(2B+N) * d]  gradient rows, one per gathered entity slot, in the order
 *                                    heads (B), positive tails (B), shared negatives (N);
 *                                    duplicates are NOT merged (kge_sparse_adam does that)
 *   g_ent_idx     int32[2B+N]        the table row each slot targets (= h, t, neg concatenated)
 *   g_rel         float[B * rel_dim] gradient of each triple's relation row
 *   g_relw        float[B * d]       TransH only (NULL otherwise)
 *   g_rel_idx     int32[B]           = r
 * The sub-gradient of a distance score at distance 0 is 0.  TransH rows of more than 512 bytes (Table 3 lists
 * TransH at d = 256, 1,024 bytes in fp32) take the route of the 1-norm variants: the score block is written to the
 * workspace (B*N floats, three of them) and both passes run on the vector pipe in fp32, about ten times slower than the
 * matrix-core route of the narrower rows.
 * Arithmetic of the two contractions per pass (scores; gradient rows): bf16 tables -> bf16 matrix cores with fp32
 * accumulation.  fp32 tables -> every operand value as three bf16 pieces x0 + x1 + x2 (round to nearest at each step:
 * 24 significand bits, the exponent range of fp32, nothing scaled) and the six piece products of total order <= 2 on
 * the bf16 matrix cores with fp32 accumulation (what is dropped is below 2^-26 |a| |b| per product); the pass over the
 * queries with rows of 1,024 bytes uses the fp32 matrix instructions.
 */
int kge_loss_bwd(const kge_model_t *model, const kge_loss_cfg_t *cfg, const int32_t *h,
                 const int32_t *r, const int32_t *t, int64_t B, const int32_t *neg, int64_t N,
                 float *loss_out, float *g_ent, int32_t *g_ent_idx, float *g_rel, float *g_relw,
                 int32_t *g_rel_idx, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * kge_loss_bwd that draws its shared negatives itself (Section 4, "Training": sample, gather, score, update; the draw of
 * eq. (negsamples) joins the gather of the rows it selects: one launch less per step, and the gather does not wait for
 * ids from memory).  The ids are those of kge_sample_negatives(seed, step, stream_tag, lo, hi, N) - with step_counter
 * set, those of kge_sample_negatives_dev(seed, step_counter, step, ...) - bit for bit.  They are written to neg_out
 * (device int32[N], required when N > 0) and are complete when the call's work is: a kge_sparse_adam_plan* that sorts
 * them comes after this call on the stream.  Everything else as kge_loss_bwd with neg = neg_out.
 */
typedef struct {
    uint64_t seed;
    uint64_t step;                    /* < 2^32 (with step_counter: step + *step_counter < 2^32) */
    const uint64_t *step_counter;     /* NULL, or a DEVICE counter as in kge_sample_negatives_dev */
    uint32_t stream_tag;
    uint32_t reserved;                /* 0 */
    int64_t lo, hi;                   /* ids in [lo, hi), 0 <= lo < hi <= 2^31 */
} kge_neg_draw_t;
int kge_loss_bwd_sampled(const kge_model_t *model, const kge_loss_cfg_t *cfg, const int32_t *h,
                         const int32_t *r, const int32_t *t, int64_t B, const kge_neg_draw_t *draw, int32_t *neg_out,
                         int64_t N, float *loss_out, float *g_ent, int32_t *g_ent_idx, float *g_rel, float *g_relw,
                         int32_t *g_rel_idx, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Duplicate-aware scatter-add + lazy sparse Adam on the touched rows only (Section 1: only the
 * rows of the mini-batch are accessed and updated; optimiser state lives beside the rows,
 * Section 4.1).  grads[i*dim .. ] (float, i < M) targets table row idx[i]; rows with equal idx
 * are summed first (sort by row, then a fixed-order segmented reduction: results do not depend
 * on scheduling), then each touched row takes ONE Adam step with the global step:
 *   m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;
 *   theta <- theta - lr * (m / (1-b1^step)) / (sqrt(v / (1-b2^step)) + eps)
 * Untouched rows and their moments are not read or written.
 *   param_f32   float[n_rows, ld]   master weights (updated in place)
 *   param_bf16  bf16 [n_rows, ld]   optional shadow copy, rewritten as RNE(theta) for touched rows
 *   m, v        float[n_rows, ld]   Adam moments (updated in place)
 * dim and ld must be multiples of 4, param_f32, m, v and grads 16-byte aligned, param_bf16 8-byte aligned (the update
 * moves four columns at a time; KGE_E_INVALID_ARG otherwise).  M = 0 is valid (no-op).  This is the only call that
 * writes a table.
 */
int kge_sparse_adam(float *param_f32, void *param_bf16, float *m, float *v, int64_t n_rows,
                    int32_t dim, int64_t ld, const int32_t *idx, const float *grads, int64_t M,
                    const kge_adam_cfg_t *cfg, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * The same update in two calls, so that the part that needs only the row ids can run while the gradients are
 * still being computed (the ids of a step - h, t and the negatives - are known before the forward pass;
 * Section 4 overlaps communication and compute in the same spirit): kge_sparse_adam_plan sorts (idx, position)
 * into the workspace; kge_sparse_adam_apply reduces the gradient rows of equal ids and takes the Adam step,
 * reading the plan from the SAME workspace (same M, n_rows and dim; nothing else may use that workspace in
 * between; the caller orders the two calls, e.g. with an event when they run on different streams).
 * kge_sparse_adam(...) == plan(...) followed by apply(...), bit for bit.  Workspace size:
 * kge_workspace_bytes(KGE_OP_SPARSE_ADAM, NULL, M, dim, 0).
 */
int kge_sparse_adam_plan(int64_t n_rows, int32_t dim, const int32_t *idx, int64_t M, void *ws, size_t ws_bytes,
                         void *hip_stream);
int kge_sparse_adam_apply(float *param_f32, void *param_bf16, float *m, float *v, int64_t n_rows, int32_t dim,
                          int64_t ld, const float *grads, int64_t M, const kge_adam_cfg_t *cfg, void *ws,
                          size_t ws_bytes, void *hip_stream);

/*
 * kge_sparse_adam_apply for several tables at once: a training step updates the entity table and one or two small
 * relation tables (Section 3.1: relation embeddings, TransH's normals), and a small table alone costs two launches for
 * a few microseconds of work.  Each table has been planned with kge_sparse_adam_plan into its own workspace; the
 * result equals one kge_sparse_adam_apply per table, bit for bit, in two launches for all of them.  1 <= n_tables <= 4;
 * the tables must not overlap; tables with M = 0 are skipped.
 */
typedef struct {
    int64_t n_rows; int32_t dim; const int32_t *idx; int64_t M;   /* as in kge_sparse_adam_plan */
    void *ws; size_t ws_bytes;
} kge_adam_plan_t;
/* kge_sparse_adam_plan for several tables (1 <= n_tables <= 4), each into its own workspace; the sorts of up to 32,768 ids
 * share one launch.  Same result in every workspace as one kge_sparse_adam_plan per table. */
int kge_sparse_adam_plan_tables(const kge_adam_plan_t *plans, int32_t n_tables, void *hip_stream);

/*
 * kge_loss_bwd_sampled and kge_sparse_adam_plan_tables in one call (Section 4, "Training": one step = sample, gather, score,
 * update).  The sorts of a step's row ids need the ids alone, so the call puts them where they cost least: with the sampled
 * softmax on bilinear bf16 rows of 512 bytes they share the launch that finishes the rows' losses between the two block
 * passes (one launch less per step, and the finish passes under the sorts); in every other configuration they follow the
 * call's other work.  Results - losses, gradients, ids, and every plan in its workspace - equal those of the two calls, bit
 * for bit.  plans[k].idx must be complete when the call starts, or be neg_out, or an array that ends in neg_out (e.g. one
 * buffer [h | t | neg_out]); g_ent_idx and g_rel_idx, which the call writes last, are rejected (KGE_E_INVALID_ARG).
 * Other errors as the two calls.
 */
int kge_loss_bwd_sampled_planned(const kge_model_t *model, const kge_loss_cfg_t *cfg, const int32_t *h,
                                 const int32_t *r, const int32_t *t, int64_t B, const kge_neg_draw_t *draw,
                                 int32_t *neg_out, int64_t N, float *loss_out, float *g_ent, int32_t *g_ent_idx,
                                 float *g_rel, float *g_relw, int32_t *g_rel_idx, void *ws, size_t ws_bytes,
                                 const kge_adam_plan_t *plans, int32_t n_tables, void *hip_stream);

typedef struct {
    float *param_f32; void *param_bf16; float *m, *v;      /* as in kge_sparse_adam */
    int64_t n_rows; int32_t dim; int64_t ld;
    const float *grads; int64_t M;
    void *ws; size_t ws_bytes;                             /* the workspace that kge_sparse_adam_plan filled */
} kge_adam_table_t;
int kge_sparse_adam_apply_tables(const kge_adam_table_t *tables, int32_t n_tables, const kge_adam_cfg_t *cfg,
                                 void *hip_stream);

/*
 * kge_sparse_adam for callers that cannot allocate device memory and have no workspace to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (minus the workspace), same kernels
 * and the same bits as kge_sparse_adam; the sort buffers and piece sums live in a buffer built into the library
 * (static device memory, kge_sparse_adam_static_limit() bytes = 4 MiB, one copy per GPU, held until the process ends).
 * The call allocates and frees nothing (the profiling hooks, off by default, create HIP events while they are on).
 * Limit: kge_workspace_bytes(KGE_OP_SPARSE_ADAM, NULL, M, dim, 0) <= kge_sparse_adam_static_limit() -- e.g. M = 24,576
 * rows of dim 256, or M = 65,536 of dim 64 -- else KGE_E_STATIC_SCRATCH_TOO_SMALL and nothing is launched.
 * Every call on a GPU shares that GPU's buffer: calls that overlap on one GPU (two streams, two threads) race; order
 * them on one stream or with events.  Nothing in the buffer needs clearing between calls (every word a call reads it
 * has written itself), so calls of any sizes may follow each other.
 */
int kge_sparse_adam_static(float *param_f32, void *param_bf16, float *m, float *v, int64_t n_rows, int32_t dim,
                           int64_t ld, const int32_t *idx, const float *grads, int64_t M,
                           const kge_adam_cfg_t *cfg, void *hip_stream);
size_t kge_sparse_adam_static_limit(void);

/*
 * Link prediction (Section 3.2, "Inference"): for each query (h_q, r_q), q < Q, rank all
 * candidate tails t in [cand_lo, cand_hi) and return the K best by (score descending, index
 * ascending):  out_idx int32[Q*K], out_score float[Q*K].  If K exceeds the number of candidates
 * the tail of each list is padded with index -1 and score -inf.  The candidate range is the
 * single-GPU image of "score against the local shard E_i"; D shard-wise lists merge to the global
 * top-K (Section 4, "Inference").
 * Exactness: candidates are pre-selected with matrix-core scores, the survivors are re-scored with
 * a sequential fp64 loop (the direct formula of Table 2, every operation rounded on its own; DistMult
 * and TransE with one fused multiply-add per column) and ordered by that key, and a rigorous error bound
 * checks that no candidate outside the pre-selection could belong to the top-K; queries that fail
 * the check are re-ranked by an exhaustive fp64 scan.  The returned indices therefore equal the
 * ordering by the fp64 key exactly.
 * true_t int32[Q] / out_rank int64[Q] (both or neither): 1-based rank of the held-out tail among
 * the candidates.  Exact whenever rank <= K (it is the list position); beyond K it is counted
 * with the matrix-core scores and may differ from the fp64 rank by the number of candidates whose
 * score lies within the rounding error of the true tail's score.
 * Scorers: DistMult, ComplEx, TransE, RotatE and TransH with p_norm = 2 (p_norm = 1, and TransH rows longer than
 * 512 bytes: KGE_E_UNSUPPORTED).  The rows of the entity table must start 16-byte aligned (model->ent and
 * ent_ld * sizeof(element) multiples of 16; else KGE_E_UNSUPPORTED): the scan copies them straight from the table.
 * kge_score and kge_loss_bwd take any row stride >= dim.
 * RotatE's key passes through cos / sin of the phases in fp64: its last bit is the math library's.  TransH's key
 * is |q' - t + (u.t) u|^2 with u = w / max(|w|, 1e-12) and q' = (h - (u.h) u) + r made once per query in fp64
 * (wave-wide sums), then u.t and the squared distance by sequential fused multiply-adds over the columns; it
 * needs 16 d more workspace bytes per query.
 * 1 <= K <= 256.
 */
int kge_topk(const kge_model_t *model, const int32_t *h, const int32_t *r, int64_t Q,
             int64_t cand_lo, int64_t cand_hi, int32_t K, int32_t *out_idx, float *out_score,
             const int32_t *true_t, int64_t *out_rank, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Power-rank ensemble (Section 3.2 "Inference", paragraph "Ensemble", eq. (ensemble)): combines the top-K lists
 * of M models.  lists int32[M*Q*K] (device), lists[(m*Q + q)*K + k-1] = the k-th best tail of model m for query
 * q, e.g. M outputs of kge_topk; entries < 0 pad a short list; an entity that a list holds twice counts at its
 * first position.  With power p != 0 every entity t scores
 *     s(t) = sum over m (in model order, fp64) of  -sgn(p) k^p           if t is the k-th entry of list m,
 *                                                   -[p > 0] (K + 1)^p    if list m does not hold t,
 * (p = -1: reciprocal-rank fusion; p = 1: minus the sum of the ranks) and the K_out entities with the largest
 * s(t), ties to the smaller id, go to out_idx int32[Q*K_out] / out_score float[Q*K_out] (padded with -1 / -inf
 * when fewer entities are listed).  Only listed entities compete: an unlisted one has the smallest possible
 * score.  The K + 1 possible terms are evaluated with the host's pow().
 * Limits: M <= 128, K <= 256, M*K <= 8192 (KGE_E_UNSUPPORTED beyond), 1 <= K_out <= 256, 0 < |p| <= 64.
 * Needs no workspace.
 */
int kge_ensemble(const int32_t *lists, int32_t M, int64_t Q, int32_t K, double p, int32_t K_out,
                 int32_t *out_idx, float *out_score, void *hip_stream);

/*
 * Partition bucketing (Section 4, "Partitioning"): entity e belongs to shard e / part_size
 * (part_size = ceil(|E|/D), ids assumed already randomly permuted); triple i falls in bucket
 * (h_i / part_size) * D + (t_i / part_size).  Outputs a stable counting sort by bucket:
 *   bucket_offsets int64[D*D + 1]   exclusive prefix sums of the bucket sizes
 *   order          int64[n]         order[k] = input position of the k-th triple in bucket order;
 *                                   triples of one bucket keep their input order
 * D <= 64.
 */
int kge_partition_triples(const int32_t *h, const int32_t *t, int64_t n, int64_t part_size,
                          int32_t D, int64_t *bucket_offsets, int64_t *order, void *ws,
                          size_t ws_bytes, void *hip_stream);

/*
 * Relation-aware triple sampler (Section 4, "Training"): the triples of a micro-batch part B_ij are
 * drawn with replacement from partition bucket T_ij with
 *     p((h, r, t)) = (1 / n_r) * cbrt(n_r) / sum_r' cbrt(n_r'),   n_r = triples of relation r in T_ij,
 * i.e. first a relation by the cube root of its frequency in the bucket, then one of its triples uniformly.
 *
 * kge_sampler_build (one-off) indexes the triples: a stable sort by (bucket, relation), bucket as in
 * kge_partition_triples, giving
 *   order        int64[n]                 input position of the k-th triple of the sorted list
 *   rel_offsets  int64[D*D*n_rel + 1]     first sorted position of every (bucket, relation) group
 *   cdf          uint64[D*D*n_rel]        inclusive prefix sums, inside each bucket, of the integer weights
 *                                         w(n_r) = floor(2^20 * n_r^(1/3)) (exact: the largest integer whose
 *                                         cube is <= n_r * 2^60), so every implementation draws alike
 * n < 2^31, D <= 64, D*D*n_rel < 2^31.
 *
 * kge_sample_triples draws n_buckets * per_bucket triples: draw q comes from bucket
 * bucket_lo + q / per_bucket.  One worker's micro-batch of eq. (microbatch) is bucket_lo = i*D,
 * n_buckets = D, per_bucket = B/D; a single partition pair is n_buckets = 1.  Philox4x32-10, key = seed,
 * counter (q_lo, q_hi, step, stream_tag): x = w1:w0 selects the first relation whose cdf exceeds
 * floor(x * total / 2^64), y = w3:w2 the triple floor(y * n_r / 2^64) of that group.  Bit-exact, no state.
 * Outputs (device; any of out_pos and the out_h/out_r/out_t triple may be NULL): out_pos int64[draws] =
 * position in the triple arrays, out_h/out_r/out_t int32[draws] = the triple itself (needs h, r, t).
 * Draws from an empty bucket give -1.
 *
 * kge_sample_negatives_sharded: the shared negatives of eq. (negsamples), per_shard ids from every
 * entity shard E_j = [j*part_size, min(n_ent, (j+1)*part_size)); slot i belongs to shard i / per_shard and
 * uses the generator block of slot i of kge_sample_negatives.  out_idx: device int32[D * per_shard].
 */
int kge_sampler_build(const int32_t *h, const int32_t *r, const int32_t *t, int64_t n, int64_t part_size,
                      int32_t D, int64_t n_rel, int64_t *order, int64_t *rel_offsets, uint64_t *cdf,
                      void *ws, size_t ws_bytes, void *hip_stream);
int kge_sample_triples(uint64_t seed, uint64_t step, uint32_t stream_tag, int64_t bucket_lo,
                       int64_t n_buckets, int64_t per_bucket, int32_t D, int64_t n_rel,
                       const int64_t *rel_offsets, const uint64_t *cdf, const int64_t *order,
                       const int32_t *h, const int32_t *r, const int32_t *t, int64_t *out_pos,
                       int32_t *out_h, int32_t *out_r, int32_t *out_t, void *hip_stream);
int kge_sample_negatives_sharded(uint64_t seed, uint64_t step, uint32_t stream_tag, int64_t part_size,
                                 int64_t n_ent, int32_t D, int64_t per_shard, int32_t *out_idx,
                                 void *hip_stream);

/*
 * Feature-projection encoder (Section 3.1 "Encoder", eq. (embedding)): the final embedding of an entity is
 *     e = e_S + M_H e_F  as a head,    e = e_S + M_T e_F  as a tail,
 * e_S the trainable shallow row, e_F the entity's fixed text-feature row, M_H, M_T trainable [dim, feat_dim]
 * projections (they may alias).  Dropout with probability `dropout` acts on the projection before the sum,
 * and the L3 norms of e, e_S and M e_F are regularised with weights reg_t, reg_s, reg_f (Section 3.1
 * "Regularisation").  Dropout mask of element (slot, column): Philox4x32-10, key = seed, counter
 * (slot, column / 4, step, dropout_tag), word column % 4; kept iff word >= floor(dropout * 2^32), then
 * scaled by 1 / (1 - dropout).
 *
 * kge_encode works on the 2B + N gathered slots of a micro-batch in the order heads (B, M_H), positive tails
 * (B, M_T), shared negatives (N, M_T) and writes
 *   e_out     [(2B+N), dim] in the encoder's dtype, row stride dim: a compact entity table for kge_score /
 *             kge_loss_bwd with h = 0..B-1, t = B..2B-1, neg = 2B..2B+N-1
 *   proj_out  float[(2B+N) * dim]  the projections M e_F (before dropout); kge_encode_bwd takes them back
 *   reg_out   float[1] (may be NULL) reg_t sum ||e||_3 + reg_s sum ||e_S||_3 + reg_f sum ||M e_F||_3
 * kge_encode_bwd takes de = float[(2B+N) * dim], the gradient of the loss with respect to e_out's rows (the
 * g_ent of kge_loss_bwd on the compact table), and writes
 *   g_es      float[(2B+N) * dim]  gradient rows of the shallow embeddings, one per slot (target rows: h, t, neg;
 *             duplicates not merged - kge_sparse_adam does that), regulariser terms included
 *   g_mh, g_mt float[dim * feat_dim] dense gradients of M_H and M_T (add them when the two alias)
 * With bf16 tables the projections run on the bf16 matrix cores with fp32 accumulation, and the backward
 * contraction rounds its left operand to bf16.  Limits: dim <= 512, feat_dim <= 1024, both multiples of 16
 * (bf16) / 8 (fp32); rows of feat, m_h, m_t 16-byte aligned.  step < 2^32.
 */
typedef struct {
    int32_t dtype;         /* kge_dtype_t of ent_s, feat, m_h, m_t as the kernels read them */
    int32_t dim;           /* d */
    int32_t feat_dim;      /* |e_F| (768 in the paper) */
    uint32_t dropout_tag;  /* stream tag of the dropout generator */
    int64_t n_ent;
    const void *ent_s;     /* [n_ent, ent_ld] */
    const void *feat;      /* [n_ent, feat_ld] */
    const void *m_h, *m_t; /* [dim, m_ld] */
    int64_t ent_ld, feat_ld, m_ld;
    float dropout;         /* in [0, 1) */
    float reg_t, reg_s, reg_f;
} kge_encoder_t;

int kge_encode(const kge_encoder_t *enc, const int32_t *h, const int32_t *t, int64_t B, const int32_t *neg,
               int64_t N, uint64_t seed, uint64_t step, void *e_out, float *proj_out, float *reg_out,
               void *ws, size_t ws_bytes, void *hip_stream);
int kge_encode_bwd(const kge_encoder_t *enc, const int32_t *h, const int32_t *t, int64_t B,
                   const int32_t *neg, int64_t N, uint64_t seed, uint64_t step, const float *proj,
                   const float *de, float *g_es, float *g_mh, float *g_mt, void *ws, size_t ws_bytes,
                   void *hip_stream);
/* Workspace of the two calls above (op = KGE_OP_ENCODE or KGE_OP_ENCODE_BWD); 0 for invalid arguments. */
size_t kge_encode_workspace_bytes(int op, const kge_encoder_t *enc, int64_t B, int64_t N);

/*
 * Workspace size in bytes for one call (pure function; host only).  Meaning of (B, N, K):
 *   KGE_OP_SCORE, KGE_OP_LOSS_BWD  B triples, N shared negatives, K unused
 *   KGE_OP_SPARSE_ADAM             B = M gradient rows, N = dim, K unused; model may be NULL
 *   KGE_OP_TOPK                    B = Q queries, N = number of candidates, K
 *   KGE_OP_PARTITION               B = n triples, N = D; model may be NULL
 *   KGE_OP_SAMPLER_BUILD           B = n triples, N = D; model may be NULL
 *   KGE_OP_ENCODE, KGE_OP_ENCODE_BWD  see kge_encode_workspace_bytes (these two take a kge_encoder_t)
 * Returns 0 for an invalid request.
 */
size_t kge_workspace_bytes(int op, const kge_model_t *model, int64_t B, int64_t N, int64_t K);

/*
 * Optional instrumentation for benchmarks: while enabled, the library brackets the launches of its
 * dominant kernels with HIP events on the caller's stream.  kge_profile_enable(on): 0 switches it off,
 * a negative value instruments every slot, a positive value is a bit mask (bit s = slot s; two event
 * records per instrumented launch cost host time, so a timed run may want the slot it reports only).
 * kge_profile_collect() waits for the recorded events of one slot, returns their summed duration and
 * count, and forgets them.
 * Host-side state shared by all callers of the process; not thread-safe; off by default.
 */
enum { KGE_PROF_BLOCK_SCORE = 0, KGE_PROF_BLOCK_FWD = 1, KGE_PROF_BLOCK_GRADT = 2, KGE_PROF_ADAM = 3,
       KGE_PROF_SORT = 4, KGE_PROF_TOPK_SCAN = 5, KGE_PROF_ENC_FWD = 6, KGE_PROF_ENC_BWD = 7,
       KGE_PROF_GATHER = 8,   /* kge_loss_bwd: query build + gather of the negatives' rows (one launch) */
       KGE_PROF_FINISH = 9,   /* kge_loss_bwd: chain rule of the queries + finish of the negatives' gradient rows (one launch) */
       KGE_PROF_SLOTS = 10 };
int kge_profile_enable(int on);
int kge_profile_collect(int slot, double *total_ms, int64_t *launches);

/*
 * Measured figures of the GPU for benchmarks that quote rooflines (not part of the method; each runs its kernel
 * twice on the given stream, times the second run with HIP events and SYNCHRONISES the stream before it returns):
 * kge_calibrate_mfma: the rate, in TFLOP/s, of 2,048 workgroups of 8 waves that each issue 4 x iters independent
 *   bf16 matrix instructions (32 x 32 x 16) on constant operands; sink: device memory of at least 2,048 x 512 floats
 *   (sink_elems says how many) that takes one value per lane; iters in [1, 2^20].
 * kge_calibrate_mfma_varied: the same loop on operands whose signs and mantissas differ from element to element, as
 *   those of embedding tables do (the chip lowers its clock with the number of bits that toggle; the sums stay finite).
 * kge_calibrate_copy: the rate, in GB/s read + written, of a plain 16-byte-per-lane copy of `bytes` bytes from src to dst
 *   (device memory, 16-byte aligned, bytes a multiple of 16, ranges must not overlap).
 * Errors: KGE_E_INVALID_ARG (nothing is launched), KGE_E_HIP.
 */
int kge_calibrate_mfma(int32_t iters, float *sink, int64_t sink_elems, double *tflops_out, void *hip_stream);
int kge_calibrate_mfma_varied(int32_t iters, float *sink, int64_t sink_elems, double *tflops_out, void *hip_stream);
int kge_calibrate_copy(const void *src, void *dst, size_t bytes, double *gbs_out, void *hip_stream);

/*
 * For tests and benchmarks that compare two kernels of one job: every job has one kernel in the library's own dispatch;
 * kge_debug_select(knob, 1) makes later calls of the whole process take the alternative, kge_debug_select(knob, 0)
 * returns to the library's choice.  Not for production use: the alternatives are slower, and a workspace must be sized
 * (kge_workspace_bytes) under the same setting as the call that uses it.
 *   KGE_DEBUG_FWD_ONE_ROLE    the pass over the queries of kge_loss_bwd (bf16, rows <= 512 bytes) as the one-role kernel
 *   KGE_DEBUG_GRADT_ONE_ROLE  the same for the pass over the negatives
 *   KGE_DEBUG_SCORE_F32_MFMA  kge_score on fp32 tables with the fp32 matrix instructions instead of two fp16 planes
 *   KGE_DEBUG_TWO_ROLE        both of those passes as the two-role kernels (the forward one is also what redoes a pass
 *                             whose scores outgrow the fixed reference exponent of the default kernel)
 *   KGE_DEBUG_GRADT_RECOMPUTE the pass over the negatives recomputes the scores also where the forward pass has kept its
 *                             weights for it (sampled softmax, bilinear scorers, bf16 rows of 512 bytes)
 * Returns KGE_E_INVALID_ARG for an unknown knob or a value other than 0 / 1.
 */
enum { KGE_DEBUG_FWD_ONE_ROLE = 0, KGE_DEBUG_GRADT_ONE_ROLE = 1, KGE_DEBUG_SCORE_F32_MFMA = 2, KGE_DEBUG_TWO_ROLE = 3,
       KGE_DEBUG_GRADT_RECOMPUTE = 4 };
int kge_debug_select(int knob, int value);

/* Static description of a status code. */
const char *kge_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* KGE_H_ */
