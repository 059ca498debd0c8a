// Host-side launchers of the row-wise kernels (implemented in prep_kernels.hip).
#pragma once
#include "kge_internal.h"

// Device-side view of kge_model_t.
struct KgeModelDev {
    int32_t scorer, bf16, dim, rel_dim;
    int32_t p1;                    // distance scorers: 1 = the 1-norm variant (Table 2, p = 1)
    int32_t vec;                   // the block passes ran on the vector pipe (1-norm; TransH rows over 512 bytes): their
                                   // partials are finished gradient rows
    const void *ent, *rel, *relw;
    int64_t ent_ld, rel_ld, relw_ld;
};

int kge_run_negatives(uint64_t seed, uint64_t step, const uint64_t *step_counter, uint32_t tag, int64_t lo, int64_t hi,
                      int64_t n, int32_t *out, hipStream_t st);
int kge_run_step_counter_add(uint64_t *counter, uint64_t inc, hipStream_t st);
int kge_run_qbuild(const KgeModelDev &m, const int32_t *h, const int32_t *r, const int32_t *t, int B, int Bp,
                   int dp, void *Q, void *W, void *Q2, float *Q32, float *W32, KgeRowInfo *rowinfo, float *pos_ws,
                   float *pos_out, hipStream_t st, void *planes = nullptr);
// planes (fp32 tables only, optional): also the two fp16 pieces of every element of the rows scaled by a power of two,
// [2][rows][dp], and 1 / scale of every row in inv_scale
constexpr float KGE_PLANE_UNIT_SCALE = 1024.f;      // scale of the planes of TransH's unit normals (all rows)
int kge_run_tgather(const KgeModelDev &m, const int32_t *neg, int N, int Np, int dp, void *T, float *tn,
                    hipStream_t st, void *planes = nullptr, float *inv_scale = nullptr);
// The draw of kge_run_negatives for a gather that makes it itself: id n of (seed, step [+ *step_counter], tag) in
// [lo, lo + range), written to out[n] as it is used.  out == nullptr: the gather reads its ids.
struct KgeNegGen { int32_t *out; uint32_t seed_lo, seed_hi, step, tag; const uint64_t *step_counter; int64_t lo; uint64_t range; };
// the two above as ONE launch (Bp > 0 and Np > 0; no positive scores out)
int kge_run_qbuild_tgather(const KgeModelDev &m, const int32_t *h, const int32_t *r, const int32_t *t, int B, int Bp,
                           int dp, void *Q, void *W, void *Q2, float *Q32, float *W32, KgeRowInfo *rowinfo, float *pos_ws,
                           const int32_t *neg, int N, int Np, void *T, float *tn, hipStream_t st, float *pos_out = nullptr,
                           void *q_planes = nullptr, void *t_planes = nullptr, float *t_inv_scale = nullptr,
                           float *bias = nullptr,             // bias [Np]: 0 for the N negatives, -inf behind them
                           const KgeNegGen *gen = nullptr);   // gen->out set: neg is ignored, the ids are drawn and written there
// gather of the negatives and their transposed copy Tt [dp][Np] in one launch
int kge_run_tgather_t(const KgeModelDev &m, const int32_t *neg, int N, int Np, int dp, void *T, void *Tt, float *tn,
                      hipStream_t st);
int kge_run_transpose(const void *src, void *dst, int R, int C, bool bf16, hipStream_t st);
// bf16 rows of 256 elements: the finish plus the query rows scaled for every forward split, Qs [nsplit][Bp][256] (block_gradp.hip)
int kge_run_rowfinish_qscale(const float4 *stat_part, int nsplit, int Bp, int B, int N, int loss, float gamma, float c_corr,
                              float scale, const float *pos, KgeRowInfo *rowinfo, float *lossb, float *gpos, const void *Q,
                              void *Qs, hipStream_t st);
int kge_run_rowfinish(const float4 *stat_part, int nsplit, int Bp, int B, int N, int loss, float gamma,
                      float c_corr, float scale, const float *pos, KgeRowInfo *rowinfo, float *lossb,
                      float *gpos, float *loss_out, hipStream_t st);     // loss_out null: the rows' losses are not summed here
// m.vec: acc_part holds finished gradient rows (coefficients already normalised), sum_part / stat_part are not read
int kge_run_chain(const KgeModelDev &m, const int32_t *h, const int32_t *r, const int32_t *t, int B, int Bp, int dp,
                  const float *acc_part, const float *acc_part2, const float4 *sum_part, const float4 *stat_part,
                  const KgeRowInfo *rowinfo, int nsplit, const float *gpos, float *g_ent, float *g_rel,
                  float *g_relw, int32_t *g_ent_idx, int32_t *g_rel_idx, float reg, float *regv, hipStream_t st);
int kge_run_tfinish(const float *accT_part, const float4 *sumT_part, int nsplit, int Np, int N, int dp, int d,
                    int dist_kind, const void *T, bool bf16, const int32_t *neg, float *g_neg, int32_t *g_neg_idx,
                    const void *ent, int64_t ent_ld, float reg, float *regn, hipStream_t st);
// kge_run_chain and kge_run_tfinish as ONE launch (B > 0 and N > 0; the rows of the negatives are read from T or,
// with T == nullptr, from the model's entity table)
int kge_run_chain_tfinish(const KgeModelDev &m, const int32_t *h, const int32_t *r, const int32_t *t, int B, int Bp, int dp,
                          const float *acc_part, const float *acc_part2, const float4 *sum_part, const float4 *stat_part,
                          const KgeRowInfo *rowinfo, int nsplit, const float *gpos, float *g_ent, float *g_rel,
                          float *g_relw, int32_t *g_ent_idx, int32_t *g_rel_idx, float reg, float *regv,
                          const float *accT_part, const float4 *sumT_part, int nsplit_t, int Np, int N, int d, int dist_kind,
                          const void *T, const int32_t *neg, float *g_neg, int32_t *g_neg_idx, float *regn,
                          const float *lossb, float scale, float *loss_out, hipStream_t st, bool part_bf16 = false);   // also loss_out = scale * sum of lossb
// loss_out += reg * (sum of regv over the 2B + N gathered slots), laid out [Bp heads][Bp tails][N negatives]
int kge_run_reg_add(const float *regv, int B, int Bp, int N, float reg, float *loss_out, hipStream_t st);

// 1-norm distance scorers (l1_kernels.hip): score block, row statistics of the loss, gradient rows
int kge_run_l1_score(bool bf16, const float *Q, const void *T, int B, int N, int Bp, int Np, int dp, float *S, int64_t ldS,
                     hipStream_t st);
int kge_run_l1_rowstat(const float *S, int64_t ldS, int B, int N, int Bp, int loss, float gamma, float adv_temp,
                       float4 *stat, hipStream_t st);
int kge_l1_nsplit(int own_pad, int str_pad, int dp, bool transh);
int kge_run_l1_grad(bool bf16, bool own_is_query, const void *own, const void *str, const float *S, int64_t ldS,
                    const KgeRowInfo *rowinfo, int B, int N, int own_pad, int str_pad, int dp, int loss, float gamma,
                    float adv_temp, int nsplit, float *acc_part, hipStream_t st);
// TransH under the 1-norm: Q, W = unrounded queries q' and unit normals [Bp][dp]; A = w^ . t and P = sign(x) . w^ per
// pair beside S (both nullptr: scores only); the pass over the queries also fills acc_part2 with the gradient of w^
int kge_run_l1h_score(bool bf16, const float *Q, const float *W, const void *T, int B, int N, int Bp, int Np, int dp, float *S,
                      float *A, float *P, int64_t ldS, hipStream_t st, int pn = 1);   // pn: the norm (1, or 2 for wide TransH rows)
int kge_run_l1h_grad(bool bf16, bool own_is_query, const float *Q, const float *W, const void *T, const float *S, const float *A,
                     const float *P, int64_t ldS, const KgeRowInfo *rowinfo, int B, int N, int own_pad, int str_pad, int dp,
                     int loss, float gamma, float adv_temp, int nsplit, float *acc_part, float *acc_part2, hipStream_t st,
                     int pn = 1);
