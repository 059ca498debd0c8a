/*
 * kge_oracle.c -- plain, slow CPU reference for the BESS knowledge-graph-embedding hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the correctness oracle: it is called by the test-suite,
 * by the smoke check and by the benchmark's "cpu_baseline" leg, never by the product path, and it
 * shares no code with the GPU library.
 *
 * Everything is evaluated from the printed definitions, in fp64, with direct loops over
 * (triple b, negative n, component j): no factorisation into matrix products, no blocking, no
 * fusion.  OpenMP "parallel for" over batch rows / queries is the only concession to run time.
 * Compile with -ffp-contract=off so that the only fused multiply-adds are the explicit fma()
 * calls of the ranking score.
 *
 * Sources followed (paper = arXiv 2211.12281):
 *   scores            Table 2 (scoring functions), p = 2
 *   losses            Section 3.1, "Loss Functions": log-sigmoid with self-adversarial weights,
 *                     sampled softmax cross-entropy with correction c = log((|E|-1)/N)
 *   negative sharing  Section 4, "Training", eq. (negsamples): one set of corrupted tails per
 *                     micro-batch, used by every triple of it
 *   sparse update     Section 1 (only the rows of the mini-batch are accessed and updated);
 *                     optimiser = Adam with "lazy" sparse semantics (the paper names none)
 *   ranking           Section 3.2, "Inference": top-K of {f(h,r,t) : t in E}; heap, O(|E| log K)
 *   partitioning      Section 4, "Partitioning": equal row shards E_1..E_D, triple buckets T_ij
 *   negative ids      Philox4x32-10 (Salmon et al., SC'11), counter-based, integer multiply-shift
 *
 * Parity pins: every function below is pinned by tests/test_oracle_*.py (closed forms, reductions
 * between scorers, finite differences, torch CPU optimisers, brute-force sorting, an independent
 * big-integer Philox; the 1-norm scorers against numpy's 1-norm of independently built difference
 * vectors, norm-equivalence bounds, the kink's sub-gradient).  Nothing here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_TRANSE = 0, ORC_TRANSH = 1, ORC_ROTATE = 2, ORC_DISTMULT = 3, ORC_COMPLEX = 4,
       /* the distance scorers with the 1-norm (Table 2: p in {1, 2}) */
       ORC_TRANSE_L1 = 5, ORC_TRANSH_L1 = 6, ORC_ROTATE_L1 = 7 };

static int orc_is_l1(int scorer) { return scorer >= ORC_TRANSE_L1 && scorer <= ORC_ROTATE_L1; }
static int orc_base_scorer(int scorer)
{
    return scorer == ORC_TRANSE_L1 ? ORC_TRANSE : scorer == ORC_TRANSH_L1 ? ORC_TRANSH
         : scorer == ORC_ROTATE_L1 ? ORC_ROTATE : scorer;
}
/* sub-gradient of |x|: 0 at the kink */
static double orc_sign(double x) { return (double)(x > 0.0) - (double)(x < 0.0); }
enum { ORC_LOGSIGMOID = 0, ORC_SAMPLED_SOFTMAX = 1 };

/* ------------------------------------------------------------------------------------------ */
/* Philox4x32-10                                                                              */
/* ------------------------------------------------------------------------------------------ */

static void orc_mulhilo32(uint32_t a, uint32_t b, uint32_t *hi, uint32_t *lo)
{
    uint64_t p = (uint64_t)a * (uint64_t)b;
    *hi = (uint32_t)(p >> 32);
    *lo = (uint32_t)p;
}

/* One block: 4 counter words, 2 key words -> 4 output words, 10 rounds. */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint32_t hi0, lo0, hi1, lo1;
        orc_mulhilo32(0xD2511F53u, c0, &hi0, &lo0);
        orc_mulhilo32(0xCD9E8D57u, c2, &hi1, &lo1);
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Exposes a single round for the hand-computed pin. */
void orc_philox_single_round(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t hi0, lo0, hi1, lo1;
    orc_mulhilo32(0xD2511F53u, ctr[0], &hi0, &lo0);
    orc_mulhilo32(0xCD9E8D57u, ctr[2], &hi1, &lo1);
    out[0] = hi1 ^ ctr[1] ^ key[0];
    out[1] = lo1;
    out[2] = hi0 ^ ctr[3] ^ key[1];
    out[3] = lo0;
}

/*
 * Shared negative ids (eq. (negsamples): a set N_i of corrupted tails per micro-batch; drawn
 * i.i.d. uniform with replacement over [lo, hi)).
 * Block k of the stream has counter (k_lo, k_hi, step, tag) and key (seed_lo, seed_hi); it yields
 * two ids: id #2k from words (w1:w0), id #2k+1 from words (w3:w2); each 64-bit word x maps to
 * lo + floor(x * (hi - lo) / 2^64).
 */
void orc_sample_negatives(uint64_t seed, uint64_t step, uint32_t tag, int64_t lo, int64_t hi,
                          int64_t n, int32_t *out)
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint64_t range = (uint64_t)(hi - lo);
    for (int64_t i = 0; i < n; ++i) {
        uint64_t block = (uint64_t)i / 2;
        uint32_t ctr[4] = { (uint32_t)block, (uint32_t)(block >> 32), (uint32_t)step, tag };
        uint32_t w[4];
        orc_philox4x32_10(ctr, key, w);
        int half = (int)(i & 1);
        uint64_t x = ((uint64_t)w[2 * half + 1] << 32) | (uint64_t)w[2 * half];
        unsigned __int128 prod = (unsigned __int128)x * (unsigned __int128)range;
        out[i] = (int32_t)(lo + (int64_t)(uint64_t)(prod >> 64));
    }
}

/* ------------------------------------------------------------------------------------------ */
/* Scores (Table 2), one triple at a time                                                     */
/* ------------------------------------------------------------------------------------------ */

static double orc_dot(const double *a, const double *b, int d)
{
    double s = 0.0;
    for (int j = 0; j < d; ++j) s += a[j] * b[j];
    return s;
}

/* unit normal of TransH: w / max(||w||_2, 1e-12) */
static double orc_unit_normal(const float *w, int d, double *what)
{
    double nn = 0.0;
    for (int j = 0; j < d; ++j) nn += (double)w[j] * (double)w[j];
    double nrm = sqrt(nn);
    if (nrm < 1e-12) nrm = 1e-12;
    for (int j = 0; j < d; ++j) what[j] = (double)w[j] / nrm;
    return nrm;
}

/*
 * f(h, r, t).  Rows are fp32 values (bf16 tables are widened exactly before the call).  Complex
 * vectors are stored as [real half | imaginary half].  For RotatE r holds d/2 phases.
 * DistMult and TransE use the sequential fused form that also serves as the ranking key:
 *   DistMult  acc = fma(h_j * r_j, t_j, acc)             (h_j * r_j is exact in fp64)
 *   TransE    x = (h_j + r_j) - t_j; acc = fma(x, x, acc); f = -sqrt(acc)
 * 1-norm variants: f = -sum_j |x_j| over the same difference vector x; for RotatE the vector is taken in
 * R^d (|Re x_j| + |Im x_j| per complex coordinate), following the identification C^{d/2} = R^d of
 * Section 3.1.  sq_out receives the ranking key (smaller = better): the squared distance, the 1-norm,
 * or minus the score.
 */
static double orc_score_one_ex(int scorer, int d, const float *h, const float *r, const float *w,
                               const float *t, double *sq_out)
{
    double acc = 0.0;
    const int l1 = orc_is_l1(scorer);
    switch (orc_base_scorer(scorer)) {
    case ORC_TRANSE:
        for (int j = 0; j < d; ++j) {
            double x = ((double)h[j] + (double)r[j]) - (double)t[j];
            acc = l1 ? acc + fabs(x) : fma(x, x, acc);
        }
        if (sq_out) *sq_out = acc;
        return l1 ? -acc : -sqrt(acc);
    case ORC_DISTMULT:
        for (int j = 0; j < d; ++j) {
            double hr = (double)h[j] * (double)r[j];
            acc = fma(hr, (double)t[j], acc);
        }
        if (sq_out) *sq_out = -acc;
        return acc;
    case ORC_COMPLEX: {
        int c = d / 2;
        for (int j = 0; j < c; ++j) {
            double hre = h[j], him = h[j + c], rre = r[j], rim = r[j + c];
            double tre = t[j], tim = t[j + c];
            double qre = hre * rre - him * rim;
            double qim = hre * rim + him * rre;
            acc += qre * tre + qim * tim;
        }
        if (sq_out) *sq_out = -acc;
        return acc;
    }
    case ORC_ROTATE: {
        int c = d / 2;
        for (int j = 0; j < c; ++j) {
            double hre = h[j], him = h[j + c], ph = r[j];
            double cs = cos(ph), sn = sin(ph);
            double qre = hre * cs - him * sn;
            double qim = hre * sn + him * cs;
            double xre = qre - (double)t[j], xim = qim - (double)t[j + c];
            acc += l1 ? fabs(xre) + fabs(xim) : xre * xre + xim * xim;
        }
        if (sq_out) *sq_out = acc;
        return l1 ? -acc : -sqrt(acc);
    }
    case ORC_TRANSH: {
        double *what = (double *)malloc(sizeof(double) * (size_t)d);
        orc_unit_normal(w, d, what);
        double wh = 0.0, wt = 0.0;
        for (int j = 0; j < d; ++j) { wh += what[j] * (double)h[j]; wt += what[j] * (double)t[j]; }
        for (int j = 0; j < d; ++j) {
            double hp = (double)h[j] - wh * what[j];
            double tp = (double)t[j] - wt * what[j];
            double x = hp + (double)r[j] - tp;
            acc += l1 ? fabs(x) : x * x;
        }
        free(what);
        if (sq_out) *sq_out = acc;
        return l1 ? -acc : -sqrt(acc);
    }
    default:
        return NAN;
    }
}

double orc_score_one(int scorer, int d, const float *h, const float *r, const float *w,
                     const float *t)
{
    return orc_score_one_ex(scorer, d, h, r, w, t, NULL);
}

static int orc_rel_dim(int scorer, int d) { return orc_base_scorer(scorer) == ORC_ROTATE ? d / 2 : d; }

/*
 * Positive scores pos[b] = f(h_b, r_b, t_b) and the shared-negative block
 * neg[b*N + n] = f(h_b, r_b, t'_n)  (eq. (negsamples): same corrupted tails for every triple).
 */
void orc_score_batch(int scorer, int d, const float *ent, const float *rel, const float *relw,
                     const int32_t *h, const int32_t *r, const int32_t *t, int64_t B,
                     const int32_t *neg, int64_t N, double *pos_out, double *neg_out)
{
    int k = orc_rel_dim(scorer, d);
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        const float *hb = ent + (int64_t)h[b] * d;
        const float *rb = rel + (int64_t)r[b] * k;
        const float *wb = relw ? relw + (int64_t)r[b] * d : NULL;
        if (pos_out) pos_out[b] = orc_score_one(scorer, d, hb, rb, wb, ent + (int64_t)t[b] * d);
        if (neg_out)
            for (int64_t n = 0; n < N; ++n)
                neg_out[b * N + n] = orc_score_one(scorer, d, hb, rb, wb, ent + (int64_t)neg[n] * d);
    }
}

/* ------------------------------------------------------------------------------------------ */
/* Gradient of one score: adds g * df/d(h, r, w, t) to the four outputs                        */
/* ------------------------------------------------------------------------------------------ */

static void orc_score_grad_one(int scorer, int d, const float *h, const float *r, const float *w,
                               const float *t, double g, double *dh, double *dr, double *dw,
                               double *dt)
{
    /* 1-norm variants: df/dx_j = -sign(x_j) replaces -x_j / ||x||_2; the chain through x is unchanged */
    const int l1 = orc_is_l1(scorer);
    switch (orc_base_scorer(scorer)) {
    case ORC_TRANSE: {
        double acc = 0.0;
        for (int j = 0; j < d; ++j) {
            double x = ((double)h[j] + (double)r[j]) - (double)t[j];
            acc += x * x;
        }
        double dist = sqrt(acc);
        if (dist == 0.0) return;              /* sub-gradient 0 at the kink */
        for (int j = 0; j < d; ++j) {
            double x = ((double)h[j] + (double)r[j]) - (double)t[j];
            double a = l1 ? -g * orc_sign(x) : -g * x / dist;         /* g * df/dx_j */
            dh[j] += a; dr[j] += a; dt[j] -= a;
        }
        return;
    }
    case ORC_DISTMULT:
        for (int j = 0; j < d; ++j) {
            dh[j] += g * (double)r[j] * (double)t[j];
            dr[j] += g * (double)h[j] * (double)t[j];
            dt[j] += g * (double)h[j] * (double)r[j];
        }
        return;
    case ORC_COMPLEX: {
        int c = d / 2;
        for (int j = 0; j < c; ++j) {
            double hre = h[j], him = h[j + c], rre = r[j], rim = r[j + c];
            double tre = t[j], tim = t[j + c];
            /* f = sum (hre rre - him rim) tre + (hre rim + him rre) tim */
            dh[j]     += g * (rre * tre + rim * tim);
            dh[j + c] += g * (-rim * tre + rre * tim);
            dr[j]     += g * (hre * tre + him * tim);
            dr[j + c] += g * (-him * tre + hre * tim);
            dt[j]     += g * (hre * rre - him * rim);
            dt[j + c] += g * (hre * rim + him * rre);
        }
        return;
    }
    case ORC_ROTATE: {
        int c = d / 2;
        double acc = 0.0;
        for (int j = 0; j < c; ++j) {
            double cs = cos((double)r[j]), sn = sin((double)r[j]);
            double xre = ((double)h[j] * cs - (double)h[j + c] * sn) - (double)t[j];
            double xim = ((double)h[j] * sn + (double)h[j + c] * cs) - (double)t[j + c];
            acc += xre * xre + xim * xim;
        }
        double dist = sqrt(acc);
        if (dist == 0.0) return;
        for (int j = 0; j < c; ++j) {
            double hre = h[j], him = h[j + c];
            double cs = cos((double)r[j]), sn = sin((double)r[j]);
            double qre = hre * cs - him * sn, qim = hre * sn + him * cs;
            double are = l1 ? -g * orc_sign(qre - (double)t[j]) : -g * (qre - (double)t[j]) / dist;          /* g * df/dq_re */
            double aim = l1 ? -g * orc_sign(qim - (double)t[j + c]) : -g * (qim - (double)t[j + c]) / dist;  /* g * df/dq_im */
            dh[j]     += are * cs + aim * sn;
            dh[j + c] += -are * sn + aim * cs;
            dr[j]     += are * (-qim) + aim * qre;              /* dq_re/dr = -q_im, dq_im/dr = q_re */
            dt[j]     -= are;
            dt[j + c] -= aim;
        }
        return;
    }
    case ORC_TRANSH: {
        double *buf = (double *)malloc(sizeof(double) * (size_t)d * 4);
        double *what = buf, *x = buf + d, *a = buf + 2 * d, *dwh = buf + 3 * d;
        double nrm = orc_unit_normal(w, d, what);
        /* u = (h - t) - (what.(h - t)) what + r */
        double s = 0.0;
        for (int j = 0; j < d; ++j) s += what[j] * ((double)h[j] - (double)t[j]);
        double acc = 0.0;
        for (int j = 0; j < d; ++j) {
            x[j] = ((double)h[j] - (double)t[j]) - s * what[j] + (double)r[j];
            acc += x[j] * x[j];
        }
        double dist = sqrt(acc);
        if (dist == 0.0) { free(buf); return; }
        double aw = 0.0;
        for (int j = 0; j < d; ++j) { a[j] = l1 ? -g * orc_sign(x[j]) : -g * x[j] / dist; aw += a[j] * what[j]; }
        for (int j = 0; j < d; ++j) {
            double ax = a[j] - aw * what[j];           /* through (h - t) */
            dh[j] += ax; dt[j] -= ax; dr[j] += a[j];
            /* through what: d/dwhat_k of -(what.(h-t)) what_j */
            dwh[j] = -((double)h[j] - (double)t[j]) * aw - s * a[j];
        }
        /* what = w / ||w||  ->  dw = (dwhat - what (what . dwhat)) / ||w|| */
        double wd = orc_dot(what, dwh, d);
        for (int j = 0; j < d; ++j) dw[j] += (dwh[j] - what[j] * wd) / nrm;
        free(buf);
        return;
    }
    default:
        return;
    }
}

/* ------------------------------------------------------------------------------------------ */
/* Losses and their derivatives with respect to the scores                                     */
/* ------------------------------------------------------------------------------------------ */

static double orc_log_sigmoid(double x)
{
    /* log sigma(x) = min(x, 0) - log1p(exp(-|x|)) */
    return (x < 0.0 ? x : 0.0) - log1p(exp(-fabs(x)));
}

static double orc_sigmoid(double x)
{
    if (x >= 0.0) return 1.0 / (1.0 + exp(-x));
    double e = exp(x);
    return e / (1.0 + e);
}

/*
 * Per-triple loss from its positive score fp and its N negative scores s[0..N), and the
 * derivatives dL/dfp and dL/ds[n].
 *  log-sigmoid:     L = -log sigma(gamma + fp) - sum_n w_n log sigma(-gamma - s_n),
 *                   w = softmax_n(a * s) held constant (StopGrad)
 *  sampled softmax: L = -fp + log(exp(fp) + sum_n exp(s_n + c)),  c = log((|E| - 1) / N)
 */
double orc_loss_one(int loss, double gamma, double adv_temp, int64_t n_ent_for_c, double fp,
                    const double *s, int64_t N, double *dfp, double *ds)
{
    if (loss == ORC_LOGSIGMOID) {
        double L = -orc_log_sigmoid(gamma + fp);
        if (dfp) *dfp = -orc_sigmoid(-(gamma + fp));
        if (N == 0) return L;
        double mx = -INFINITY;
        for (int64_t n = 0; n < N; ++n) if (adv_temp * s[n] > mx) mx = adv_temp * s[n];
        double z = 0.0;
        for (int64_t n = 0; n < N; ++n) z += exp(adv_temp * s[n] - mx);
        for (int64_t n = 0; n < N; ++n) {
            double wn = exp(adv_temp * s[n] - mx) / z;
            L -= wn * orc_log_sigmoid(-gamma - s[n]);
            if (ds) ds[n] = wn * orc_sigmoid(gamma + s[n]);
        }
        return L;
    }
    /* sampled softmax */
    if (N == 0) { if (dfp) *dfp = 0.0; return 0.0; }
    double c = log((double)(n_ent_for_c - 1) / (double)N);
    double mx = fp;
    for (int64_t n = 0; n < N; ++n) if (s[n] + c > mx) mx = s[n] + c;
    double z = exp(fp - mx);
    for (int64_t n = 0; n < N; ++n) z += exp(s[n] + c - mx);
    double lse = mx + log(z);
    if (dfp) *dfp = exp(fp - lse) - 1.0;
    if (ds) for (int64_t n = 0; n < N; ++n) ds[n] = exp(s[n] + c - lse);
    return -fp + lse;
}

/*
 * Micro-batch loss  loss_scale * sum_b L_b  and its gradient with respect to every gathered row,
 * per slot (duplicates are NOT merged here; that is the scatter's job):
 *   g_ent  [(2B+N) * d] : heads (slots 0..B), positive tails (B..2B), shared negatives (2B..2B+N)
 *   g_rel  [B * k], g_relw [B * d] (TransH only)
 */
/* L3 norm of one embedding row, (sum_j |x_j|^3)^(1/3) (Section 3.1 "Regularisation": the norm itself,
   not its cube), and, when g is given, lambda * its gradient added to g:
   d||x||_3 / dx_j = sign(x_j) x_j^2 / ||x||_3^2, taken as 0 at x = 0. */
double orc_l3_norm(int d, const float *x, double lambda, double *g)
{
    double s = 0.0;
    for (int j = 0; j < d; ++j) { double a = fabs((double)x[j]); s += a * a * a; }
    double nrm = cbrt(s);
    if (g && nrm > 0.0)
        for (int j = 0; j < d; ++j) {
            double v = (double)x[j];
            g[j] += lambda * (v < 0.0 ? -1.0 : 1.0) * v * v / (nrm * nrm);
        }
    return nrm;
}

/* Micro-batch loss loss_scale * sum_b L_b + reg_l3 * Omega_S with
   Omega_S = sum_b (||h_b||_3 + ||t_b||_3) + sum_i ||t'_i||_3 over the gathered shallow embeddings
   (Section 3.1 "Regularisation"; without text features Omega_T = Omega_S and Omega_F = 0). */
double orc_loss_bwd(int scorer, int loss, int d, const float *ent, const float *rel,
                    const float *relw, const int32_t *h, const int32_t *r, const int32_t *t,
                    int64_t B, const int32_t *neg, int64_t N, double gamma, double adv_temp,
                    double loss_scale, int64_t n_ent_for_c, double reg_l3, double *g_ent, double *g_rel,
                    double *g_relw, double *per_triple_loss)
{
    int k = orc_rel_dim(scorer, d);
    if (g_ent) memset(g_ent, 0, sizeof(double) * (size_t)(2 * B + N) * (size_t)d);
    if (g_rel) memset(g_rel, 0, sizeof(double) * (size_t)B * (size_t)k);
    if (g_relw) memset(g_relw, 0, sizeof(double) * (size_t)B * (size_t)d);
    double *Lb = (double *)malloc(sizeof(double) * (size_t)(B > 0 ? B : 1));
    /* per-thread accumulation of the shared negatives' gradients would reorder sums between
       runs; instead every b writes its own G row, and the negatives are summed over b in order. */
    double *G = (double *)malloc(sizeof(double) * (size_t)(B * N > 0 ? B * N : 1));
    double *Gp = (double *)malloc(sizeof(double) * (size_t)(B > 0 ? B : 1));
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        const float *hb = ent + (int64_t)h[b] * d;
        const float *rb = rel + (int64_t)r[b] * k;
        const float *wb = relw ? relw + (int64_t)r[b] * d : NULL;
        double *s = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
        double fp = orc_score_one(scorer, d, hb, rb, wb, ent + (int64_t)t[b] * d);
        for (int64_t n = 0; n < N; ++n)
            s[n] = orc_score_one(scorer, d, hb, rb, wb, ent + (int64_t)neg[n] * d);
        double dfp = 0.0;
        Lb[b] = orc_loss_one(loss, gamma, adv_temp, n_ent_for_c, fp, s, N, &dfp, G + b * N);
        Gp[b] = dfp;
        free(s);
    }
    double total = 0.0;
    for (int64_t b = 0; b < B; ++b) total += Lb[b];
    if (per_triple_loss) memcpy(per_triple_loss, Lb, sizeof(double) * (size_t)B);
    if (g_ent) {
        /* rows owned by triple b: its head, its positive tail, its relation rows */
#pragma omp parallel for schedule(static)
        for (int64_t b = 0; b < B; ++b) {
            const float *hb = ent + (int64_t)h[b] * d;
            const float *rb = rel + (int64_t)r[b] * k;
            const float *wb = relw ? relw + (int64_t)r[b] * d : NULL;
            double *dh = g_ent + b * d, *dtp = g_ent + (B + b) * d;
            double *dr = g_rel + b * k;
            double *dw = g_relw ? g_relw + b * d : NULL;
            double *scratch = (double *)calloc((size_t)d, sizeof(double));
            orc_score_grad_one(scorer, d, hb, rb, wb, ent + (int64_t)t[b] * d,
                               loss_scale * Gp[b], dh, dr, dw, dtp);
            for (int64_t n = 0; n < N; ++n) {
                memset(scratch, 0, sizeof(double) * (size_t)d);
                orc_score_grad_one(scorer, d, hb, rb, wb, ent + (int64_t)neg[n] * d,
                                   loss_scale * G[b * N + n], dh, dr, dw, scratch);
            }
            free(scratch);
        }
        /* shared negatives: slot 2B+n collects over all b, in increasing b */
#pragma omp parallel for schedule(static)
        for (int64_t n = 0; n < N; ++n) {
            double *dtn = g_ent + (2 * B + n) * d;
            double *sh = (double *)malloc(sizeof(double) * (size_t)d * 3);
            for (int64_t b = 0; b < B; ++b) {
                const float *hb = ent + (int64_t)h[b] * d;
                const float *rb = rel + (int64_t)r[b] * k;
                const float *wb = relw ? relw + (int64_t)r[b] * d : NULL;
                memset(sh, 0, sizeof(double) * (size_t)d * 3);
                orc_score_grad_one(scorer, d, hb, rb, wb, ent + (int64_t)neg[n] * d,
                                   loss_scale * G[b * N + n], sh, sh + d, sh + 2 * d, dtn);
            }
            free(sh);
        }
    }
    free(Lb); free(G); free(Gp);
    double omega = 0.0;
    if (reg_l3 != 0.0) {
        /* one term per gathered slot, in slot order: heads, positive tails, shared negatives */
        for (int64_t b = 0; b < B; ++b)
            omega += orc_l3_norm(d, ent + (int64_t)h[b] * d, reg_l3, g_ent ? g_ent + b * d : NULL);
        for (int64_t b = 0; b < B; ++b)
            omega += orc_l3_norm(d, ent + (int64_t)t[b] * d, reg_l3, g_ent ? g_ent + (B + b) * d : NULL);
        for (int64_t n = 0; n < N; ++n)
            omega += orc_l3_norm(d, ent + (int64_t)neg[n] * d, reg_l3, g_ent ? g_ent + (2 * B + n) * d : NULL);
    }
    return loss_scale * total + reg_l3 * omega;
}

/* ------------------------------------------------------------------------------------------ */
/* Duplicate-aware scatter-add + lazy sparse Adam                                              */
/* ------------------------------------------------------------------------------------------ */

/*
 * Gradient rows grads[M*d] target table rows idx[M] (duplicates allowed).  Rows aiming at the
 * same table row are summed in increasing position, in fp64; each touched row then takes one
 * Adam step with global step t >= 1:
 *    m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;
 *    theta <- theta - lr * (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps)
 * Untouched rows and their moments do not change.  touched[n_rows] is set to 1 for updated rows.
 */
void orc_sparse_adam(double *theta, double *m, double *v, int64_t n_rows, int d,
                     const int32_t *idx, const float *grads, int64_t M, double lr, double beta1,
                     double beta2, double eps, int64_t step, uint8_t *touched)
{
    double *gsum = (double *)calloc((size_t)n_rows * (size_t)d, sizeof(double));
    uint8_t *hit = (uint8_t *)calloc((size_t)n_rows, 1);
    for (int64_t i = 0; i < M; ++i) {
        int64_t row = idx[i];
        hit[row] = 1;
        for (int j = 0; j < d; ++j) gsum[row * d + j] += (double)grads[i * d + j];
    }
    double bc1 = 1.0 - pow(beta1, (double)step);
    double bc2 = 1.0 - pow(beta2, (double)step);
    for (int64_t row = 0; row < n_rows; ++row) {
        if (!hit[row]) continue;
        for (int j = 0; j < d; ++j) {
            int64_t e = row * d + j;
            double g = gsum[e];
            m[e] = beta1 * m[e] + (1.0 - beta1) * g;
            v[e] = beta2 * v[e] + (1.0 - beta2) * g * g;
            double mhat = m[e] / bc1, vhat = v[e] / bc2;
            theta[e] -= lr * mhat / (sqrt(vhat) + eps);
        }
    }
    if (touched) memcpy(touched, hit, (size_t)n_rows);
    free(gsum); free(hit);
}

/* round-to-nearest-even fp32 -> bf16 bit pattern (finite inputs) */
uint16_t orc_bf16_rne(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

void orc_bf16_rne_array(const float *x, int64_t n, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = orc_bf16_rne(x[i]);
}

/* ------------------------------------------------------------------------------------------ */
/* Full ranking: top-K by (score descending, index ascending), rank of a held-out tail         */
/* ------------------------------------------------------------------------------------------ */

typedef struct { double key; int32_t idx; } orc_item;   /* smaller key = better (key = -score or dist^2) */

/* "a is worse than b": larger key, or same key and larger index */
static int orc_worse(orc_item a, orc_item b)
{
    return a.key > b.key || (a.key == b.key && a.idx > b.idx);
}

static void orc_sift_down(orc_item *hp, int n, int i)
{
    for (;;) {                              /* max-heap on "worse": the root is the worst kept */
        int l = 2 * i + 1, r = l + 1, top = i;
        if (l < n && orc_worse(hp[l], hp[top])) top = l;
        if (r < n && orc_worse(hp[r], hp[top])) top = r;
        if (top == i) return;
        orc_item tmp = hp[i]; hp[i] = hp[top]; hp[top] = tmp;
        i = top;
    }
}

static void orc_sift_up(orc_item *hp, int i)
{
    while (i > 0) {
        int p = (i - 1) / 2;
        if (!orc_worse(hp[i], hp[p])) return;
        orc_item tmp = hp[i]; hp[i] = hp[p]; hp[p] = tmp;
        i = p;
    }
}

/*
 * For each query (h_q, r_q): score every candidate t in [cand_lo, cand_hi), keep the K best in a
 * size-K heap, emit them best first.  Ranking key: DistMult -score, distance scorers dist^2
 * (monotone in the score, avoids the square root in comparisons); ties go to the lower index.
 * out_score is the score itself.  If K exceeds the number of candidates the tail of the list is
 * padded with index -1 and score -inf.
 * rank(true) = 1 + #{t : key(t) < key(true)} + #{t < true : key(t) = key(true)}   (1-based),
 * counted over the same candidate range (the true tail need not lie inside it).
 */
void orc_topk_band(int scorer, int d, const float *ent, const float *rel, const float *relw,
                   const int32_t *h, const int32_t *r, int64_t Q, int64_t cand_lo, int64_t cand_hi,
                   int32_t K, int32_t *out_idx, double *out_score, const int32_t *true_t,
                   int64_t *out_rank, const double *band_eps, int64_t *out_band);

void orc_topk(int scorer, int d, const float *ent, const float *rel, const float *relw,
              const int32_t *h, const int32_t *r, int64_t Q, int64_t cand_lo, int64_t cand_hi,
              int32_t K, int32_t *out_idx, double *out_score, const int32_t *true_t,
              int64_t *out_rank)
{
    orc_topk_band(scorer, d, ent, rel, relw, h, r, Q, cand_lo, cand_hi, K, out_idx, out_score, true_t,
                  out_rank, NULL, NULL);
}

/*
 * The same ranking, and in the same pass over the candidates (band_eps and out_band given, with a held-out
 * tail): out_band[q] = #{t in the range : |key(t) - key(true_q)| <= band_eps[q]}, the number of candidates
 * whose ranking key lies within band_eps[q] of the held-out tail's.  A ranking that compares approximate
 * keys, each within eps/2 of the exact one, can misplace the held-out tail by at most that many positions.
 */
void orc_topk_band(int scorer, int d, const float *ent, const float *rel, const float *relw,
                   const int32_t *h, const int32_t *r, int64_t Q, int64_t cand_lo, int64_t cand_hi,
                   int32_t K, int32_t *out_idx, double *out_score, const int32_t *true_t,
                   int64_t *out_rank, const double *band_eps, int64_t *out_band)
{
    int k = orc_rel_dim(scorer, d);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < Q; ++q) {
        const float *hq = ent + (int64_t)h[q] * d;
        const float *rq = rel + (int64_t)r[q] * k;
        const float *wq = relw ? relw + (int64_t)r[q] * d : NULL;
        orc_item *hp = (orc_item *)malloc(sizeof(orc_item) * (size_t)(K > 0 ? K : 1));
        int cnt = 0;
        double true_key = 0.0;
        int64_t above = 0, band = 0;
        if (true_t && out_rank)
            orc_score_one_ex(scorer, d, hq, rq, wq, ent + (int64_t)true_t[q] * d, &true_key);
        for (int64_t t = cand_lo; t < cand_hi; ++t) {
            orc_item it;
            it.idx = (int32_t)t;
            orc_score_one_ex(scorer, d, hq, rq, wq, ent + t * d, &it.key);
            if (true_t && out_rank) {
                if (it.key < true_key || (it.key == true_key && t < (int64_t)true_t[q])) ++above;
                if (band_eps && fabs(it.key - true_key) <= band_eps[q]) ++band;
            }
            if (K <= 0) continue;
            if (cnt < K) {
                hp[cnt] = it;
                orc_sift_up(hp, cnt);
                ++cnt;
            } else if (orc_worse(hp[0], it)) {
                hp[0] = it;
                orc_sift_down(hp, cnt, 0);
            }
        }
        if (true_t && out_rank) out_rank[q] = 1 + above;
        if (true_t && out_rank && band_eps && out_band) out_band[q] = band;
        /* pop worst-first into the back of the list */
        int kept = cnt;
        for (int i = kept - 1; i >= 0; --i) {
            orc_item worst = hp[0];
            hp[0] = hp[cnt - 1];
            --cnt;
            orc_sift_down(hp, cnt, 0);
            out_idx[q * K + i] = worst.idx;
            double sc;
            if (scorer == ORC_DISTMULT || scorer == ORC_COMPLEX || orc_is_l1(scorer)) sc = -worst.key;
            else sc = -sqrt(worst.key);
            out_score[q * K + i] = sc;
        }
        for (int i = kept; i < K; ++i) { out_idx[q * K + i] = -1; out_score[q * K + i] = -INFINITY; }
        free(hp);
    }
}

/* ------------------------------------------------------------------------------------------ */
/* Partition bucketing (Section 4, "Partitioning")                                             */
/* ------------------------------------------------------------------------------------------ */

/*
 * Entities are split into D shards of part_size = ceil(|E| / D) consecutive ids (the ids are
 * assumed already randomly permuted); triple (h, r, t) falls in bucket part(h) * D + part(t).
 * Outputs: counts[D*D]; offsets[D*D + 1] (exclusive prefix sums); order[n] = the stable
 * counting-sort permutation (triples of one bucket keep their input order).
 */
void orc_bucket_triples(const int32_t *h, const int32_t *t, int64_t n, int64_t part_size, int D,
                        int64_t *counts, int64_t *offsets, int64_t *order)
{
    int nb = D * D;
    for (int i = 0; i < nb; ++i) counts[i] = 0;
    for (int64_t i = 0; i < n; ++i)
        counts[(h[i] / part_size) * D + (t[i] / part_size)]++;
    offsets[0] = 0;
    for (int i = 0; i < nb; ++i) offsets[i + 1] = offsets[i] + counts[i];
    if (order) {
        int64_t *cur = (int64_t *)malloc(sizeof(int64_t) * (size_t)nb);
        for (int i = 0; i < nb; ++i) cur[i] = offsets[i];
        for (int64_t i = 0; i < n; ++i) {
            int bkt = (int)((h[i] / part_size) * D + (t[i] / part_size));
            order[cur[bkt]++] = i;
        }
        free(cur);
    }
}

/* ------------------------------------------------------------------------------------------ */
/* Relation-aware triple sampler (Section 4, "Training")                                       */
/* ------------------------------------------------------------------------------------------ */

/* Weight of a relation with n triples in a bucket: w(n) = floor(2^20 * n^(1/3)), the largest integer
   whose cube does not exceed n * 2^60.  Exact integer arithmetic, so that every implementation of the
   sampler draws from the same table.  The paper's law is p(r) proportional to the cube root of n_r;
   the truncation changes a probability by less than one part in 2^20.  n < 2^32. */
uint64_t orc_cbrt_weight(uint64_t n)
{
    unsigned __int128 target = (unsigned __int128)n << 60;
    uint64_t w = 0;
    for (int bit = 31; bit >= 0; --bit) {       /* w < 2^32 since n < 2^32 */
        uint64_t c = w | (1ull << bit);
        unsigned __int128 cube = (unsigned __int128)c * c * c;
        if (cube <= target) w = c;
    }
    return w;
}

/* Index over the triples: a stable sort by (bucket, relation), bucket = (h / part_size) * D + t / part_size
   (Section 4, "Partitioning"), with
     order       [n]                position in the input of the k-th triple of the sorted list
     rel_offsets [D*D*n_rel + 1]    first sorted position of every (bucket, relation) group
     cdf         [D*D*n_rel]        inclusive prefix sums, inside each bucket, of w(n_r)                  */
void orc_sampler_build(const int32_t *h, const int32_t *r, const int32_t *t, int64_t n, int64_t part_size,
                       int D, int64_t n_rel, int64_t *order, int64_t *rel_offsets, uint64_t *cdf)
{
    int64_t groups = (int64_t)D * D * n_rel;
    for (int64_t g = 0; g <= groups; ++g) rel_offsets[g] = 0;
    for (int64_t i = 0; i < n; ++i) {
        int64_t g = ((h[i] / part_size) * D + (t[i] / part_size)) * n_rel + r[i];
        rel_offsets[g + 1]++;
    }
    for (int64_t g = 0; g < groups; ++g) rel_offsets[g + 1] += rel_offsets[g];
    int64_t *cur = (int64_t *)malloc(sizeof(int64_t) * (size_t)(groups > 0 ? groups : 1));
    for (int64_t g = 0; g < groups; ++g) cur[g] = rel_offsets[g];
    for (int64_t i = 0; i < n; ++i) {
        int64_t g = ((h[i] / part_size) * D + (t[i] / part_size)) * n_rel + r[i];
        order[cur[g]++] = i;
    }
    free(cur);
    for (int64_t b = 0; b < (int64_t)D * D; ++b) {
        uint64_t run = 0;
        for (int64_t q = 0; q < n_rel; ++q) {
            int64_t g = b * n_rel + q;
            run += orc_cbrt_weight((uint64_t)(rel_offsets[g + 1] - rel_offsets[g]));
            cdf[g] = run;
        }
    }
}

/* Draw q of the call, q < n_buckets * per_bucket, samples from bucket bucket_lo + q / per_bucket: first a
   relation with probability w(n_r) / sum_r' w(n_r'), then one of its n_r triples uniformly, with replacement:
       p((h, r, t)) = (1 / n_r) * cbrt(n_r) / sum_r' cbrt(n_r').
   Philox4x32-10 with key = seed and counter (q_lo, q_hi, step, tag); x = w1:w0 picks the relation as the
   first one whose cdf exceeds floor(x * total / 2^64), y = w3:w2 the triple floor(y * n_r / 2^64) of the group.
   out_pos[q] = position of the triple in the input arrays, or -1 when the bucket is empty. */
void orc_sample_triples(uint64_t seed, uint64_t step, uint32_t tag, int64_t bucket_lo, int64_t n_buckets,
                        int64_t per_bucket, int64_t n_rel, const int64_t *rel_offsets, const uint64_t *cdf,
                        const int64_t *order, int64_t *out_pos)
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    for (int64_t q = 0; q < n_buckets * per_bucket; ++q) {
        int64_t b = bucket_lo + q / per_bucket;
        const uint64_t *c = cdf + b * n_rel;
        uint64_t total = n_rel > 0 ? c[n_rel - 1] : 0;
        if (total == 0) { out_pos[q] = -1; continue; }
        uint32_t ctr[4] = { (uint32_t)q, (uint32_t)((uint64_t)q >> 32), (uint32_t)step, tag };
        uint32_t w[4];
        orc_philox4x32_10(ctr, key, w);
        uint64_t x = ((uint64_t)w[1] << 32) | w[0], y = ((uint64_t)w[3] << 32) | w[2];
        uint64_t pick = (uint64_t)(((unsigned __int128)x * total) >> 64);
        int64_t rel = 0;
        while (c[rel] <= pick) ++rel;           /* plain scan: the first relation whose cdf exceeds pick */
        int64_t g = b * n_rel + rel;
        uint64_t cnt = (uint64_t)(rel_offsets[g + 1] - rel_offsets[g]);
        uint64_t k = (uint64_t)(((unsigned __int128)y * cnt) >> 64);
        out_pos[q] = order[rel_offsets[g] + (int64_t)k];
    }
}

/* Shared negatives of one worker's micro-batch (Section 4, eq. (negsamples)): per_shard ids from every
   entity shard E_j = [j * part_size, min(n_ent, (j+1) * part_size)), slot n belongs to shard n / per_shard.
   Same generator layout as orc_sample_negatives (block n/2, two ids per block). */
void orc_sample_negatives_sharded(uint64_t seed, uint64_t step, uint32_t tag, int64_t part_size, int64_t n_ent,
                                  int D, int64_t per_shard, int32_t *out)
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    for (int64_t i = 0; i < (int64_t)D * per_shard; ++i) {
        int64_t j = i / per_shard, lo = j * part_size, hi = lo + part_size < n_ent ? lo + part_size : n_ent;
        uint64_t block = (uint64_t)i / 2;
        uint32_t ctr[4] = { (uint32_t)block, (uint32_t)(block >> 32), (uint32_t)step, tag };
        uint32_t w[4];
        orc_philox4x32_10(ctr, key, w);
        int half = (int)(i & 1);
        uint64_t x = ((uint64_t)w[2 * half + 1] << 32) | (uint64_t)w[2 * half];
        out[i] = (int32_t)(lo + (int64_t)(uint64_t)(((unsigned __int128)x * (uint64_t)(hi - lo)) >> 64));
    }
}

/* ------------------------------------------------------------------------------------------ */
/* Feature-projection encoder (Section 3.1 "Encoder", eq. (embedding))                         */
/* ------------------------------------------------------------------------------------------ */

/* Dropout mask of element (slot, column): Philox4x32-10, key = seed, counter (slot_lo, slot_hi / column block,
   step, tag): counter = (slot, column / 4, step, tag), word column % 4; the element is KEPT when its word is
   >= floor(p * 2^32) and then scaled by 1 / (1 - p) (Section 3.1 "Regularisation": dropout on the linear
   projections before they are summed with the shallow embedding).  p = 0 keeps everything. */
static double orc_dropout_factor(uint64_t seed, uint64_t step, uint32_t tag, int64_t slot, int col, double p)
{
    if (p <= 0.0) return 1.0;
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t ctr[4] = { (uint32_t)slot, (uint32_t)(col / 4), (uint32_t)step, tag };
    uint32_t w[4];
    orc_philox4x32_10(ctr, key, w);
    uint32_t thr = (uint32_t)floor(p * 4294967296.0);
    return w[col % 4] >= thr ? 1.0 / (1.0 - p) : 0.0;
}

/* Forward over the 2B + N gathered slots (heads, positive tails, shared negatives):
     proj[i] = M f_i          (M = M_H for the B head slots, M_T for the others; f_i the slot's feature row)
     e[i]    = s_i + D_i o proj[i]      (s_i the slot's shallow embedding, D the dropout factors)
   and the regulariser value reg_t sum ||e_i||_3 + reg_s sum ||s_i||_3 + reg_f sum ||proj_i||_3.
   idx: the 2B + N entity ids in slot order.  proj, e: [(2B+N), d] fp64. */
double orc_encode(int d, int fd, const float *ent_s, const float *feat, const float *m_h, const float *m_t,
                  const int32_t *idx, int64_t B, int64_t N, double p, uint64_t seed, uint64_t step, uint32_t tag,
                  double reg_t, double reg_s, double reg_f, double *proj, double *e)
{
    int64_t n = 2 * B + N;
    double omega = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        const float *M = i < B ? m_h : m_t;
        const float *f = feat + (int64_t)idx[i] * fd, *s = ent_s + (int64_t)idx[i] * d;
        double t3 = 0.0, s3 = 0.0, f3 = 0.0;
        for (int j = 0; j < d; ++j) {
            double acc = 0.0;
            for (int k = 0; k < fd; ++k) acc += (double)M[(int64_t)j * fd + k] * (double)f[k];
            proj[i * d + j] = acc;
            double ev = (double)s[j] + orc_dropout_factor(seed, step, tag, i, j, p) * acc;
            e[i * d + j] = ev;
            t3 += fabs(ev) * ev * ev; s3 += fabs((double)s[j]) * (double)s[j] * (double)s[j]; f3 += fabs(acc) * acc * acc;
        }
        omega += reg_t * cbrt(t3) + reg_s * cbrt(s3) + reg_f * cbrt(f3);
    }
    return omega;
}

static void orc_l3_grad_d(int d, const double *x, double lambda, double *g)
{
    double s = 0.0;
    for (int j = 0; j < d; ++j) s += fabs(x[j]) * x[j] * x[j];
    double nrm = cbrt(s);
    if (nrm > 0.0)
        for (int j = 0; j < d; ++j) g[j] += lambda * (x[j] < 0.0 ? -1.0 : 1.0) * x[j] * x[j] / (nrm * nrm);
}

/* Backward: de [(2B+N), d] is the gradient of the loss with respect to e.  With e = s + D o proj, proj = M f:
     de' = de + reg_t grad||e||_3;   g_s = de' + reg_s grad||s||_3;   dproj = D o de' + reg_f grad||proj||_3;
     g_mh = sum over head slots of dproj_i f_i^t,   g_mt = the same over the tail and negative slots. */
void orc_encode_bwd(int d, int fd, const float *ent_s, const float *feat, const float *m_h, const float *m_t,
                    const int32_t *idx, int64_t B, int64_t N, double p, uint64_t seed, uint64_t step, uint32_t tag,
                    double reg_t, double reg_s, double reg_f, const double *de, double *g_s, double *g_mh,
                    double *g_mt)
{
    int64_t n = 2 * B + N;
    double *proj = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1) * (size_t)d);
    double *e = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1) * (size_t)d);
    orc_encode(d, fd, ent_s, feat, m_h, m_t, idx, B, N, p, seed, step, tag, 0.0, 0.0, 0.0, proj, e);
    memset(g_mh, 0, sizeof(double) * (size_t)d * (size_t)fd);
    memset(g_mt, 0, sizeof(double) * (size_t)d * (size_t)fd);
    double *dep = (double *)malloc(sizeof(double) * (size_t)d), *dpr = (double *)malloc(sizeof(double) * (size_t)d);
    double *sd = (double *)malloc(sizeof(double) * (size_t)d);
    for (int64_t i = 0; i < n; ++i) {
        const float *f = feat + (int64_t)idx[i] * fd, *s = ent_s + (int64_t)idx[i] * d;
        double *gm = i < B ? g_mh : g_mt;
        for (int j = 0; j < d; ++j) { dep[j] = de[i * d + j]; sd[j] = (double)s[j]; }
        orc_l3_grad_d(d, e + i * d, reg_t, dep);
        for (int j = 0; j < d; ++j) g_s[i * d + j] = dep[j];
        orc_l3_grad_d(d, sd, reg_s, g_s + i * d);
        for (int j = 0; j < d; ++j) dpr[j] = orc_dropout_factor(seed, step, tag, i, j, p) * dep[j];
        orc_l3_grad_d(d, proj + i * d, reg_f, dpr);
        for (int j = 0; j < d; ++j)
            for (int k = 0; k < fd; ++k) gm[(int64_t)j * fd + k] += dpr[j] * (double)f[k];
    }
    free(proj); free(e); free(dep); free(dpr); free(sd);
}

/* ------------------------------------------------------------------------------------------ */
/* Power-rank ensemble (Section 3.2 "Inference", paragraph "Ensemble", eq. (ensemble))          */
/* ------------------------------------------------------------------------------------------ */

/*
 * lists[(m * Q + q) * K + k-1] is the k-th best tail of model m for query q (distinct entities; -1 pads a
 * short list).  Every entity t gets s(t) = sum over the models, in model order, of
 *     -sgn(p) k^p          if t is the k-th entry of the model's list (its first occurrence counts),
 *     -[p > 0] (K + 1)^p   if the model's list does not hold t,
 * and the K_out entities with the largest s(t), ties to the smaller entity id, are returned.  An entity in no
 * list has the smallest possible score, so only entities that occur in some list are candidates; if
 * fewer than K_out occur the output is padded with -1 / -inf.
 */
void orc_ensemble(const int32_t *lists, int M, int64_t Q, int K, double p, int K_out, int32_t *out_idx,
                  double *out_score)
{
    const double absent = p > 0.0 ? -pow((double)(K + 1), p) : 0.0;
    const double sg = p > 0.0 ? -1.0 : 1.0;
    for (int64_t q = 0; q < Q; ++q) {
        int32_t *cand = (int32_t *)malloc(sizeof(int32_t) * (size_t)(M * K > 0 ? M * K : 1));
        double *sc = (double *)malloc(sizeof(double) * (size_t)(M * K > 0 ? M * K : 1));
        int nc = 0;
        /* candidates: every entity of every list, once */
        for (int m = 0; m < M; ++m)
            for (int k = 0; k < K; ++k) {
                int32_t t = lists[((int64_t)m * Q + q) * K + k];
                if (t < 0) continue;
                int seen = 0;
                for (int i = 0; i < nc && !seen; ++i) seen = cand[i] == t;
                if (!seen) cand[nc++] = t;
            }
        for (int i = 0; i < nc; ++i) {
            double s = 0.0;
            for (int m = 0; m < M; ++m) {
                const int32_t *lm = lists + ((int64_t)m * Q + q) * K;
                int rank = 0;
                for (int k = 0; k < K && !rank; ++k)
                    if (lm[k] == cand[i]) rank = k + 1;
                s += rank ? sg * pow((double)rank, p) : absent;
            }
            sc[i] = s;
        }
        /* selection of the K_out best, one at a time */
        for (int o = 0; o < K_out; ++o) {
            int best = -1;
            for (int i = 0; i < nc; ++i) {
                if (cand[i] < 0) continue;
                if (best < 0 || sc[i] > sc[best] || (sc[i] == sc[best] && cand[i] < cand[best])) best = i;
            }
            if (best < 0) { out_idx[q * K_out + o] = -1; out_score[q * K_out + o] = -INFINITY; continue; }
            out_idx[q * K_out + o] = cand[best];
            out_score[q * K_out + o] = sc[best];
            cand[best] = -1;
        }
        free(cand); free(sc);
    }
}
