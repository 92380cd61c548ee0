/*
 * tli_oracle.c -- CPU oracle for the Token-Level Intersection (TLI) draft-and-verify step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, fp64 statement of what the GPU library has
 * to compute.  Nothing in the product path may call, link or import it; it shares no code, header,
 * table or helper with the HIP sources.  Callers: the tests, the smoke check and the benchmark's
 * cpu_baseline leg.
 *
 * What it follows (paper sections, not listings):
 *   - TLI algorithm (token-level intersection): the drafter distribution q over D is restricted to
 *     the tokens shared with T and renormalised, q'(x) = q(x) / sum_{t in T∩D} q(t) for shared x and
 *     0 otherwise; standard speculative decoding is then run with p and q'.
 *   - Standard speculative decoding (appendix "Standard Speculative Decoding"): draw i draft tokens
 *     d_j ~ q', take the i+1 target rows, for j = 1..i accept d_j with probability
 *     min(1, p(d_j)/q'(d_j)) and stop at the first rejection; the extra token is drawn from the
 *     residual r(t) = (p(t) - min(p(t), q'(t))) / (1 - sum_t' min(p(t'), q'(t'))) of the rejected
 *     position, or from p of row i+1 when nothing was rejected.
 *   - Logits stand for the distributions: p = softmax(logits_t / tau_t), q = softmax(logits_d / tau_d).
 *
 * Conventions the paper leaves open (listed with their reasons in the design notes of the repository):
 *   - every random choice consumes a caller-supplied uniform u in [0,1);
 *   - inverse-CDF sampling walks ids in ascending order with a sequential fp64 running sum C and
 *     returns the first id whose C exceeds u * C_last (strict), so zero-weight ids are never chosen;
 *   - a draft is accepted iff u * q'(d) < p(d) (strict), which has probability min(1, p/q') exactly;
 *   - all K accept tests are evaluated, the accepted count is the length of the all-accept prefix.
 *
 * All arithmetic is IEEE double.  Inputs are taken exactly as stored (fp32, or bf16 as its 16 bits).
 * Every function in this file is pinned by tests/test_oracle_pins.py and tests/test_oracle_pins_next.py
 * (printed examples of the paper, its table of expected acceptance rates and its theorems, closed forms,
 * library routines, exact enumeration of the output distribution).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { TLO_F32 = 0, TLO_BF16 = 1 };

/* status bits (per drafter row / per sequence) */
enum {
    TLO_NONFINITE = 1,  /* a logit that takes part in the computation is NaN or +inf              */
    TLO_ZERO_MASS = 2,  /* the shared ids of a drafter row carry no mass (all -inf): q' is 0/0     */
    TLO_BAD_DRAFT = 4,  /* a draft id given to verify is not a shared drafter id (or is -1)        */
    TLO_DEGENERATE = 8  /* rejected, but the residual is identically zero: extra token drawn from p */
};

static double load_logit(const void *base, int dtype, int64_t idx) {
    if (dtype == TLO_F32) return (double)((const float *)base)[idx];
    uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/*
 * softmax(logits / tau) over n entries -> prob[n]; *log_norm = log sum_x exp(logits[x]/tau).
 * Returns TLO_NONFINITE if an entry is NaN or +inf (prob then unspecified), 0 otherwise.
 * -inf entries get probability 0.  A row of only -inf gives prob = 0 everywhere and log_norm = -inf.
 */
int tlo_softmax(const void *logits, int dtype, int64_t n, double tau, double *prob, double *log_norm) {
    double M = -INFINITY;
    int bad = 0;
    for (int64_t x = 0; x < n; ++x) {
        double z = load_logit(logits, dtype, x) / tau;
        if (isnan(z) || z == INFINITY) bad = 1;
        if (z > M) M = z;
    }
    if (bad) { *log_norm = NAN; return TLO_NONFINITE; }
    if (M == -INFINITY) {
        for (int64_t x = 0; x < n; ++x) prob[x] = 0.0;
        *log_norm = -INFINITY;
        return 0;
    }
    double Z = 0.0;
    for (int64_t x = 0; x < n; ++x) {
        prob[x] = exp(load_logit(logits, dtype, x) / tau - M);
        Z += prob[x];
    }
    for (int64_t x = 0; x < n; ++x) prob[x] /= Z;
    *log_norm = M + log(Z);
    return 0;
}

/*
 * TLI's adjusted drafter.  q = softmax(logits_d / tau_d) over all of D, then
 * q'(x) = q(x) / sum_{y shared} q(y) for shared x (d2t[x] >= 0), 0 otherwise.
 * The quotient is taken in log space: with z = logits_d / tau_d,
 *     q(x) / sum_{y shared} q(y) = exp(z_x - L_all) / exp(L_sh - L_all) = exp(z_x - L_sh),
 * L_sh = log sum_{y shared} exp(z_y) formed around the shared ids' own maximum.  (Divided as two fp64 numbers the
 * quotient turns into 0/0 once every shared id lies some 745 nats below the drafter's largest logit -- a cold
 * drafter whose favourites are outside the intersection -- although q' is then as well defined as anywhere.)
 * q[Vd] and qprime[Vd] are outputs; *log_norm_shared = L_sh, the normaliser that turns a shared logit straight
 * into log q'.
 * Status: NONFINITE if a SHARED logit is NaN/+inf; ZERO_MASS if the shared ids have total mass 0 (all -inf).
 * Unshared drafter logits must be finite or -inf (the method never looks at them again).
 */
int tlo_adjusted_drafter(const void *logits_d, int dtype, int64_t Vd, double tau_d, const int32_t *d2t,
                         double *q, double *qprime, double *log_norm_shared) {
    double Ms = -INFINITY;
    for (int64_t x = 0; x < Vd; ++x) {
        if (d2t[x] < 0) continue;
        double z = load_logit(logits_d, dtype, x);
        if (isnan(z) || z == INFINITY) {
            for (int64_t y = 0; y < Vd; ++y) { q[y] = NAN; qprime[y] = NAN; }
            *log_norm_shared = NAN;
            return TLO_NONFINITE;
        }
        if (z / tau_d > Ms) Ms = z / tau_d;
    }
    double log_norm_all;
    tlo_softmax(logits_d, dtype, Vd, tau_d, q, &log_norm_all);
    if (Ms == -INFINITY) {
        for (int64_t x = 0; x < Vd; ++x) qprime[x] = 0.0;
        *log_norm_shared = -INFINITY;
        return TLO_ZERO_MASS;
    }
    double Zs = 0.0;
    for (int64_t x = 0; x < Vd; ++x) {
        qprime[x] = (d2t[x] >= 0) ? exp(load_logit(logits_d, dtype, x) / tau_d - Ms) : 0.0;
        Zs += qprime[x];
    }
    for (int64_t x = 0; x < Vd; ++x) qprime[x] /= Zs;
    *log_norm_shared = Ms + log(Zs);
    return 0;
}

/*
 * Inverse-CDF sample from non-negative weights w[n] with uniform u in [0,1):
 * C_x = w_0 + ... + w_x (sequential), theta = u * C_{n-1}, result = min{x : C_x > theta}.
 * If rounding leaves no such x, the last id with w > 0.  Returns -1 if the total is 0.
 * *margin (may be NULL) = distance from theta to the nearer edge of the chosen id's CDF interval,
 * as a fraction of the total.
 */
int64_t tlo_inverse_cdf(const double *w, int64_t n, double u, double *margin) {
    double total = 0.0;
    for (int64_t x = 0; x < n; ++x) total += w[x];
    if (margin) *margin = 0.0;
    if (!(total > 0.0)) return -1;
    double theta = u * total;
    double C = 0.0, Cprev = 0.0;
    int64_t last_pos = -1;
    for (int64_t x = 0; x < n; ++x) {
        Cprev = C;
        C += w[x];
        if (w[x] > 0.0) last_pos = x;
        if (C > theta) {
            if (margin) {
                double lo = theta - Cprev, hi = C - theta;
                *margin = (lo < hi ? lo : hi) / total;
            }
            return x;
        }
    }
    return last_pos;
}

/*
 * Draft sampling for R independent drafter rows (row r at logits_d + r*row_stride elements):
 * tok_d[r] ~ q'_r by inverse CDF with u_draft[r]; tok_t[r] = d2t[tok_d[r]];
 * q_tok[r] = q'_r(tok_d[r]); lse_q[r] = log sum_{shared} exp(logit/tau_d).
 * Rows flagged NONFINITE or ZERO_MASS return tok_d = tok_t = -1 and q_tok = 0.
 * work must hold 2*Vd doubles.
 */
void tlo_draft_sample(const void *logits_d, int dtype, int64_t row_stride, int64_t R, int64_t Vd,
                      double tau_d, const int32_t *d2t, const double *u_draft,
                      int32_t *tok_d, int32_t *tok_t, double *q_tok, double *lse_q,
                      int32_t *row_status, double *cdf_margin, double *work) {
    size_t esz = (dtype == TLO_F32) ? 4 : 2;
    double *q = work, *qp = work + Vd;
    for (int64_t r = 0; r < R; ++r) {
        const void *row = (const char *)logits_d + (size_t)r * (size_t)row_stride * esz;
        int st = tlo_adjusted_drafter(row, dtype, Vd, tau_d, d2t, q, qp, &lse_q[r]);
        row_status[r] = st;
        tok_d[r] = -1; tok_t[r] = -1; q_tok[r] = 0.0;
        if (cdf_margin) cdf_margin[r] = 0.0;
        if (st) continue;
        double mg;
        int64_t d = tlo_inverse_cdf(qp, Vd, u_draft[r], &mg);
        tok_d[r] = (int32_t)d;
        tok_t[r] = d2t[d];
        q_tok[r] = qp[d];
        if (cdf_margin) cdf_margin[r] = mg;
    }
}

/*
 * Weights of the extra token for one sequence, unnormalised over target ids:
 *   rejected at position j : r(t) = (p_j(t) - min(p_j(t), q'_j(t))) / (1 - sum min(p_j, q'_j))
 *   nothing rejected       : p_{K+1}(t)
 * qprime_t[Vt] is q'_j laid out over target ids (0 for target-only ids).
 * Returns 1 if the residual is degenerate (normaliser <= 0 or all numerators 0); w is then p.
 */
static int residual_weights(const double *p, const double *qprime_t, int64_t Vt, double *w) {
    double overlap = 0.0;
    for (int64_t t = 0; t < Vt; ++t) overlap += fmin(p[t], qprime_t[t]);
    double denom = 1.0 - overlap;
    double total = 0.0;
    for (int64_t t = 0; t < Vt; ++t) {
        w[t] = p[t] - fmin(p[t], qprime_t[t]);
        total += w[t];
    }
    if (!(denom > 0.0) || !(total > 0.0)) {
        for (int64_t t = 0; t < Vt; ++t) w[t] = p[t];
        return 1;
    }
    for (int64_t t = 0; t < Vt; ++t) w[t] /= denom;
    return 0;
}

/*
 * One TLI verification for B independent sequences.
 *   logits_t [B, K+1, Vt] dense, logits_d [B, K, Vd] dense, tok_d [B,K] draft ids in drafter space,
 *   u_acc [B,K], u_fin [B].
 * Outputs per sequence: accept[K] (every position tested on its own), n_acc = length of the
 * all-accept prefix, out_tok[K+1] = accepted target ids, then the extra token, then -1 padding;
 * p_tok/q_tok [K] = p_k(d_k), q'_k(d_k); lse_p [K+1] (entry K is NaN unless the bonus row was used);
 * lse_q [K]; acc_margin[K] = |u - p/q'| (inf when p >= q'); fin_margin = CDF margin of the extra token.
 * If fin_weights != NULL it receives [B, Vt] the weights the extra token was drawn from.
 * A sequence with a NONFINITE target row among the rows it needs returns n_acc = 0 and out_tok = -1.
 * work must hold 3*Vt + 2*Vd doubles.
 */
void tlo_verify(const void *logits_t, const void *logits_d, int dtype, int64_t B, int64_t K,
                int64_t Vt, int64_t Vd, double tau_t, double tau_d, const int32_t *d2t,
                const int32_t *tok_d, const double *u_acc, const double *u_fin,
                int32_t *n_acc, int32_t *out_tok, uint8_t *accept, double *p_tok, double *q_tok,
                double *lse_p, double *lse_q, int32_t *seq_status, double *acc_margin,
                double *fin_margin, double *fin_weights, double *work) {
    size_t esz = (dtype == TLO_F32) ? 4 : 2;
    double *p = work, *qpt = work + Vt, *w = work + 2 * Vt, *q = work + 3 * Vt, *qp = q + Vd;
    for (int64_t b = 0; b < B; ++b) {
        const char *lt_b = (const char *)logits_t + (size_t)b * (size_t)(K + 1) * (size_t)Vt * esz;
        const char *ld_b = (const char *)logits_d + (size_t)b * (size_t)K * (size_t)Vd * esz;
        int status = 0;
        int first_reject = -1;
        for (int64_t k = 0; k < K; ++k) {
            int64_t o = b * K + k;
            int st_p = tlo_softmax(lt_b + (size_t)k * Vt * esz, dtype, Vt, tau_t, p, &lse_p[b * (K + 1) + k]);
            status |= st_p;
            int32_t d = tok_d[o];
            accept[o] = 0; p_tok[o] = 0.0; q_tok[o] = 0.0; acc_margin[o] = INFINITY; lse_q[o] = NAN;
            if (d < 0 || d >= Vd || d2t[d] < 0) {
                status |= TLO_BAD_DRAFT;
            } else if (!st_p) {
                int st_q = tlo_adjusted_drafter(ld_b + (size_t)k * Vd * esz, dtype, Vd, tau_d, d2t, q, qp, &lse_q[o]);
                if (st_q) {
                    status |= st_q;
                } else {
                    double pd = p[d2t[d]], qd = qp[d];
                    p_tok[o] = pd; q_tok[o] = qd;
                    accept[o] = (u_acc[o] * qd < pd) ? 1 : 0;
                    if (pd < qd) acc_margin[o] = fabs(u_acc[o] - pd / qd);
                }
            }
            if (!accept[o] && first_reject < 0) first_reject = (int)k;
        }
        lse_p[b * (K + 1) + K] = NAN;
        int32_t *out = out_tok + b * (K + 1);
        for (int64_t k = 0; k <= K; ++k) out[k] = -1;
        fin_margin[b] = 0.0;
        if (status & TLO_NONFINITE) {
            n_acc[b] = 0; seq_status[b] = status;
            if (fin_weights) for (int64_t t = 0; t < Vt; ++t) fin_weights[b * Vt + t] = NAN;
            continue;
        }
        int64_t n = (first_reject < 0) ? K : first_reject;
        if (n < K) {
            /* rejected at position n: residual of (p_n, q'_n); q' == 0 if the draft there was unusable */
            tlo_softmax(lt_b + (size_t)n * Vt * esz, dtype, Vt, tau_t, p, &lse_p[b * (K + 1) + n]);
            for (int64_t t = 0; t < Vt; ++t) qpt[t] = 0.0;
            int32_t d = tok_d[b * K + n];
            if (!(d < 0 || d >= Vd || d2t[d] < 0)) {
                double tmp;
                int st_q = tlo_adjusted_drafter(ld_b + (size_t)n * Vd * esz, dtype, Vd, tau_d, d2t, q, qp, &tmp);
                if (!st_q)
                    for (int64_t x = 0; x < Vd; ++x)
                        if (d2t[x] >= 0) qpt[d2t[x]] = qp[x];
            }
            if (residual_weights(p, qpt, Vt, w)) status |= TLO_DEGENERATE;
        } else {
            int st = tlo_softmax(lt_b + (size_t)K * Vt * esz, dtype, Vt, tau_t, w, &lse_p[b * (K + 1) + K]);
            if (st) {
                n_acc[b] = 0; seq_status[b] = status | st;
                if (fin_weights) for (int64_t t = 0; t < Vt; ++t) fin_weights[b * Vt + t] = NAN;
                continue;
            }
        }
        if (fin_weights) memcpy(fin_weights + b * Vt, w, (size_t)Vt * sizeof(double));
        int64_t extra = tlo_inverse_cdf(w, Vt, u_fin[b], &fin_margin[b]);
        for (int64_t k = 0; k < n; ++k) out[k] = d2t[tok_d[b * K + k]];
        out[n] = (int32_t)extra;
        n_acc[b] = (int32_t)n;
        seq_status[b] = status;
    }
}

/* ======================================================================================================
 * Beyond the TLI step: the other token-level pieces of the paper that run on the same rows.
 *   - the "union" algorithm (simple extension of SD to heterogeneous vocabularies): p and q are
 *     extended by zeros to T ∪ D and standard SD is run unchanged;
 *   - the table of expected acceptance rates: sum_{T∩D} min{p, q} (union) and
 *     sum_{T∩D} min{p, q / sum_{T∩D} q} (TLI), and the theorem alpha_union <= alpha_TLI;
 *   - the data-parallel tail of string-level exact matching (SLEM): one token is drawn from each of the
 *     m+1 target rows, the first index where it differs from the re-tokenised draft ends the match;
 *   - temperature zero (the paper runs SLEM at temperature zero): every draw becomes an argmax.
 * ====================================================================================================== */

/*
 * Draft step of the union algorithm: d ~ q = softmax(logits_d / tau_d) over ALL of D (no restriction).
 * tok_t = d2t[d], which is -1 for a token outside T (such a draft is always rejected by the target).
 * lse_q[r] = log sum_{x in D} exp(logit/tau_d).  Every drafter logit takes part: a NaN/+inf anywhere
 * in the row flags it NONFINITE; a row of only -inf is ZERO_MASS.  work: Vd doubles.
 */
void tlo_union_draft_sample(const void *logits_d, int dtype, int64_t row_stride, int64_t R, int64_t Vd,
                            double tau_d, const int32_t *d2t, const double *u_draft, int32_t *tok_d,
                            int32_t *tok_t, double *q_tok, double *lse_q, int32_t *row_status,
                            double *cdf_margin, double *work) {
    size_t esz = (dtype == TLO_F32) ? 4 : 2;
    double *q = work;
    for (int64_t r = 0; r < R; ++r) {
        const void *row = (const char *)logits_d + (size_t)r * (size_t)row_stride * esz;
        int st = tlo_softmax(row, dtype, Vd, tau_d, q, &lse_q[r]);
        if (!st && lse_q[r] == -INFINITY) st = TLO_ZERO_MASS;
        row_status[r] = st;
        tok_d[r] = -1; tok_t[r] = -1; q_tok[r] = 0.0;
        if (cdf_margin) cdf_margin[r] = 0.0;
        if (st) continue;
        double mg;
        int64_t d = tlo_inverse_cdf(q, Vd, u_draft[r], &mg);
        tok_d[r] = (int32_t)d;
        tok_t[r] = d2t[d];
        q_tok[r] = q[d];
        if (cdf_margin) cdf_margin[r] = mg;
    }
}

/*
 * Verification of the union algorithm: standard SD with p' (p on T, 0 on D\T) and q' (q on D, 0 on T\D).
 * A draft outside T has p'(d) = 0 and is rejected for every u; the residual max(0, p' - q') vanishes
 * outside T, so the extra token is a target token.  Same outputs as tlo_verify; q_tok = q(d), lse_q =
 * the normaliser of q over all of D.  BAD_DRAFT only for ids that are not drafter ids at all (< 0 or >= Vd):
 * such a position is rejected with q = 0.  work must hold 3*Vt + Vd doubles.
 */
void tlo_union_verify(const void *logits_t, const void *logits_d, int dtype, int64_t B, int64_t K,
                      int64_t Vt, int64_t Vd, double tau_t, double tau_d, const int32_t *d2t,
                      const int32_t *tok_d, const double *u_acc, const double *u_fin,
                      int32_t *n_acc, int32_t *out_tok, uint8_t *accept, double *p_tok, double *q_tok,
                      double *lse_p, double *lse_q, int32_t *seq_status, double *acc_margin,
                      double *fin_margin, double *fin_weights, double *work) {
    size_t esz = (dtype == TLO_F32) ? 4 : 2;
    double *p = work, *qt = work + Vt, *w = work + 2 * Vt, *q = work + 3 * Vt;
    for (int64_t b = 0; b < B; ++b) {
        const char *lt_b = (const char *)logits_t + (size_t)b * (size_t)(K + 1) * (size_t)Vt * esz;
        const char *ld_b = (const char *)logits_d + (size_t)b * (size_t)K * (size_t)Vd * esz;
        int status = 0, first_reject = -1;
        for (int64_t k = 0; k < K; ++k) {
            int64_t o = b * K + k;
            int st_p = tlo_softmax(lt_b + (size_t)k * Vt * esz, dtype, Vt, tau_t, p, &lse_p[b * (K + 1) + k]);
            status |= st_p;
            int32_t d = tok_d[o];
            accept[o] = 0; p_tok[o] = 0.0; q_tok[o] = 0.0; acc_margin[o] = INFINITY; lse_q[o] = NAN;
            if (d < 0 || d >= Vd) {
                status |= TLO_BAD_DRAFT;
            } else if (!st_p) {
                int st_q = tlo_softmax(ld_b + (size_t)k * Vd * esz, dtype, Vd, tau_d, q, &lse_q[o]);
                if (st_q) {
                    status |= st_q;
                } else {
                    double pd = (d2t[d] >= 0) ? p[d2t[d]] : 0.0, qd = q[d];
                    p_tok[o] = pd; q_tok[o] = qd;
                    accept[o] = (u_acc[o] * qd < pd) ? 1 : 0;
                    if (pd < qd) acc_margin[o] = fabs(u_acc[o] - pd / qd);
                }
            }
            if (!accept[o] && first_reject < 0) first_reject = (int)k;
        }
        lse_p[b * (K + 1) + K] = NAN;
        int32_t *out = out_tok + b * (K + 1);
        for (int64_t k = 0; k <= K; ++k) out[k] = -1;
        fin_margin[b] = 0.0;
        if (status & TLO_NONFINITE) {
            n_acc[b] = 0; seq_status[b] = status;
            if (fin_weights) for (int64_t t = 0; t < Vt; ++t) fin_weights[b * Vt + t] = NAN;
            continue;
        }
        int64_t n = (first_reject < 0) ? K : first_reject;
        if (n < K) {
            tlo_softmax(lt_b + (size_t)n * Vt * esz, dtype, Vt, tau_t, p, &lse_p[b * (K + 1) + n]);
            for (int64_t t = 0; t < Vt; ++t) qt[t] = 0.0;
            int32_t d = tok_d[b * K + n];
            if (!(d < 0 || d >= Vd)) {
                double tmp;
                tlo_softmax(ld_b + (size_t)n * Vd * esz, dtype, Vd, tau_d, q, &tmp);
                for (int64_t x = 0; x < Vd; ++x)
                    if (d2t[x] >= 0) qt[d2t[x]] = q[x];
            }
            if (residual_weights(p, qt, Vt, w)) status |= TLO_DEGENERATE;
        } else {
            int st = tlo_softmax(lt_b + (size_t)K * Vt * esz, dtype, Vt, tau_t, w, &lse_p[b * (K + 1) + K]);
            if (st) {
                n_acc[b] = 0; seq_status[b] = status | st;
                if (fin_weights) for (int64_t t = 0; t < Vt; ++t) fin_weights[b * Vt + t] = NAN;
                continue;
            }
        }
        if (fin_weights) memcpy(fin_weights + b * Vt, w, (size_t)Vt * sizeof(double));
        int64_t extra = tlo_inverse_cdf(w, Vt, u_fin[b], &fin_margin[b]);
        for (int64_t k = 0; k < n; ++k) out[k] = d2t[tok_d[b * K + k]];
        out[n] = (int32_t)extra;
        n_acc[b] = (int32_t)n;
        seq_status[b] = status;
    }
}

/*
 * Expected acceptance rates of one draft token, per row pair (target row r at logits_t + r*stride_t,
 * drafter row r at logits_d + r*stride_d), as the paper's table states them:
 *   alpha_union = sum_{t in T∩D} min{p(t), q(t)}
 *   alpha_tli   = sum_{t in T∩D} min{p(t), q(t) / sum_{x in T∩D} q(x)}
 * status: NONFINITE if a target logit or ANY drafter logit is NaN/+inf (alphas NaN); ZERO_MASS if the
 * shared ids carry no drafter mass (alpha_tli = 0, as for an empty intersection).
 * work must hold Vt + Vd doubles.
 */
void tlo_acceptance_rates(const void *logits_t, int64_t stride_t, const void *logits_d, int64_t stride_d,
                          int dtype, int64_t R, int64_t Vt, int64_t Vd, double tau_t, double tau_d,
                          const int32_t *d2t, double *alpha_tli, double *alpha_union, int32_t *status,
                          double *work) {
    size_t esz = (dtype == TLO_F32) ? 4 : 2;
    double *p = work, *q = work + Vt;
    for (int64_t r = 0; r < R; ++r) {
        const void *lt = (const char *)logits_t + (size_t)r * (size_t)stride_t * esz;
        const void *ld = (const char *)logits_d + (size_t)r * (size_t)stride_d * esz;
        double lp, lq;
        int st = tlo_softmax(lt, dtype, Vt, tau_t, p, &lp) | tlo_softmax(ld, dtype, Vd, tau_d, q, &lq);
        if (st) { status[r] = TLO_NONFINITE; alpha_tli[r] = NAN; alpha_union[r] = NAN; continue; }
        /* q(t) / sum_{x shared} q(x) in log space, as in tlo_adjusted_drafter: exp(z_t - Ms) / Zs */
        double Ms = -INFINITY, Zs = 0.0;
        for (int64_t x = 0; x < Vd; ++x)
            if (d2t[x] >= 0 && load_logit(ld, dtype, x) / tau_d > Ms) Ms = load_logit(ld, dtype, x) / tau_d;
        if (Ms > -INFINITY)
            for (int64_t x = 0; x < Vd; ++x)
                if (d2t[x] >= 0) Zs += exp(load_logit(ld, dtype, x) / tau_d - Ms);
        double au = 0.0, at = 0.0;
        for (int64_t x = 0; x < Vd; ++x) {
            if (d2t[x] < 0) continue;
            au += fmin(p[d2t[x]], q[x]);
            if (Ms > -INFINITY) at += fmin(p[d2t[x]], exp(load_logit(ld, dtype, x) / tau_d - Ms) / Zs);
        }
        alpha_union[r] = au;
        alpha_tli[r] = at;
        status[r] = (Ms > -INFINITY) ? 0 : TLO_ZERO_MASS;
    }
}

/*
 * argmax of a row at temperature zero: the largest logit, the lowest id among equal ones (the limit of
 * the ascending inverse CDF as tau -> 0 puts the draw on the first maximiser for every u below the
 * reciprocal of their number; one convention is needed and this is it).  If `d2t` != NULL only shared ids
 * (d2t[x] >= 0) compete.  Returns -1 with *status = NONFINITE if a competing logit is NaN or +inf,
 * -1 with ZERO_MASS if every competing logit is -inf (or none competes).
 */
int64_t tlo_argmax(const void *logits, int dtype, int64_t n, const int32_t *d2t, int32_t *status) {
    int64_t best = -1;
    double bv = -INFINITY;
    *status = 0;
    for (int64_t x = 0; x < n; ++x) {
        if (d2t && d2t[x] < 0) continue;
        double z = load_logit(logits, dtype, x);
        if (isnan(z) || z == INFINITY) { *status = TLO_NONFINITE; return -1; }
        if (z > bv) { bv = z; best = x; }
    }
    if (best < 0) *status = TLO_ZERO_MASS;
    return best;
}

/*
 * One token from each of R rows: t_r ~ softmax(logits_r / tau) by inverse CDF with u[r], or the argmax
 * when tau == 0.  p_tok[r] = probability of the returned token (1 at tau == 0), lse[r] = log-normaliser
 * (NaN at tau == 0).  Flagged rows return -1.  work: V doubles.
 */
void tlo_sample_rows(const void *logits, int dtype, int64_t row_stride, int64_t R, int64_t V, double tau,
                     const double *u, int32_t *tok, double *p_tok, double *lse, int32_t *status,
                     double *cdf_margin, double *work) {
    size_t esz = (dtype == TLO_F32) ? 4 : 2;
    for (int64_t r = 0; r < R; ++r) {
        const void *row = (const char *)logits + (size_t)r * (size_t)row_stride * esz;
        tok[r] = -1; p_tok[r] = 0.0; lse[r] = NAN;
        if (cdf_margin) cdf_margin[r] = 0.0;
        if (tau == 0.0) {
            int32_t st;
            int64_t t = tlo_argmax(row, dtype, V, NULL, &st);
            status[r] = st;
            if (!st) { tok[r] = (int32_t)t; p_tok[r] = 1.0; }
            continue;
        }
        int st = tlo_softmax(row, dtype, V, tau, work, &lse[r]);
        if (!st && lse[r] == -INFINITY) st = TLO_ZERO_MASS;
        status[r] = st;
        if (st) continue;
        double mg;
        int64_t t = tlo_inverse_cdf(work, V, u[r], &mg);
        tok[r] = (int32_t)t;
        p_tok[r] = work[t];
        if (cdf_margin) cdf_margin[r] = mg;
    }
}

/*
 * Tail of string-level exact matching for B sequences: target rows [B, m+1, Vt], re-tokenised drafts
 * draft_t [B, m] (target ids; a negative entry = no draft token there).  t'_j is drawn from row j for all
 * j = 1..m+1 (tau_t == 0: argmax); j* = first j with t'_j != draft_j (m+1 if none); output
 * draft_1..draft_{j*-1}, t'_{j*}; n_acc = j* - 1.  tgt_tok [B, m+1] receives every t'_j.
 * A NONFINITE / ZERO_MASS row among the m+1 flags the sequence: n_acc = 0, out_tok = -1.
 * With tau_t == 0 and draft_t = the target ids of greedy TLI drafts this is TLI's verification at
 * temperature zero (accept iff the draft is the target's argmax; the extra token is the argmax of the
 * first rejected row, or of row m+1).  work: Vt doubles.
 */
void tlo_exact_match_verify(const void *logits_t, int dtype, int64_t B, int64_t m, int64_t Vt, double tau_t,
                            const int32_t *draft_t, const double *u, int32_t *n_acc, int32_t *out_tok,
                            int32_t *tgt_tok, int32_t *seq_status, double *cdf_margin, double *work) {
    size_t esz = (dtype == TLO_F32) ? 4 : 2;
    for (int64_t b = 0; b < B; ++b) {
        const char *lt_b = (const char *)logits_t + (size_t)b * (size_t)(m + 1) * (size_t)Vt * esz;
        int32_t *tt = tgt_tok + b * (m + 1);
        int32_t *out = out_tok + b * (m + 1);
        int status = 0;
        for (int64_t j = 0; j <= m; ++j) {
            double pt, l;
            int32_t st;
            tlo_sample_rows(lt_b + (size_t)j * Vt * esz, dtype, Vt, 1, Vt, tau_t, &u[b * (m + 1) + j], &tt[j], &pt, &l,
                            &st, cdf_margin ? &cdf_margin[b * (m + 1) + j] : NULL, work);
            status |= st;
            out[j] = -1;
        }
        seq_status[b] = status;
        n_acc[b] = 0;
        if (status) continue;
        int64_t j = 0;
        while (j < m && draft_t[b * m + j] >= 0 && draft_t[b * m + j] == tt[j]) ++j;
        for (int64_t k = 0; k < j; ++k) out[k] = draft_t[b * m + k];
        out[j] = tt[j];
        n_acc[b] = (int32_t)j;
    }
}

/*
 * Greedy draft of TLI (temperature zero): d = argmax of the drafter row over the SHARED ids, lowest id on
 * ties; tok_t = d2t[d].  Flagged rows (NONFINITE / ZERO_MASS among the shared logits) return -1.
 */
void tlo_greedy_draft(const void *logits_d, int dtype, int64_t row_stride, int64_t R, int64_t Vd,
                      const int32_t *d2t, int32_t *tok_d, int32_t *tok_t, int32_t *row_status) {
    size_t esz = (dtype == TLO_F32) ? 4 : 2;
    for (int64_t r = 0; r < R; ++r) {
        const void *row = (const char *)logits_d + (size_t)r * (size_t)row_stride * esz;
        int32_t st;
        int64_t d = tlo_argmax(row, dtype, Vd, d2t, &st);
        row_status[r] = st;
        tok_d[r] = (int32_t)d;
        tok_t[r] = (d >= 0) ? d2t[d] : -1;
    }
}

/* ======================================================================================================
 * Logit warpers ahead of the softmax (top-k, top-p).  The paper does not use them (its runs are plain
 * temperature sampling, or temperature zero); they are the standard serving knobs around the same softmax
 * and are defined here by value thresholds so that the result does not depend on any sort order:
 *   top-k : keep the ids whose logit is >= the k-th largest competing logit (equal logits at the
 *           threshold are all kept, so more than k ids may survive);
 *   top-p : on the distribution that survived top-k (renormalised), keep id x iff the probability mass of
 *           the ids with a strictly larger logit is < top_p -- the smallest top set whose mass reaches
 *           top_p, with equal logits kept or dropped together.  The largest logit is always kept.
 * A dropped id gets logit -inf, i.e. probability zero in every later step.
 * ====================================================================================================== */
typedef struct { double v; } tlo_val;
static int cmp_desc(const void *a, const void *b) {
    double x = ((const tlo_val *)a)->v, y = ((const tlo_val *)b)->v;
    return (x < y) - (x > y);
}

/*
 * For each of R rows: threshold thr[r] (a logit value; -inf if nothing is dropped), kept[r] = number of
 * surviving ids, keep_mask[r*V + x] in {0,1}; margin[r] = distance of the top-p decision from flipping:
 * min over the two neighbouring cut positions of |mass_above / Z_k - top_p| (inf if top-p is off).
 * d2t != NULL: only ids with d2t[x] >= 0 compete, the others are dropped outright.
 * top_k <= 0 switches top-k off, top_p >= 1 switches top-p off.  tau > 0.
 * status: NONFINITE if a competing logit is NaN/+inf, ZERO_MASS if none competes or all are -inf (then
 * nothing is kept, thr = NaN).  work: V tlo_val-sized doubles.
 */
void tlo_warp_rows(const void *logits, int dtype, int64_t row_stride, int64_t R, int64_t V, double tau,
                   const int32_t *d2t, int64_t top_k, double top_p, double *thr, int32_t *kept,
                   uint8_t *keep_mask, int32_t *status, double *margin, double *work) {
    size_t esz = (dtype == TLO_F32) ? 4 : 2;
    tlo_val *s = (tlo_val *)work;
    for (int64_t r = 0; r < R; ++r) {
        const void *row = (const char *)logits + (size_t)r * (size_t)row_stride * esz;
        int64_t n = 0;
        int bad = 0;
        for (int64_t x = 0; x < V; ++x) {
            keep_mask[r * V + x] = 0;
            if (d2t && d2t[x] < 0) continue;
            double z = load_logit(row, dtype, x);
            if (isnan(z) || z == INFINITY) bad = 1;
            if (z > -INFINITY) s[n++].v = z;
        }
        thr[r] = NAN; kept[r] = 0; margin[r] = INFINITY;
        if (bad) { status[r] = TLO_NONFINITE; continue; }
        if (n == 0) { status[r] = TLO_ZERO_MASS; continue; }
        status[r] = 0;
        qsort(s, (size_t)n, sizeof(tlo_val), cmp_desc);
        /* top-k: value of the k-th largest, all ties kept */
        int64_t nk = n;
        double th = -INFINITY;
        if (top_k > 0 && top_k < n) {
            th = s[top_k - 1].v;
            nk = top_k;
            while (nk < n && s[nk].v == th) ++nk;
        }
        /* top-p on the survivors */
        if (top_p < 1.0) {
            double M = s[0].v / tau, Z = 0.0;
            for (int64_t i = 0; i < nk; ++i) Z += exp(s[i].v / tau - M);
            double above = 0.0;   /* mass of strictly larger logits, as a fraction of Z */
            int64_t i = 0, cut = nk;
            double best_margin = INFINITY;
            while (i < nk) {
                int64_t j = i;
                double g = 0.0;
                while (j < nk && s[j].v == s[i].v) { g += exp(s[j].v / tau - M); ++j; }
                double frac = above / Z;
                if (i > 0 && fabs(frac - top_p) < best_margin) best_margin = fabs(frac - top_p);
                if (!(frac < top_p)) { cut = i; break; }
                above += g;
                i = j;
            }
            margin[r] = best_margin;
            if (cut < nk) { nk = cut; th = s[cut - 1].v; }
        }
        thr[r] = th;
        kept[r] = (int32_t)nk;
        for (int64_t x = 0; x < V; ++x) {
            if (d2t && d2t[x] < 0) continue;
            double z = load_logit(row, dtype, x);
            keep_mask[r * V + x] = (z > -INFINITY && z >= th) ? 1 : 0;
        }
    }
}
