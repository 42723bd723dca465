/*
 * Token-by-token fp64 oracle for Kaczmarz Linear Attention.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what
 * the GPU library must compute.  It is called from tests, from the smoke check
 * and from the CPU-baseline leg of the benchmark; the product path never links
 * or calls it, and it shares no code, header or table with the HIP sources.
 *
 * What it follows: the tokenwise update of Algorithm 1 (left panel) with the
 * coefficient of eq. (3), in the order the algorithm lists the lines:
 *     decay  ->  residual against the decayed state  ->  beta  ->  rank-one
 *     write  ->  read from the updated state.
 * Readings taken where the paper leaves a choice:
 *   - the readout is o_t = S_t^T q_t on q as given (the l2 normalisation of q
 *     named in Sec. 3.3 is linear in q and left to the caller);
 *   - the decay gate is passed as its natural logarithm, alpha = exp(log_alpha);
 *   - if ||k||^2 + eps == 0 (zero key, eps = 0) then beta := 0: the write
 *     beta k e^T vanishes for every finite beta, so this is its continuous
 *     completion.
 * State layout: S is d_k x d_v, row-major (d_v contiguous), as in Sec. 2.
 * All arithmetic is IEEE double; q, k, v arrive as float (a bf16 or fp32 input
 * widens to float, and float to double, without rounding).  Plain loops, naive
 * summation order, no blocking.
 *
 * Two options, both off in the plain entry points (the *_opts entry points take
 * them):
 *   - normalize_q: the readout of Sec. 3.3 / Algorithm 1 (left) as printed,
 *     o_t = S_t^T q_t / ||q_t||; a zero query gives o_t = 0 (S^T 0 = 0);
 *   - gdn_beta: beta_t = eta_t, the gated delta rule the paper starts from
 *     (Table 2; the "w/o normalization" row of the ablation), i.e. eq. (3)
 *     without the key-norm denominator.
 *
 * Pins: see tests/test_oracle_pins.py (Theorem 1 projection property,
 * Proposition 2 contraction factor, Proposition 1 stationarity, eq. (4) line
 * search, pure decay at eta = 0, brute-force product form of Table 5, textbook
 * Kaczmarz limits checked against numpy's pseudo-inverse, a hand-worked
 * rational example under tests/golden/).
 *
 * Diagonal gating (the *_diag entry points): the decay operator of line 1 is
 * D_t = diag(alpha_t) with one decay per key channel (App. B, "Extension to
 * diagonal gating"; the decay-agnostic remark of App. A), S~ = diag(alpha_t) S,
 * i.e. row i of the d_k x d_v state is scaled by alpha_t[i].  Lines 2-5 are
 * unchanged.  log_alpha then has d_k entries per token and head.
 *
 * Gradients (kla_oracle_sequence_bwd): the paper states the forward map only and
 * mentions training without deriving a backward pass, so the gradient oracle is
 * the plain reverse accumulation through the same five lines of Algorithm 1
 * (left), token by token from the last to the first, including the dependence of
 * beta on k through eq. (3).  Its pins are central finite differences of the
 * forward oracle above and closed forms for a single step and for eta = 0.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

/* One token of Algorithm 1 (left) on one head.  S is updated in place; o gets
 * d_v outputs; e is caller-provided scratch of d_v doubles. */
static void kla_token(double *S, const float *q, const float *k, const float *v,
                      double log_alpha, double eta, double eps, int dk, int dv,
                      double *o, double *e, int normalize_q, int gdn_beta)
{
    int i, j;
    /* line 1: S~ = alpha S */
    const double alpha = exp(log_alpha);
    for (i = 0; i < dk; ++i)
        for (j = 0; j < dv; ++j)
            S[(size_t)i * dv + j] *= alpha;
    /* line 2: e = v - S~^T k */
    for (j = 0; j < dv; ++j) {
        double p = 0.0;
        for (i = 0; i < dk; ++i)
            p += S[(size_t)i * dv + j] * (double)k[i];
        e[j] = (double)v[j] - p;
    }
    /* line 3 / eq. (3): beta = eta / (||k||^2 + eps) */
    double nk = 0.0;
    for (i = 0; i < dk; ++i)
        nk += (double)k[i] * (double)k[i];
    const double den = nk + eps;
    double beta = (den == 0.0) ? 0.0 : eta / den;
    if (gdn_beta)                 /* the delta rule without the Kaczmarz denominator */
        beta = eta;
    /* line 4: S = S~ + beta k e^T */
    for (i = 0; i < dk; ++i)
        for (j = 0; j < dv; ++j)
            S[(size_t)i * dv + j] += beta * (double)k[i] * e[j];
    /* line 5 (without the division by ||q||): o = S^T q */
    for (j = 0; j < dv; ++j) {
        double r = 0.0;
        for (i = 0; i < dk; ++i)
            r += S[(size_t)i * dv + j] * (double)q[i];
        o[j] = r;
    }
    if (normalize_q) {            /* line 5 as printed: o = S^T q / ||q|| */
        double nq = 0.0;
        for (i = 0; i < dk; ++i)
            nq += (double)q[i] * (double)q[i];
        nq = sqrt(nq);
        for (j = 0; j < dv; ++j)
            o[j] = (nq == 0.0) ? 0.0 : o[j] / nq;
    }
}

/*
 * Runs one (sequence, head) unit.
 *   q, k      [n_tokens_total, H, dk]   float
 *   v         [n_tokens_total, H, dv]   float
 *   log_alpha, eta [n_tokens_total, H]  double
 *   h0        [dk, dv] double for this unit, or NULL for zeros
 *   o         [n_tokens_total, H, dv]   double (only this unit's rows written)
 *   hT        [dk, dv] double for this unit (out), may be NULL
 *   t0, len   first token and token count of the sequence in the token axis
 *   h         head index
 * Returns 0, or -1 if scratch could not be allocated.
 */
int kla_oracle_sequence_opts(const float *q, const float *k, const float *v,
                             const double *log_alpha, const double *eta, double eps,
                             const double *h0, double *o, double *hT,
                             long t0, long len, int h, int H, int dk, int dv,
                             int normalize_q, int gdn_beta)
{
    double *S = (double *)malloc(sizeof(double) * (size_t)dk * dv);
    double *e = (double *)malloc(sizeof(double) * (size_t)dv);
    if (!S || !e) { free(S); free(e); return -1; }
    if (h0) memcpy(S, h0, sizeof(double) * (size_t)dk * dv);
    else    memset(S, 0, sizeof(double) * (size_t)dk * dv);
    for (long t = t0; t < t0 + len; ++t) {
        const size_t th = (size_t)t * H + h;
        kla_token(S, q + th * dk, k + th * dk, v + th * dv,
                  log_alpha[th], eta[th], eps, dk, dv, o + th * dv, e, normalize_q, gdn_beta);
    }
    if (hT) memcpy(hT, S, sizeof(double) * (size_t)dk * dv);
    free(S); free(e);
    return 0;
}

int kla_oracle_sequence(const float *q, const float *k, const float *v,
                        const double *log_alpha, const double *eta, double eps,
                        const double *h0, double *o, double *hT,
                        long t0, long len, int h, int H, int dk, int dv)
{
    return kla_oracle_sequence_opts(q, k, v, log_alpha, eta, eps, h0, o, hT, t0, len, h, H, dk, dv, 0, 0);
}

/*
 * One decode step for one (batch, head) unit: a single iteration of the same
 * loop body starting from the given state.  S [dk, dv] double is updated in
 * place, o [dv] double is written.  Returns 0 or -1.
 */
int kla_oracle_decode_unit_opts(const float *q, const float *k, const float *v,
                                double log_alpha, double eta, double eps,
                                double *S, double *o, int dk, int dv,
                                int normalize_q, int gdn_beta)
{
    double *e = (double *)malloc(sizeof(double) * (size_t)dv);
    if (!e) return -1;
    kla_token(S, q, k, v, log_alpha, eta, eps, dk, dv, o, e, normalize_q, gdn_beta);
    free(e);
    return 0;
}

int kla_oracle_decode_unit(const float *q, const float *k, const float *v,
                           double log_alpha, double eta, double eps,
                           double *S, double *o, int dk, int dv)
{
    return kla_oracle_decode_unit_opts(q, k, v, log_alpha, eta, eps, S, o, dk, dv, 0, 0);
}

/* Forward lines 1-4 of Algorithm 1 (left) for one token, out of place: Snew = alpha S + beta k e^T.
 * Returns beta and 1/(||k||^2 + eps) (0 if the denominator is 0); St gets the decayed state alpha S, e the residual;
 * Snew may be NULL when only those are wanted. */
static double kla_token_state(const double *S, const float *k, const float *v, double log_alpha, double eta,
                              double eps, int dk, int dv, double *St, double *e, double *Snew, double *inv_den,
                              int gdn_beta)
{
    int i, j;
    const double alpha = exp(log_alpha);
    for (i = 0; i < dk * dv; ++i) St[i] = alpha * S[i];
    for (j = 0; j < dv; ++j) {
        double p = 0.0;
        for (i = 0; i < dk; ++i) p += St[(size_t)i * dv + j] * (double)k[i];
        e[j] = (double)v[j] - p;
    }
    double nk = 0.0;
    for (i = 0; i < dk; ++i) nk += (double)k[i] * (double)k[i];
    const double den = nk + eps;
    *inv_den = (den == 0.0) ? 0.0 : 1.0 / den;
    if (gdn_beta) *inv_den = 1.0;                /* beta = eta: the coefficient does not see the key */
    const double beta = eta * *inv_den;
    if (Snew)
        for (i = 0; i < dk; ++i)
            for (j = 0; j < dv; ++j)
                Snew[(size_t)i * dv + j] = St[(size_t)i * dv + j] + beta * (double)k[i] * e[j];
    return beta;
}

/*
 * Gradient of  L = sum_t <d_o[t], o_t> + <d_hT, h_T>  for one (sequence, head) unit of
 * kla_oracle_sequence (no options), by reverse accumulation through Algorithm 1 (left).
 *   d_o               [n_tokens_total, H, dv] double
 *   d_hT              [dk, dv] double for this unit, or NULL for zeros
 *   dq, dk_           [n_tokens_total, H, dk] double (only this unit's rows written)
 *   dv_               [n_tokens_total, H, dv] double
 *   dlog_alpha, deta  [n_tokens_total, H]     double
 *   dh0               [dk, dv] double for this unit (out), may be NULL
 * The states are recomputed from checkpoints kept every 64 tokens, so memory stays at
 * (len/64 + 65) states.  normalize_q: the read-out is o_t = S_t^T q_t / ||q_t||.  gdn_beta: beta_t = eta_t (no
 * dependence on k).  Returns 0, or -1 if memory could not be
 * allocated.
 */
int kla_oracle_sequence_bwd_opts(const float *q, const float *k, const float *v,
                                 const double *log_alpha, const double *eta, double eps,
                                 const double *h0, const double *d_o, const double *d_hT,
                                 double *dq, double *dk_, double *dv_, double *dlog_alpha, double *deta,
                                 double *dh0, long t0, long len, int h, int H, int dk, int dv,
                                 int normalize_q, int gdn_beta)
{
    enum { SEG = 64 };
    const size_t sz = (size_t)dk * dv;
    const long nseg = (len + SEG - 1) / SEG;
    double *chk = (double *)malloc(sizeof(double) * sz * (size_t)(nseg + 1));
    double *st = (double *)malloc(sizeof(double) * sz * (SEG + 1));
    double *St = (double *)malloc(sizeof(double) * sz);
    double *dS = (double *)malloc(sizeof(double) * sz);
    double *e = (double *)malloc(sizeof(double) * (size_t)dv);
    double *de = (double *)malloc(sizeof(double) * (size_t)dv);
    if (!chk || !st || !St || !dS || !e || !de) { free(chk); free(st); free(St); free(dS); free(e); free(de); return -1; }
    int i, j;
    double inv_den;

    /* forward sweep: the state at every segment start */
    if (h0) memcpy(chk, h0, sizeof(double) * sz);
    else    memset(chk, 0, sizeof(double) * sz);
    for (long sg = 0; sg < nseg; ++sg) {
        memcpy(st, chk + sz * (size_t)sg, sizeof(double) * sz);
        const long a = t0 + sg * SEG, b = (a + SEG < t0 + len) ? a + SEG : t0 + len;
        for (long t = a; t < b; ++t) {
            const size_t th = (size_t)t * H + h;
            kla_token_state(st, k + th * dk, v + th * dv, log_alpha[th], eta[th], eps, dk, dv, St, e, st + sz, &inv_den, gdn_beta);
            memcpy(st, st + sz, sizeof(double) * sz);
        }
        memcpy(chk + sz * (size_t)(sg + 1), st, sizeof(double) * sz);
    }

    /* reverse sweep */
    if (d_hT) memcpy(dS, d_hT, sizeof(double) * sz);
    else      memset(dS, 0, sizeof(double) * sz);
    for (long sg = nseg - 1; sg >= 0; --sg) {
        const long a = t0 + sg * SEG, b = (a + SEG < t0 + len) ? a + SEG : t0 + len;
        /* st[i] = state before token a + i, st[i + 1] = state after it */
        memcpy(st, chk + sz * (size_t)sg, sizeof(double) * sz);
        for (long t = a; t < b; ++t) {
            const size_t th = (size_t)t * H + h;
            kla_token_state(st + sz * (size_t)(t - a), k + th * dk, v + th * dv, log_alpha[th], eta[th], eps, dk, dv,
                            St, e, st + sz * (size_t)(t - a + 1), &inv_den, gdn_beta);
        }
        for (long t = b - 1; t >= a; --t) {
            const size_t th = (size_t)t * H + h;
            const float *qt = q + th * dk, *kt = k + th * dk, *vt = v + th * dv;
            const double *go = d_o + th * dv;
            const double *Sprev = st + sz * (size_t)(t - a), *Scur = st + sz * (size_t)(t - a + 1);
            double *gq = dq + th * dk, *gk = dk_ + th * dk, *gv = dv_ + th * dv;
            /* line 5: o = S^T q, or o = S^T q / ||q|| (a zero query: o = 0, nothing flows back).
             * With r = S^T q and n = ||q||:  dr = go / n,  dn = -<go, r> / n^2,  dq = S dr + dn q / n. */
            double rn = 1.0, dn_over_n = 0.0;
            if (normalize_q) {
                double nq = 0.0, gr = 0.0;
                for (i = 0; i < dk; ++i) nq += (double)qt[i] * (double)qt[i];
                nq = sqrt(nq);
                rn = (nq == 0.0) ? 0.0 : 1.0 / nq;
                for (j = 0; j < dv; ++j) {
                    double r = 0.0;
                    for (i = 0; i < dk; ++i) r += Scur[(size_t)i * dv + j] * (double)qt[i];
                    gr += go[j] * r;
                }
                dn_over_n = -gr * rn * rn * rn;
            }
            for (i = 0; i < dk; ++i) {
                double acc = 0.0;
                for (j = 0; j < dv; ++j) {
                    acc += Scur[(size_t)i * dv + j] * go[j] * rn;
                    dS[(size_t)i * dv + j] += (double)qt[i] * go[j] * rn;
                }
                gq[i] = acc + dn_over_n * (double)qt[i];
            }
            /* the forward quantities of this token again: decayed state, residual, beta */
            const double beta = kla_token_state(Sprev, kt, vt, log_alpha[th], eta[th], eps, dk, dv, St, e, NULL, &inv_den, gdn_beta);
            /* line 4: S = S~ + beta k e^T */
            double dbeta = 0.0;
            for (j = 0; j < dv; ++j) de[j] = 0.0;
            for (i = 0; i < dk; ++i) {
                double acc = 0.0;
                for (j = 0; j < dv; ++j) {
                    acc += dS[(size_t)i * dv + j] * e[j];
                    de[j] += dS[(size_t)i * dv + j] * (double)kt[i];
                }
                dbeta += (double)kt[i] * acc;
                gk[i] = beta * acc;
            }
            for (j = 0; j < dv; ++j) de[j] *= beta;
            /* line 2: e = v - S~^T k   (dS becomes the gradient of the decayed state) */
            for (j = 0; j < dv; ++j) gv[j] = de[j];
            for (i = 0; i < dk; ++i) {
                double acc = 0.0;
                for (j = 0; j < dv; ++j) {
                    acc += St[(size_t)i * dv + j] * de[j];
                    dS[(size_t)i * dv + j] -= (double)kt[i] * de[j];
                }
                gk[i] -= acc;
            }
            /* line 3 / eq. (3): beta = eta / (||k||^2 + eps) */
            deta[th] = dbeta * inv_den;
            if (!gdn_beta)
                for (i = 0; i < dk; ++i) gk[i] -= 2.0 * beta * dbeta * inv_den * (double)kt[i];
            /* line 1: S~ = alpha S, alpha = exp(log_alpha) */
            double dla = 0.0;
            const double alpha = exp(log_alpha[th]);
            for (i = 0; i < dk * dv; ++i) { dla += dS[i] * St[i]; dS[i] *= alpha; }
            dlog_alpha[th] = dla;
        }
    }
    if (dh0) memcpy(dh0, dS, sizeof(double) * sz);
    free(chk); free(st); free(St); free(dS); free(e); free(de);
    return 0;
}

/* One token with diagonal gating: row i of S decays by exp(log_alpha[i]); lines 2-5 as in kla_token. */
static void kla_token_diag(double *S, const float *q, const float *k, const float *v,
                           const double *log_alpha, double eta, double eps, int dk, int dv,
                           double *o, double *e, int normalize_q, int gdn_beta)
{
    int i, j;
    /* line 1 with D_t = diag(alpha_t): S~ = diag(alpha) S */
    for (i = 0; i < dk; ++i) {
        const double alpha = exp(log_alpha[i]);
        for (j = 0; j < dv; ++j)
            S[(size_t)i * dv + j] *= alpha;
    }
    /* line 2: e = v - S~^T k */
    for (j = 0; j < dv; ++j) {
        double p = 0.0;
        for (i = 0; i < dk; ++i)
            p += S[(size_t)i * dv + j] * (double)k[i];
        e[j] = (double)v[j] - p;
    }
    /* line 3 / eq. (3) */
    double nk = 0.0;
    for (i = 0; i < dk; ++i)
        nk += (double)k[i] * (double)k[i];
    const double den = nk + eps;
    double beta = (den == 0.0) ? 0.0 : eta / den;
    if (gdn_beta) beta = eta;                    /* the gated delta rule: no key-norm denominator */
    /* line 4: S = S~ + beta k e^T */
    for (i = 0; i < dk; ++i)
        for (j = 0; j < dv; ++j)
            S[(size_t)i * dv + j] += beta * (double)k[i] * e[j];
    /* line 5: o = S^T q, or as printed o = S^T q / ||q|| (a zero query gives 0) */
    for (j = 0; j < dv; ++j) {
        double r = 0.0;
        for (i = 0; i < dk; ++i)
            r += S[(size_t)i * dv + j] * (double)q[i];
        o[j] = r;
    }
    if (normalize_q) {
        double nq = 0.0;
        for (i = 0; i < dk; ++i)
            nq += (double)q[i] * (double)q[i];
        nq = sqrt(nq);
        for (j = 0; j < dv; ++j)
            o[j] = (nq == 0.0) ? 0.0 : o[j] / nq;
    }
}

/* kla_oracle_sequence with diagonal gating: log_alpha is [n_tokens_total, H, dk]; everything else as there. */
int kla_oracle_sequence_diag_opts(const float *q, const float *k, const float *v,
                                  const double *log_alpha, const double *eta, double eps,
                                  const double *h0, double *o, double *hT,
                                  long t0, long len, int h, int H, int dk, int dv, int normalize_q, int gdn_beta)
{
    double *S = (double *)malloc(sizeof(double) * (size_t)dk * dv);
    double *e = (double *)malloc(sizeof(double) * (size_t)dv);
    if (!S || !e) { free(S); free(e); return -1; }
    if (h0) memcpy(S, h0, sizeof(double) * (size_t)dk * dv);
    else    memset(S, 0, sizeof(double) * (size_t)dk * dv);
    for (long t = t0; t < t0 + len; ++t) {
        const size_t th = (size_t)t * H + h;
        kla_token_diag(S, q + th * dk, k + th * dk, v + th * dv, log_alpha + th * dk, eta[th], eps, dk, dv,
                       o + th * dv, e, normalize_q, gdn_beta);
    }
    if (hT) memcpy(hT, S, sizeof(double) * (size_t)dk * dv);
    free(S); free(e);
    return 0;
}

int kla_oracle_sequence_diag(const float *q, const float *k, const float *v,
                             const double *log_alpha, const double *eta, double eps,
                             const double *h0, double *o, double *hT,
                             long t0, long len, int h, int H, int dk, int dv)
{
    return kla_oracle_sequence_diag_opts(q, k, v, log_alpha, eta, eps, h0, o, hT, t0, len, h, H, dk, dv, 0, 0);
}

/* One decode step with diagonal gating: log_alpha has dk entries. */
int kla_oracle_decode_unit_diag_opts(const float *q, const float *k, const float *v,
                                     const double *log_alpha, double eta, double eps,
                                     double *S, double *o, int dk, int dv, int normalize_q, int gdn_beta)
{
    double *e = (double *)malloc(sizeof(double) * (size_t)dv);
    if (!e) return -1;
    kla_token_diag(S, q, k, v, log_alpha, eta, eps, dk, dv, o, e, normalize_q, gdn_beta);
    free(e);
    return 0;
}

int kla_oracle_decode_unit_diag(const float *q, const float *k, const float *v,
                                const double *log_alpha, double eta, double eps,
                                double *S, double *o, int dk, int dv)
{
    return kla_oracle_decode_unit_diag_opts(q, k, v, log_alpha, eta, eps, S, o, dk, dv, 0, 0);
}

/* The gradient for the plain recurrence (beta of eq. (3)). */
int kla_oracle_sequence_bwd(const float *q, const float *k, const float *v,
                            const double *log_alpha, const double *eta, double eps,
                            const double *h0, const double *d_o, const double *d_hT,
                            double *dq, double *dk_, double *dv_, double *dlog_alpha, double *deta,
                            double *dh0, long t0, long len, int h, int H, int dk, int dv)
{
    return kla_oracle_sequence_bwd_opts(q, k, v, log_alpha, eta, eps, h0, d_o, d_hT, dq, dk_, dv_, dlog_alpha, deta, dh0,
                                        t0, len, h, H, dk, dv, 0, 0);
}
