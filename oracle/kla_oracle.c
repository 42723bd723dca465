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
