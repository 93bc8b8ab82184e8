/*
 * CPU oracle for the dual-state linear attention (DSLA) layer forward.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * layer computes, used to check the GPU library.  It shares no code with the
 * GPU library and the library never calls it.
 *
 * Everything is fp64.  All (batch, head) pairs are independent; OpenMP is used
 * over that pair index only, so the arithmetic inside one pair is the plain
 * sequential definition.
 *
 * Notation (paper, Section 4.1 "Dual-State Linear Attention"):
 *   q_t, k_t : row vectors of length dk      v_t, o_t : row vectors of length dv
 *   S1, S2   : dk x dv states (history, recency)
 *   G^i_t    : forget gate of state i; here the gate is a per-token vector
 *              alpha^i_t in (0,1]^dk broadcast along dv (the outer-product form
 *              of the background section with the second vector fixed to ones).
 *              Gates are passed as natural logarithms  g^i_t = log alpha^i_t <= 0.
 *   gamma    : blend coefficient of the layer (one value per head is accepted so
 *              that a per-layer scalar is the special case of equal entries).
 *
 * Tensor layouts (all contiguous, last index fastest):
 *   q, k, g1, g2 : [B][T][H][dk]      v, o : [B][T][H][dv]
 *   S1, S2       : [B][H][dk][dv]     gamma : [H]
 *
 * Parity pins (tests/test_oracle_pins.py): hand-computed d=1 example, the
 * geometric closed form for constant gates, the ungated case against a
 * library matmul of tril(QK^T)V, the per-head scalar-gate masked-matmul form,
 * agreement of the recurrence with the unrolled attention-score form, state
 * disabling (gamma in {0,1}, equal gates), linearity and continuation.
 * dsla_oracle_nstate (N states, outer-product gate, grouped key/value heads): a
 * hand-computed d=1 example with both gate vectors, bit-equality with
 * dsla_oracle_recurrent for N = 2 without a beta gate, brute-force loops, the
 * unrolled form with both gate vectors, the geometric closed form with ratio
 * alpha_d beta_j, linearity in the blend, grouped heads against repeated heads.
 * The blend of more than two states is a reading (the paper prints two): that
 * choice is unpinned by the paper, the function itself is pinned as listed.
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int dsla_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Token-by-token recurrence.
 *
 * Section 4.1, state-update equation: each state decays by its own gate and
 * then takes the outer product k_t^T v_t,
 *     S^i_t = diag(alpha^i_t) S^i_{t-1} + k_t^T v_t,   i = 1, 2,
 * (each state recurs on itself: the unrolled form of the same section uses
 * only gate-1 products for state 1 and only gate-2 products for state 2).
 * Section 4.1, read-out equation, evaluated on the already updated states:
 *     o_t = scale * q_t ( gamma S^1_t + (1 - gamma) S^2_t ).
 *
 * S1, S2 hold the initial states on entry and the final states on return.
 * T = 0 leaves everything untouched.  A decode step is the call with T = 1.
 */
void dsla_oracle_recurrent(int B, int T, int H, int dk, int dv,
                           const double *q, const double *k, const double *v,
                           const double *g1, const double *g2,
                           const double *gamma, double scale,
                           double *S1, double *S2, double *o)
{
    const int BH = B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < BH; ++bh) {
        const int b = bh / H, h = bh % H;
        double *s1 = S1 + (size_t)bh * dk * dv;
        double *s2 = S2 + (size_t)bh * dk * dv;
        const double gm = gamma[h];
        for (int t = 0; t < T; ++t) {
            const size_t rk = (((size_t)b * T + t) * H + h) * (size_t)dk;
            const size_t rv = (((size_t)b * T + t) * H + h) * (size_t)dv;
            const double *qt = q + rk, *kt = k + rk, *vt = v + rv;
            const double *g1t = g1 + rk, *g2t = g2 + rk;
            double *ot = o + rv;
            for (int d = 0; d < dk; ++d) {
                const double a1 = exp(g1t[d]);
                const double a2 = exp(g2t[d]);
                for (int j = 0; j < dv; ++j) {
                    s1[(size_t)d * dv + j] = a1 * s1[(size_t)d * dv + j] + kt[d] * vt[j];
                    s2[(size_t)d * dv + j] = a2 * s2[(size_t)d * dv + j] + kt[d] * vt[j];
                }
            }
            for (int j = 0; j < dv; ++j) {
                double acc = 0.0;
                for (int d = 0; d < dk; ++d)
                    acc += qt[d] * (gm * s1[(size_t)d * dv + j] + (1.0 - gm) * s2[(size_t)d * dv + j]);
                ot[j] = scale * acc;
            }
        }
    }
}

/*
 * Unrolled "attention score" form, zero initial states.
 *
 * Section 4.1, last display (and the single-state version in Section 3):
 * for the query at position t, token s <= t receives the weight
 *     sum_d  q_t[d] k_s[d] ( gamma * prod_{tau=s+1..t} alpha^1_tau[d]
 *                          + (1-gamma) * prod_{tau=s+1..t} alpha^2_tau[d] ),
 * the empty product (s = t) being one, and  o_t = scale * sum_s weight * v_s.
 * The paper writes this for the last query only; here it is applied to every
 * query position.  The gate products are formed by literal multiplication of
 * the per-token gates, walking s downwards from t.  O(T^2) per head: small
 * inputs only.
 */
void dsla_oracle_unrolled(int B, int T, int H, int dk, int dv,
                          const double *q, const double *k, const double *v,
                          const double *g1, const double *g2,
                          const double *gamma, double scale, double *o)
{
    const int BH = B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < BH; ++bh) {
        const int b = bh / H, h = bh % H;
        const double gm = gamma[h];
        double *p1 = (double *)malloc(sizeof(double) * (size_t)dk);
        double *p2 = (double *)malloc(sizeof(double) * (size_t)dk);
        for (int t = 0; t < T; ++t) {
            const size_t rkt = (((size_t)b * T + t) * H + h) * (size_t)dk;
            const size_t rvt = (((size_t)b * T + t) * H + h) * (size_t)dv;
            double *ot = o + rvt;
            for (int j = 0; j < dv; ++j) ot[j] = 0.0;
            for (int d = 0; d < dk; ++d) { p1[d] = 1.0; p2[d] = 1.0; }
            for (int s = t; s >= 0; --s) {
                const size_t rks = (((size_t)b * T + s) * H + h) * (size_t)dk;
                const size_t rvs = (((size_t)b * T + s) * H + h) * (size_t)dv;
                double w = 0.0;
                for (int d = 0; d < dk; ++d)
                    w += q[rkt + d] * k[rks + d] * (gm * p1[d] + (1.0 - gm) * p2[d]);
                for (int j = 0; j < dv; ++j) ot[j] += w * v[rvs + j];
                /* extend the products to cover tau = s .. t for the next (earlier) token */
                for (int d = 0; d < dk; ++d) {
                    p1[d] *= exp(g1[rks + d]);
                    p2[d] *= exp(g2[rks + d]);
                }
            }
            for (int j = 0; j < dv; ++j) ot[j] *= scale;
        }
        free(p1);
        free(p2);
    }
}

/*
 * The recurrence with N states, the general outer-product gate and grouped key/value heads.
 *
 * Background section on gated linear attention: the forget gate of a state is a dk x dv matrix formed as the
 * outer product of two vectors, G_t = alpha_t^T beta_t, applied elementwise to the state:
 *     S^n_t[d][j] = alpha^n_t[d] * beta^n_t[j] * S^n_{t-1}[d][j] + k_t[d] * v_t[j],     n = 1 .. N.
 * Section 4.2 ("Why Two States Suffice?") and the ablation over the number of states in Section 5.5 speak of the
 * same layer with 1, 2, 4 or 8 states, each with its own gate.  The paper prints the blend for two states only
 * (gamma, 1 - gamma); for N states the reading taken here is one real coefficient per state,
 *     o_t = scale * q_t * sum_n w_n S^n_t,
 * of which (gamma, 1 - gamma) is the case N = 2.
 * Grouped-query shapes (the Llama-3 teacher of Section 5.5): q and the gates have H heads, k and v have Hkv heads,
 * H a multiple of Hkv; head h reads key/value head h / (H / Hkv).  Every query head keeps its own states.
 *
 * Gates are natural logarithms.  galpha: [N][B][T][H][dk]; gbeta: [N][B][T][H][dv] or NULL (beta = 1);
 * w: [N][H]; S: [N][B][H][dk][dv], initial states on entry, final states on return.
 */
void dsla_oracle_nstate(int N, int B, int T, int H, int Hkv, int dk, int dv,
                        const double *q, const double *k, const double *v,
                        const double *galpha, const double *gbeta,
                        const double *w, double scale, double *S, double *o)
{
    const int BH = B * H;
    const int group = H / Hkv;
    const size_t gstride_a = (size_t)B * T * H * dk, gstride_b = (size_t)B * T * H * dv;
    const size_t sstride = (size_t)B * H * dk * dv;
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < BH; ++bh) {
        const int b = bh / H, h = bh % H, hk = h / group;
        for (int t = 0; t < T; ++t) {
            const size_t rq = (((size_t)b * T + t) * H + h) * (size_t)dk;
            const size_t ro = (((size_t)b * T + t) * H + h) * (size_t)dv;
            const size_t rk = (((size_t)b * T + t) * Hkv + hk) * (size_t)dk;
            const size_t rv = (((size_t)b * T + t) * Hkv + hk) * (size_t)dv;
            for (int n = 0; n < N; ++n) {
                double *s = S + n * sstride + (size_t)bh * dk * dv;
                const double *ga = galpha + n * gstride_a + rq;
                const double *gb = gbeta ? gbeta + n * gstride_b + ro : NULL;
                for (int d = 0; d < dk; ++d) {
                    const double a = exp(ga[d]);
                    for (int j = 0; j < dv; ++j) {
                        const double bj = gb ? exp(gb[j]) : 1.0;
                        s[(size_t)d * dv + j] = a * bj * s[(size_t)d * dv + j] + k[rk + d] * v[rv + j];
                    }
                }
            }
            for (int j = 0; j < dv; ++j) {
                double acc = 0.0;
                for (int d = 0; d < dk; ++d) {
                    double mix = 0.0;
                    for (int n = 0; n < N; ++n)
                        mix += w[(size_t)n * H + h] * S[n * sstride + (size_t)bh * dk * dv + (size_t)d * dv + j];
                    acc += q[rq + d] * mix;
                }
                o[ro + j] = scale * acc;
            }
        }
    }
}
