/*
 * CPU oracle for the SliceMoE layer forward pass.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, fp64.  It follows the layer's definition (paper Section 3, Section 3.1,
 * Eq. 1) slice by slice with no grouping, tiling or fusion; the grouped execution the
 * paper describes in Section 3.4 only reorders independent per-slice work, so it reaches
 * exactly this result.  Only tests, the smoke check and the benchmark's CPU-baseline leg
 * may call this file; the product path never does, and the two share no code.
 *
 * Conventions (the paper is silent on some of these; they are the stated readings):
 *   - slice n = t*S + s is the contiguous segment h[t, s*ds : (s+1)*ds]  (Section 3), so the
 *     slice view of a row-major h[T, d] is simply x[Ns, ds] with Ns = T*S.
 *   - Linear layers are y = x W + b with W stored [in, out] row-major; both router layers
 *     and both expert layers have biases.
 *   - router: g = ReLU(x Wr1 + br1) Wr2 + br2;  p = softmax(g) over all E experts
 *     (temperature 1, Appendix B default), NOT renormalised over the selected k.
 *   - top-k: selected on the logits (softmax is monotone) after rounding them to fp32,
 *     the precision in which the GPU path takes the same decision; equal values go to the
 *     lower expert index; slot 0 holds the largest.
 *   - Eq. 1 weights the expert INPUT: expert e_j sees p_j * x; its bias is not scaled.
 *   - expert: phi_e(v) = act(v W1[e] + b1[e]) W2[e] + b2[e], act = exact (erf) GELU.
 *   - the k expert outputs of one slice are summed; the S slices are concatenated, which in
 *     the slice view means out[n, :] sits at the same place as x[n, :].
 *   - capacity (not in the paper; benchmark contract): within an expert, rows are ranked by
 *     ascending slice id n; an assignment with rank >= C is dropped and contributes zero.
 *   - flat assignment id a = n*k + j;  perm[row] = a;  inv[a] = row, or -1 if dropped.
 *
 * Pins (tests/test_oracle_*.py): brute-force stable sort for top-k and dispatch, count sum,
 * bijection, E=1/k=1 dense-FFN reduction against library matmul+erf, S=1 token-level MoE,
 * W2=0 and identity-activation closed forms, load-statistic closed forms; for the training-time
 * router: reduction to oracle_route, the power law of the temperature, shift invariance and
 * planted bumps for the noise, hand-worked dropout cases; for the backward: central finite
 * differences of the forward functions in this file, parameter by parameter.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_ACT_GELU 0
#define ORACLE_ACT_IDENTITY 1 /* used only by closed-form pins */

static double act_fn(double z, int act)
{
    if (act == ORACLE_ACT_IDENTITY) return z;
    /* z * Phi(z), Phi(z) = (1 + erf(z/sqrt 2))/2 = erfc(-z/sqrt 2)/2 (the erfc form keeps
     * full relative accuracy in the negative tail) */
    return 0.5 * z * erfc(-z * 0.70710678118654752440);
}

/* Exposed so a test can pin it against closed forms and a library normal CDF. */
double oracle_gelu(double z) { return act_fn(z, ORACLE_ACT_GELU); }

/* Router logits of one slice (Section 3.1): g = ReLU(x Wr1 + br1) Wr2 + br2. */
static void router_logits(const double *x, int ds, int Hr, int E,
                          const double *Wr1, const double *br1,
                          const double *Wr2, const double *br2,
                          double *u /*[Hr] scratch*/, double *g /*[E]*/)
{
    for (int j = 0; j < Hr; ++j) u[j] = br1[j];
    for (int i = 0; i < ds; ++i)
        for (int j = 0; j < Hr; ++j) u[j] += x[i] * Wr1[(size_t)i * Hr + j];
    for (int j = 0; j < Hr; ++j) u[j] = u[j] > 0.0 ? u[j] : 0.0;
    for (int e = 0; e < E; ++e) g[e] = br2[e];
    for (int j = 0; j < Hr; ++j)
        for (int e = 0; e < E; ++e) g[e] += u[j] * Wr2[(size_t)j * E + e];
}

/*
 * Routing of every slice (Section 3.1).
 *   x[Ns, ds]  ->  idx[Ns, k] (int32), pk[Ns, k] (softmax probability of each selected
 *   expert), optional logits[Ns, E] and margin[Ns] (= fp32 logit of the k-th selected
 *   minus the largest unselected one; +inf when k == E).
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int oracle_route(const double *x, int64_t Ns, int ds, int Hr, int E, int k,
                 const double *Wr1, const double *br1, const double *Wr2, const double *br2,
                 int32_t *idx, double *pk, double *logits, double *margin)
{
    if (!x || !idx || !pk || Ns < 0 || ds < 1 || Hr < 1 || E < 1 || k < 1 || k > E) return -1;
    int fail = 0;
#pragma omp parallel
    {
        double *u = (double *)malloc(sizeof(double) * (size_t)Hr);
        double *g = (double *)malloc(sizeof(double) * (size_t)E);
        double *p = (double *)malloc(sizeof(double) * (size_t)E);
        float *gf = (float *)malloc(sizeof(float) * (size_t)E);
        char *taken = (char *)malloc((size_t)E);
        if (!u || !g || !p || !gf || !taken) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(static)
            for (int64_t n = 0; n < Ns; ++n) {
                router_logits(x + n * ds, ds, Hr, E, Wr1, br1, Wr2, br2, u, g);
                if (logits) memcpy(logits + n * E, g, sizeof(double) * (size_t)E);
                /* softmax over all E experts */
                double m = g[0];
                for (int e = 1; e < E; ++e) m = g[e] > m ? g[e] : m;
                double den = 0.0;
                for (int e = 0; e < E; ++e) { p[e] = exp(g[e] - m); den += p[e]; }
                for (int e = 0; e < E; ++e) p[e] /= den;
                /* top-k: k rounds of "largest remaining fp32 logit, lowest index on ties" */
                for (int e = 0; e < E; ++e) { gf[e] = (float)g[e]; taken[e] = 0; }
                for (int j = 0; j < k; ++j) {
                    int best = -1;
                    for (int e = 0; e < E; ++e)
                        if (!taken[e] && (best < 0 || gf[e] > gf[best])) best = e;
                    taken[best] = 1;
                    idx[n * k + j] = best;
                    pk[n * k + j] = p[best];
                }
                if (margin) {
                    int rest = -1;
                    for (int e = 0; e < E; ++e)
                        if (!taken[e] && (rest < 0 || gf[e] > gf[rest])) rest = e;
                    margin[n] = rest < 0 ? INFINITY
                                         : (double)gf[idx[n * k + k - 1]] - (double)gf[rest];
                }
            }
        }
        free(u); free(g); free(p); free(gf); free(taken);
    }
    return fail ? -1 : 0;
}

/*
 * Training-time routing of every slice: the router of Section 3.1 with the three variations
 * the paper describes around it, in the order logits -> noise -> top-k and softmax -> dropout.
 *   - Gaussian logit noise (Section 5, robustness to router noise): g <- g + sigma * noise[n, e],
 *     added before the softmax, hence also before the selection.  The standard-normal draws
 *     are an INPUT (noise[Ns, E], may be NULL when sigma == 0).
 *   - softmax temperature (Appendix B): p = softmax(g / tau) over all E experts.  The selection
 *     is taken on g itself (dividing by tau > 0 does not change the order), rounded to fp32 as
 *     in oracle_route.
 *   - cross-slice dropout (Section 3.3; Appendix A gives the rate 0.2): each of the k selected
 *     assignments of a slice is dropped independently when its uniform draw drop_u[n, j] is
 *     below `rate` (draws are an INPUT, compared as fp32 values); the remaining probabilities of
 *     the slice are renormalised to sum to 1 and the dropped ones are 0.  A slice whose k draws
 *     would all drop keeps slot 0, its largest, so every slice still reaches an expert.  With
 *     rate > 0 the renormalisation applies to every slice, dropped from or not.  idx keeps all
 *     k experts: a dropped assignment stays assigned with probability 0 (by Eq. 1 its expert
 *     then sees the zero vector).
 * With tau = 1, sigma = 0 and rate = 0 this is oracle_route.  Outputs as oracle_route; `logits`
 * receives the noisy logits, `margin` is taken on them.
 */
int oracle_route_train(const double *x, int64_t Ns, int ds, int Hr, int E, int k,
                       const double *Wr1, const double *br1, const double *Wr2, const double *br2,
                       double tau, double sigma, const double *noise, double rate, const double *drop_u,
                       int32_t *idx, double *pk, double *logits, double *margin)
{
    if (!x || !idx || !pk || Ns < 0 || ds < 1 || Hr < 1 || E < 1 || k < 1 || k > E) return -1;
    if (!(tau > 0.0) || !(sigma >= 0.0) || !(rate >= 0.0) || !(rate < 1.0)) return -1;
    if ((sigma > 0.0 && !noise) || (rate > 0.0 && !drop_u)) return -1;
    int fail = 0;
#pragma omp parallel
    {
        double *u = (double *)malloc(sizeof(double) * (size_t)Hr);
        double *g = (double *)malloc(sizeof(double) * (size_t)E);
        double *p = (double *)malloc(sizeof(double) * (size_t)E);
        float *gf = (float *)malloc(sizeof(float) * (size_t)E);
        char *taken = (char *)malloc((size_t)E);
        char *keep = (char *)malloc((size_t)k);
        if (!u || !g || !p || !gf || !taken || !keep) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(static)
            for (int64_t n = 0; n < Ns; ++n) {
                router_logits(x + n * ds, ds, Hr, E, Wr1, br1, Wr2, br2, u, g);
                if (sigma > 0.0)
                    for (int e = 0; e < E; ++e) g[e] += sigma * noise[n * E + e];
                if (logits) memcpy(logits + n * E, g, sizeof(double) * (size_t)E);
                /* softmax of g / tau over all E experts */
                double m = g[0];
                for (int e = 1; e < E; ++e) m = g[e] > m ? g[e] : m;
                double den = 0.0;
                for (int e = 0; e < E; ++e) { p[e] = exp((g[e] - m) / tau); den += p[e]; }
                for (int e = 0; e < E; ++e) p[e] /= den;
                /* top-k on the fp32-rounded (noisy) logits, lowest index on ties */
                for (int e = 0; e < E; ++e) { gf[e] = (float)g[e]; taken[e] = 0; }
                for (int j = 0; j < k; ++j) {
                    int best = -1;
                    for (int e = 0; e < E; ++e)
                        if (!taken[e] && (best < 0 || gf[e] > gf[best])) best = e;
                    taken[best] = 1;
                    idx[n * k + j] = best;
                    pk[n * k + j] = p[best];
                }
                if (margin) {
                    int rest = -1;
                    for (int e = 0; e < E; ++e)
                        if (!taken[e] && (rest < 0 || gf[e] > gf[rest])) rest = e;
                    margin[n] = rest < 0 ? INFINITY
                                         : (double)gf[idx[n * k + k - 1]] - (double)gf[rest];
                }
                if (rate > 0.0) {
                    int kept = 0;
                    for (int j = 0; j < k; ++j) {
                        keep[j] = !((float)drop_u[n * k + j] < (float)rate);
                        kept += keep[j];
                    }
                    if (kept == 0) keep[0] = 1;
                    double sum = 0.0;
                    for (int j = 0; j < k; ++j) if (keep[j]) sum += pk[n * k + j];
                    for (int j = 0; j < k; ++j) pk[n * k + j] = keep[j] ? pk[n * k + j] / sum : 0.0;
                }
            }
        }
        free(u); free(g); free(p); free(gf); free(taken); free(keep);
    }
    return fail ? -1 : 0;
}

/*
 * Dispatch: group assignments per expert in stable slice order, with optional capacity.
 *   idx[Ns, k] -> counts_raw[E], counts[E] (= min(counts_raw, C)), offsets[E+1]
 *   (exclusive scan of counts; offsets[E] = kept rows), perm[Ns*k] (first offsets[E]
 *   entries valid, the rest set to -1), inv[Ns*k].
 * capacity < 0 means dropless.  One serial pass in ascending n with per-expert counters.
 */
int oracle_dispatch(const int32_t *idx, int64_t Ns, int k, int E, int64_t capacity,
                    int32_t *counts_raw, int32_t *counts, int32_t *offsets,
                    int32_t *perm, int32_t *inv)
{
    if (!idx || !counts_raw || !counts || !offsets || !perm || !inv || E < 1 || k < 1) return -1;
    int64_t Na = Ns * k;
    for (int e = 0; e < E; ++e) counts_raw[e] = 0;
    for (int64_t a = 0; a < Na; ++a) {
        if (idx[a] < 0 || idx[a] >= E) return -1;
        counts_raw[idx[a]]++;
    }
    offsets[0] = 0;
    for (int e = 0; e < E; ++e) {
        counts[e] = (capacity >= 0 && counts_raw[e] > capacity) ? (int32_t)capacity : counts_raw[e];
        offsets[e + 1] = offsets[e] + counts[e];
    }
    int64_t *seen = (int64_t *)calloc((size_t)E, sizeof(int64_t));
    if (!seen) return -1;
    for (int64_t a = 0; a < Na; ++a) perm[a] = -1;
    for (int64_t n = 0; n < Ns; ++n)
        for (int j = 0; j < k; ++j) {
            int64_t a = n * k + j;
            int e = idx[a];
            int64_t rank = seen[e]++;
            if (capacity < 0 || rank < capacity) {
                int64_t row = offsets[e] + rank;
                perm[row] = (int32_t)a;
                inv[a] = (int32_t)row;
            } else {
                inv[a] = -1;
            }
        }
    free(seen);
    return 0;
}

/* One expert on one weighted slice (Eq. 1 and the expert FFN of Section 3.1):
 * y = act((p x) W1 + b1) W2 + b2. */
static void expert_apply(const double *x, double p, int ds, int He,
                         const double *W1, const double *b1, const double *W2, const double *b2,
                         int act, double *z /*[He] scratch*/, double *y /*[ds]*/)
{
    for (int j = 0; j < He; ++j) z[j] = b1[j];
    for (int i = 0; i < ds; ++i) {
        double xi = p * x[i];
        for (int j = 0; j < He; ++j) z[j] += xi * W1[(size_t)i * He + j];
    }
    for (int j = 0; j < He; ++j) z[j] = act_fn(z[j], act);
    for (int i = 0; i < ds; ++i) y[i] = b2[i];
    for (int j = 0; j < He; ++j)
        for (int i = 0; i < ds; ++i) y[i] += z[j] * W2[(size_t)j * ds + i];
}

/*
 * Expert stage on the stacked batch (Section 3.4 states the grouping; the values are those
 * of Section 3.1): for each kept row r, a = perm[r], n = a / k, e = idx[a],
 *   y[r, :] = phi_e(pk[a] * x[n, :]).
 */
int oracle_expert_rows(const double *x, int ds, int He, int k,
                       const int32_t *idx, const double *pk, const int32_t *perm, int64_t n_rows,
                       const double *W1, const double *b1, const double *W2, const double *b2,
                       int act, double *y)
{
    if (!x || !idx || !pk || !perm || !y || n_rows < 0) return -1;
    int fail = 0;
#pragma omp parallel
    {
        double *z = (double *)malloc(sizeof(double) * (size_t)He);
        if (!z) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(static)
            for (int64_t r = 0; r < n_rows; ++r) {
                int64_t a = perm[r];
                int64_t n = a / k;
                int e = idx[a];
                expert_apply(x + n * ds, pk[a], ds, He,
                             W1 + (size_t)e * ds * He, b1 + (size_t)e * He,
                             W2 + (size_t)e * He * ds, b2 + (size_t)e * ds, act, z, y + r * ds);
            }
        }
        free(z);
    }
    return fail ? -1 : 0;
}

/*
 * Combine (Section 3.1): out[n, :] = sum over the kept assignments j of slice n of
 * y[inv[n*k + j], :]; a slice whose k assignments were all dropped yields zeros.
 */
int oracle_combine(const double *y, const int32_t *inv, int64_t Ns, int k, int ds, double *out)
{
    if (!y || !inv || !out) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < Ns; ++n) {
        double *o = out + n * ds;
        for (int i = 0; i < ds; ++i) o[i] = 0.0;
        for (int j = 0; j < k; ++j) {
            int64_t r = inv[n * k + j];
            if (r < 0) continue;
            for (int i = 0; i < ds; ++i) o[i] += y[r * ds + i];
        }
    }
    return 0;
}

/*
 * Expert + combine by the plain per-slice definition, given routing and the keep mask:
 *   out[n, :] = sum_{j : inv[n*k+j] >= 0} phi_{idx[n,j]}(pk[n,j] * x[n, :]).
 * `inv` may be NULL (nothing dropped).  Slices are independent, so this also serves
 * sampled subsets: pass only the sampled rows of x / idx / pk / inv.
 */
int oracle_slices(const double *x, int64_t Ns, int ds, int He, int k,
                  const int32_t *idx, const double *pk, const int32_t *inv,
                  const double *W1, const double *b1, const double *W2, const double *b2,
                  int act, double *out)
{
    if (!x || !idx || !pk || !out) return -1;
    int fail = 0;
#pragma omp parallel
    {
        double *z = (double *)malloc(sizeof(double) * (size_t)He);
        double *y = (double *)malloc(sizeof(double) * (size_t)ds);
        if (!z || !y) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(static)
            for (int64_t n = 0; n < Ns; ++n) {
                double *o = out + n * ds;
                for (int i = 0; i < ds; ++i) o[i] = 0.0;
                for (int j = 0; j < k; ++j) {
                    int64_t a = n * k + j;
                    if (inv && inv[a] < 0) continue;
                    int e = idx[a];
                    expert_apply(x + n * ds, pk[a], ds, He,
                                 W1 + (size_t)e * ds * He, b1 + (size_t)e * He,
                                 W2 + (size_t)e * He * ds, b2 + (size_t)e * ds, act, z, y);
                    for (int i = 0; i < ds; ++i) o[i] += y[i];
                }
            }
        }
        free(z); free(y);
    }
    return fail ? -1 : 0;
}

/*
 * Whole layer: h[T, d] -> h'[T, d]  (route, dispatch, experts, combine).
 * Optional outputs (may be NULL): idx[Ns,k], pk[Ns,k], margin[Ns], counts_raw[E],
 * counts[E], offsets[E+1], perm[Ns*k], inv[Ns*k].
 */
int oracle_forward(const double *h, int64_t T, int d, int S, int Hr, int E, int k, int He,
                   int64_t capacity,
                   const double *Wr1, const double *br1, const double *Wr2, const double *br2,
                   const double *W1, const double *b1, const double *W2, const double *b2,
                   int act, double *h_out,
                   int32_t *idx_o, double *pk_o, double *margin_o, int32_t *counts_raw_o,
                   int32_t *counts_o, int32_t *offsets_o, int32_t *perm_o, int32_t *inv_o)
{
    if (!h || !h_out || T < 0 || S < 1 || d < 1 || d % S) return -1;
    int ds = d / S;
    int64_t Ns = T * S, Na = Ns * k;
    int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)(Na + 1));
    double *pk = (double *)malloc(sizeof(double) * (size_t)(Na + 1));
    int32_t *perm = (int32_t *)malloc(sizeof(int32_t) * (size_t)(Na + 1));
    int32_t *inv = (int32_t *)malloc(sizeof(int32_t) * (size_t)(Na + 1));
    int32_t *cr = (int32_t *)malloc(sizeof(int32_t) * (size_t)E);
    int32_t *cc = (int32_t *)malloc(sizeof(int32_t) * (size_t)E);
    int32_t *off = (int32_t *)malloc(sizeof(int32_t) * (size_t)(E + 1));
    int rc = -1;
    if (idx && pk && perm && inv && cr && cc && off) {
        rc = oracle_route(h, Ns, ds, Hr, E, k, Wr1, br1, Wr2, br2, idx, pk, NULL, margin_o);
        if (!rc) rc = oracle_dispatch(idx, Ns, k, E, capacity, cr, cc, off, perm, inv);
        if (!rc) rc = oracle_slices(h, Ns, ds, He, k, idx, pk, inv, W1, b1, W2, b2, act, h_out);
        if (!rc) {
            if (idx_o) memcpy(idx_o, idx, sizeof(int32_t) * (size_t)Na);
            if (pk_o) memcpy(pk_o, pk, sizeof(double) * (size_t)Na);
            if (perm_o) memcpy(perm_o, perm, sizeof(int32_t) * (size_t)Na);
            if (inv_o) memcpy(inv_o, inv, sizeof(int32_t) * (size_t)Na);
            if (counts_raw_o) memcpy(counts_raw_o, cr, sizeof(int32_t) * (size_t)E);
            if (counts_o) memcpy(counts_o, cc, sizeof(int32_t) * (size_t)E);
            if (offsets_o) memcpy(offsets_o, off, sizeof(int32_t) * (size_t)(E + 1));
        }
    }
    free(idx); free(pk); free(perm); free(inv); free(cr); free(cc); free(off);
    return rc;
}

/*
 * Backward of the layer: gradients of a scalar loss that depends on h and on the weights only
 * through h', given G = dL/dh' (slice view [Ns, ds]).  Chain rule through the definition, slice
 * by slice: the k-sum, the expert FFN (Section 3.1), the input weighting of Eq. 1, and the router
 * (Section 3.1; training-time variations as in oracle_route_train).
 *
 * Readings (the paper gives no backward):
 *   - the routing DECISIONS are piecewise constant and held fixed: which experts a slice selects,
 *     which assignments a capacity limit dropped (inv[a] < 0: no contribution, no gradient) and
 *     which the cross-slice dropout zeroed.  The router receives gradient only through the
 *     selected probabilities, which weight the expert inputs (Eq. 1: z = p (x W1) + b1, so
 *     dL/dp = sum_hidden dL/dz * (x W1)).
 *   - with dropout the renormalisation pk'_j = p_j / s (s = sum of the kept p) is differentiated:
 *     dL/dp_j = (dL/dpk'_j - sum_i dL/dpk'_i pk'_i) / s for kept j, 0 for dropped j.
 *   - softmax with temperature: dL/dg_e = (1/tau) sum_j dL/dp_j p_j ([e == e_j] - p_e); the noise
 *     is an additive constant.
 *   - the capacity loss of Eq. 2 is a function of integer counts and has zero gradient as
 *     written.  Section 3.1 says the router is trained with it and Section 3.2 speaks of its
 *     gradients, so its authors differentiate something the paper does not state.  The reading
 *     offered here (off unless the caller passes capg) is the usual one for a count-based
 *     balance loss: the count of expert e is replaced by the sum of the final probabilities of
 *     the assignments routed to it, c_e = sum_{a: e(a) = e} p_a, and the loss by
 *     alpha * CV^2(c_1..c_E) (population variance).  Then dL_cap/dp_a = capg[e(a)], with
 *     capg[e] = alpha * (2E / S^2) (c_e - Q / S), S = sum c, Q = sum c^2, which the caller
 *     computes from the forward pass's probabilities.  Every assignment carries it, also one
 *     that a capacity limit dropped (it still counts as assigned); one that the dropout zeroed
 *     has a constant probability of zero and passes nothing on.
 * idx[Ns,k] and inv[Ns*k] are the forward pass's (oracle_route_train / oracle_dispatch); the
 * probabilities are recomputed here.  Outputs (all overwritten): dx[Ns, ds] and one array per
 * weight tensor in its logical layout.  Returns 0, or -1 on bad arguments / allocation failure.
 */
static double gelu_grad(double z)
{
    /* d/dz [z Phi(z)] = Phi(z) + z phi(z) */
    return 0.5 * erfc(-z * 0.70710678118654752440) + z * exp(-0.5 * z * z) * 0.39894228040143267794;
}

int oracle_backward(const double *x, int64_t Ns, int ds, int Hr, int E, int k, int He,
                    const double *Wr1, const double *br1, const double *Wr2, const double *br2,
                    const double *W1, const double *b1, const double *W2, const double *b2,
                    double tau, double sigma, const double *noise, double rate, const double *drop_u,
                    const int32_t *idx, const int32_t *inv, const double *G, const double *capg,
                    double *dx, double *dWr1, double *dbr1, double *dWr2, double *dbr2,
                    double *dW1, double *db1, double *dW2, double *db2)
{
    if (!x || !idx || !inv || !G || !dx || !dWr1 || !dbr1 || !dWr2 || !dbr2 || !dW1 || !db1 || !dW2 || !db2) return -1;
    if (Ns < 0 || ds < 1 || Hr < 1 || E < 1 || k < 1 || k > E || He < 1) return -1;
    if (!(tau > 0.0) || !(sigma >= 0.0) || !(rate >= 0.0) || !(rate < 1.0)) return -1;
    if ((sigma > 0.0 && !noise) || (rate > 0.0 && !drop_u)) return -1;
    (void)b2; /* the output bias shifts h' and does not enter any derivative */
    const size_t nWr1 = (size_t)ds * Hr, nWr2 = (size_t)Hr * E, nW = (size_t)E * ds * He;
    const size_t nb1 = (size_t)E * He, nb2 = (size_t)E * ds;
    memset(dWr1, 0, sizeof(double) * nWr1); memset(dbr1, 0, sizeof(double) * (size_t)Hr);
    memset(dWr2, 0, sizeof(double) * nWr2); memset(dbr2, 0, sizeof(double) * (size_t)E);
    memset(dW1, 0, sizeof(double) * nW); memset(db1, 0, sizeof(double) * nb1);
    memset(dW2, 0, sizeof(double) * nW); memset(db2, 0, sizeof(double) * nb2);
    int fail = 0;
#pragma omp parallel
    {
        /* per-thread partial weight gradients, added up at the end */
        const size_t total = nWr1 + (size_t)Hr + nWr2 + (size_t)E + 2 * nW + nb1 + nb2;
        double *part = (double *)calloc(total, sizeof(double));
        double *ur = (double *)malloc(sizeof(double) * (size_t)Hr);
        double *dur = (double *)malloc(sizeof(double) * (size_t)Hr);
        double *g = (double *)malloc(sizeof(double) * (size_t)E);
        double *pa = (double *)malloc(sizeof(double) * (size_t)E);
        double *dg = (double *)malloc(sizeof(double) * (size_t)E);
        double *u = (double *)malloc(sizeof(double) * (size_t)He);
        double *dz = (double *)malloc(sizeof(double) * (size_t)He);
        double *pf = (double *)malloc(sizeof(double) * (size_t)k);   /* final probabilities */
        double *dpf = (double *)malloc(sizeof(double) * (size_t)k);  /* dL/d(final probability) */
        char *keep = (char *)malloc((size_t)k);
        if (!part || !ur || !dur || !g || !pa || !dg || !u || !dz || !pf || !dpf || !keep) {
#pragma omp atomic write
            fail = 1;
        } else {
            double *qWr1 = part, *qbr1 = qWr1 + nWr1, *qWr2 = qbr1 + Hr, *qbr2 = qWr2 + nWr2;
            double *qW1 = qbr2 + E, *qb1 = qW1 + nW, *qW2 = qb1 + nb1, *qb2 = qW2 + nW;
#pragma omp for schedule(static)
            for (int64_t n = 0; n < Ns; ++n) {
                const double *xn = x + n * ds, *Gn = G + n * ds;
                double *dxn = dx + n * ds;
                for (int i = 0; i < ds; ++i) dxn[i] = 0.0;
                /* forward quantities of the router, as in oracle_route_train */
                router_logits(xn, ds, Hr, E, Wr1, br1, Wr2, br2, ur, g);
                if (sigma > 0.0)
                    for (int e = 0; e < E; ++e) g[e] += sigma * noise[n * E + e];
                double m = g[0];
                for (int e = 1; e < E; ++e) m = g[e] > m ? g[e] : m;
                double den = 0.0;
                for (int e = 0; e < E; ++e) { pa[e] = exp((g[e] - m) / tau); den += pa[e]; }
                for (int e = 0; e < E; ++e) pa[e] /= den;
                double ssum = 1.0;
                for (int j = 0; j < k; ++j) { keep[j] = 1; pf[j] = pa[idx[n * k + j]]; }
                if (rate > 0.0) {
                    int kept = 0;
                    for (int j = 0; j < k; ++j) { keep[j] = !((float)drop_u[n * k + j] < (float)rate); kept += keep[j]; }
                    if (kept == 0) keep[0] = 1;
                    ssum = 0.0;
                    for (int j = 0; j < k; ++j) if (keep[j]) ssum += pf[j];
                    for (int j = 0; j < k; ++j) pf[j] = keep[j] ? pf[j] / ssum : 0.0;
                }
                /* experts */
                for (int j = 0; j < k; ++j) {
                    int64_t a = n * k + j;
                    int e = idx[a];
                    dpf[j] = capg ? capg[e] : 0.0;
                    if (inv[a] < 0) continue;
                    const double *w1 = W1 + (size_t)e * ds * He, *w2 = W2 + (size_t)e * He * ds;
                    double p = pf[j];
                    for (int h = 0; h < He; ++h) u[h] = 0.0;
                    for (int i = 0; i < ds; ++i)
                        for (int h = 0; h < He; ++h) u[h] += xn[i] * w1[(size_t)i * He + h];
                    for (int i = 0; i < ds; ++i) qb2[(size_t)e * ds + i] += Gn[i];
                    for (int h = 0; h < He; ++h) {
                        double z = p * u[h] + b1[(size_t)e * He + h];
                        double a1 = act_fn(z, ORACLE_ACT_GELU);
                        double da1 = 0.0;
                        for (int i = 0; i < ds; ++i) {
                            qW2[((size_t)e * He + h) * ds + i] += a1 * Gn[i];
                            da1 += Gn[i] * w2[(size_t)h * ds + i];
                        }
                        dz[h] = da1 * gelu_grad(z);
                        qb1[(size_t)e * He + h] += dz[h];
                        dpf[j] += dz[h] * u[h];
                    }
                    for (int i = 0; i < ds; ++i) {
                        double acc = 0.0;
                        for (int h = 0; h < He; ++h) {
                            qW1[((size_t)e * ds + i) * He + h] += xn[i] * p * dz[h];
                            acc += dz[h] * w1[(size_t)i * He + h];
                        }
                        dxn[i] += p * acc;
                    }
                }
                /* through the renormalisation of the dropout, then the softmax */
                if (rate > 0.0) {
                    double dot = 0.0;
                    for (int j = 0; j < k; ++j) if (keep[j]) dot += dpf[j] * pf[j];
                    for (int j = 0; j < k; ++j) dpf[j] = keep[j] ? (dpf[j] - dot) / ssum : 0.0;
                }
                for (int e = 0; e < E; ++e) dg[e] = 0.0;
                for (int j = 0; j < k; ++j) {
                    int ej = idx[n * k + j];
                    double c = dpf[j] * pa[ej];
                    for (int e = 0; e < E; ++e) dg[e] += c * ((e == ej ? 1.0 : 0.0) - pa[e]);
                }
                for (int e = 0; e < E; ++e) dg[e] /= tau;
                /* router MLP */
                for (int e = 0; e < E; ++e) qbr2[e] += dg[e];
                for (int h = 0; h < Hr; ++h) {
                    double acc = 0.0;
                    for (int e = 0; e < E; ++e) {
                        qWr2[(size_t)h * E + e] += ur[h] * dg[e];
                        acc += dg[e] * Wr2[(size_t)h * E + e];
                    }
                    dur[h] = ur[h] > 0.0 ? acc : 0.0;
                    qbr1[h] += dur[h];
                }
                for (int i = 0; i < ds; ++i) {
                    double acc = 0.0;
                    for (int h = 0; h < Hr; ++h) {
                        qWr1[(size_t)i * Hr + h] += xn[i] * dur[h];
                        acc += dur[h] * Wr1[(size_t)i * Hr + h];
                    }
                    dxn[i] += acc;
                }
            }
#pragma omp critical
            {
                for (size_t t = 0; t < nWr1; ++t) dWr1[t] += qWr1[t];
                for (int t = 0; t < Hr; ++t) dbr1[t] += qbr1[t];
                for (size_t t = 0; t < nWr2; ++t) dWr2[t] += qWr2[t];
                for (int t = 0; t < E; ++t) dbr2[t] += qbr2[t];
                for (size_t t = 0; t < nW; ++t) { dW1[t] += qW1[t]; dW2[t] += qW2[t]; }
                for (size_t t = 0; t < nb1; ++t) db1[t] += qb1[t];
                for (size_t t = 0; t < nb2; ++t) db2[t] += qb2[t];
            }
        }
        free(part); free(ur); free(dur); free(g); free(pa); free(dg); free(u); free(dz); free(pf); free(dpf); free(keep);
    }
    return fail ? -1 : 0;
}

/*
 * Load statistics of per-expert counts.
 *   cv_pop / cv_sample : std/mean with the population (1/E) and sample (1/(E-1)) variance;
 *                        the capacity loss of Eq. 2 is alpha * cv^2 (population reading).
 *   ele                : -sum_e load_e log load_e / log E with load_e = counts_e / sum
 *                        (Section 4, Metrics); 0 log 0 = 0; defined as 1 when E == 1.
 */
int oracle_load_stats(const int32_t *counts, int E, double *cv_pop, double *cv_sample, double *ele)
{
    if (!counts || E < 1) return -1;
    double sum = 0.0;
    for (int e = 0; e < E; ++e) sum += counts[e];
    double mean = sum / E, ss = 0.0, ent = 0.0;
    for (int e = 0; e < E; ++e) {
        double dlt = counts[e] - mean;
        ss += dlt * dlt;
        if (counts[e] > 0 && sum > 0) { double l = counts[e] / sum; ent -= l * log(l); }
    }
    if (cv_pop) *cv_pop = mean > 0 ? sqrt(ss / E) / mean : 0.0;
    if (cv_sample) *cv_sample = (mean > 0 && E > 1) ? sqrt(ss / (E - 1)) / mean : 0.0;
    if (ele) *ele = E > 1 ? ent / log((double)E) : 1.0;
    return 0;
}

/* Number of OpenMP threads a parallel region of this library uses. */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif
