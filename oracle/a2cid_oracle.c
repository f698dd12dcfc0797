/*
 * A2CiD2 reference oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, serial, event-by-event fp64 implementation of the continuous-momentum
 * gossip dynamic of the A2CiD2 paper (arXiv 2306.08289).  It exists only so that
 * tests, the smoke check and the benchmark's CPU-baseline leg have something
 * independent to compare the GPU library against.  It shares no source, header,
 * table or helper with the GPU library and is never called by it.
 *
 * Reading of the paper used here (all deliberate, see the citations per function):
 *   - the state of worker i is (x_i, xt_i, t_i): parameters, momentum copy and the
 *     time at which they were last brought up to date (Algorithm 1, initialisation);
 *   - an event at time t first applies the mixing flow exp((t - t_i) A),
 *     A = [[-eta, eta], [eta, -eta]], to every worker the event touches, THEN
 *     evaluates the jump from the mixed values (Eq. (1): the jump terms are taken
 *     at x_t, which already contains the continuous flow up to t);
 *   - a gossip jump on edge (i, j) uses ONE difference m = x_i - x_j for both
 *     endpoints and for both buffers; the momentum buffer moves by alpha_tilde * m
 *     built from the x difference, not from the xt difference (Eq. (1), second line).
 *
 * Every pin that ties these functions to something other than themselves lives in
 * tests/ (marked "not gpu"): scipy's matrix exponential, dense operator products,
 * conservation laws, the paper's printed chi values.
 *
 * Build: gcc -O2 -ffp-contract=off -shared -fPIC (see oracle/build.py).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Mixing step of Algorithm 1: (x, xt) <- exp(tau * A) (x, xt), element-wise.  */
/* A = eta * [[-1, 1], [1, -1]] has eigenvalue 0 on (1, 1) and -2 eta on       */
/* (1, -1), hence exp(tau A) = 1/2 [[1 + e, 1 - e], [1 - e, 1 + e]] with       */
/* e = exp(-2 eta tau).                                                        */
/* ------------------------------------------------------------------------- */
void a2o_mix_row(double *x, double *xt, int64_t d, double eta, double tau)
{
    const double e = exp(-2.0 * eta * tau);
    const double a = 0.5 * (1.0 + e);
    const double b = 0.5 * (1.0 - e);
    for (int64_t k = 0; k < d; ++k) {
        const double xo = x[k], xto = xt[k];
        x[k] = a * xo + b * xto;
        xt[k] = b * xo + a * xto;
    }
}

/* ------------------------------------------------------------------------- */
/* Worker clocks (section "Practical implementation of the dynamic": time is     */
/* normalised by a running average of the durations of the previous gradient    */
/* steps, read per worker): rate_i is the speed of worker i's own clock against */
/* the clock of the event times, so the mixing of worker i from its last event  */
/* to te lasts rate_i * (te - t_i).  rate_i = 1 is the plain dynamic.           */
/* ------------------------------------------------------------------------- */
/* Gradient jump of Eq. (1) / gradient thread of Algorithm 1 for worker i at    */
/* time te: mix to te, g = gscale * h .* (x_i - c) + xi, then the SAME          */
/* gamma * g is subtracted from x_i and from xt_i.  This g is the gradient of   */
/* the local objective f_i(x) = gscale/2 sum_k h_k (x_k - c_k)^2 plus the noise */
/* xi of a stochastic oracle: mu-strongly convex and L-smooth with              */
/* mu = gscale min h, L = gscale max h (the first setting of Proposition 3.2).  */
/* c, xi and h may be NULL (c, xi: zeros; h: ones, i.e. a scalar curvature).    */
/* ------------------------------------------------------------------------- */
static double a2o_local_gradient(double x, int64_t k, double gscale,
                                 const double *c, const double *xi, const double *h)
{
    double g = gscale * (h ? h[k] : 1.0) * (x - (c ? c[k] : 0.0));
    if (xi) g += xi[k];
    return g;
}

void a2o_gradient_event(double *x_i, double *xt_i, double *t_i, double rate_i, int64_t d,
                        double eta, double te, double gamma, double gscale,
                        const double *c, const double *xi, const double *h)
{
    a2o_mix_row(x_i, xt_i, d, eta, rate_i * (te - *t_i));
    *t_i = te;
    for (int64_t k = 0; k < d; ++k) {
        const double g = a2o_local_gradient(x_i[k], k, gscale, c, xi, h);
        x_i[k] -= gamma * g;
        xt_i[k] -= gamma * g;
    }
}

/* ------------------------------------------------------------------------- */
/* Gossip jump of Eq. (1) / communication thread of Algorithm 1 on edge (i, j)  */
/* at time te: both workers mix to te, m = x_i - x_j from the mixed values,     */
/* x_i -= alpha m, x_j += alpha m, xt_i -= alpha_t m, xt_j += alpha_t m.        */
/* ------------------------------------------------------------------------- */
void a2o_gossip_event(double *x_i, double *xt_i, double *t_i, double rate_i,
                      double *x_j, double *xt_j, double *t_j, double rate_j, int64_t d,
                      double eta, double te, double alpha, double alpha_t)
{
    a2o_mix_row(x_i, xt_i, d, eta, rate_i * (te - *t_i));
    *t_i = te;
    a2o_mix_row(x_j, xt_j, d, eta, rate_j * (te - *t_j));
    *t_j = te;
    for (int64_t k = 0; k < d; ++k) {
        const double m = x_i[k] - x_j[k];
        x_i[k] -= alpha * m;
        x_j[k] += alpha * m;
        xt_i[k] -= alpha_t * m;
        xt_j[k] += alpha_t * m;
    }
}

/* ------------------------------------------------------------------------- */
/* The same two jumps in the order in which Algorithm 1 LISTS its lines: the     */
/* gradient g (resp. the difference m_ij) is formed from the stored, not yet    */
/* mixed values, then the worker is mixed to te, then the jump is applied.  In   */
/* a real system g takes a whole forward/backward pass and is stale in exactly   */
/* this way.  Kept as a variant; the default reading is the one above.           */
/* ------------------------------------------------------------------------- */
void a2o_gradient_event_listing(double *x_i, double *xt_i, double *t_i, double rate_i, int64_t d,
                                double eta, double te, double gamma, double gscale,
                                const double *c, const double *xi, const double *h)
{
    double *g = (double *)malloc(sizeof(double) * (size_t)d);
    for (int64_t k = 0; k < d; ++k) g[k] = a2o_local_gradient(x_i[k], k, gscale, c, xi, h);
    a2o_mix_row(x_i, xt_i, d, eta, rate_i * (te - *t_i));
    *t_i = te;
    for (int64_t k = 0; k < d; ++k) {
        x_i[k] -= gamma * g[k];
        xt_i[k] -= gamma * g[k];
    }
    free(g);
}

void a2o_gossip_event_listing(double *x_i, double *xt_i, double *t_i, double rate_i,
                              double *x_j, double *xt_j, double *t_j, double rate_j, int64_t d,
                              double eta, double te, double alpha, double alpha_t)
{
    double *m = (double *)malloc(sizeof(double) * (size_t)d);
    for (int64_t k = 0; k < d; ++k) m[k] = x_i[k] - x_j[k];
    a2o_mix_row(x_i, xt_i, d, eta, rate_i * (te - *t_i));
    *t_i = te;
    a2o_mix_row(x_j, xt_j, d, eta, rate_j * (te - *t_j));
    *t_j = te;
    for (int64_t k = 0; k < d; ++k) {
        x_i[k] -= alpha * m[k];
        x_j[k] += alpha * m[k];
        xt_i[k] -= alpha_t * m[k];
        xt_j[k] += alpha_t * m[k];
    }
    free(m);
}

/* ------------------------------------------------------------------------- */
/* Serial event loop.  x, xt are n x d row-major, t has n entries.              */
/* kind[e] == 0: gradient on worker wi[e]; kind[e] == 1: gossip on (wi, wj).    */
/* xi_row[e] / c_row[e] / h_row[e] index rows of the dense matrices xi / c / h  */
/* (or -1: none; the row arrays themselves may be NULL).                        */
/* order 0: jumps evaluated after the mixing (Eq. (1)); order 1: Algorithm 1's    */
/* listing order (see above).                                                   */
/* rate (n entries, may be NULL: all 1): the speed of every worker's clock, read */
/* and updated; speed[e] > 0 on a gradient event sets its worker's rate after   */
/* the event (speed may be NULL).                                               */
/* Returns 0, or -(e+1) for the first malformed event (nothing after it runs).  */
/* ------------------------------------------------------------------------- */
int64_t a2o_apply_events(int32_t n, int64_t d, double *x, double *xt, double *t,
                         double eta, double alpha, double alpha_t,
                         int64_t n_events, const double *te, const int32_t *kind,
                         const int32_t *wi, const int32_t *wj,
                         const double *gamma, const double *gscale,
                         const int64_t *xi_row, const double *xi,
                         const int64_t *c_row, const double *c,
                         const int64_t *h_row, const double *h, int32_t order,
                         double *rate, const double *speed)
{
    for (int64_t e = 0; e < n_events; ++e) {
        const int32_t i = wi[e];
        if (i < 0 || i >= n) return -(e + 1);
        const double rate_i = rate ? rate[i] : 1.0;
        if (kind[e] == 0) {
            if (te[e] < t[i]) return -(e + 1);
            const double *ce = (c_row && c_row[e] >= 0) ? c + c_row[e] * d : NULL;
            const double *xe = (xi_row && xi_row[e] >= 0) ? xi + xi_row[e] * d : NULL;
            const double *he = (h_row && h_row[e] >= 0) ? h + h_row[e] * d : NULL;
            (order ? a2o_gradient_event_listing : a2o_gradient_event)(
                x + (int64_t)i * d, xt + (int64_t)i * d, t + i, rate_i, d, eta, te[e], gamma[e], gscale[e], ce, xe, he);
            /* the finished gradient step sets the speed of the worker's clock from here on */
            if (rate && speed && speed[e] > 0.0) rate[i] = speed[e];
        } else if (kind[e] == 1) {
            const int32_t j = wj[e];
            if (j < 0 || j >= n || j == i) return -(e + 1);
            if (te[e] < t[i] || te[e] < t[j]) return -(e + 1);
            (order ? a2o_gossip_event_listing : a2o_gossip_event)(
                x + (int64_t)i * d, xt + (int64_t)i * d, t + i, rate_i,
                x + (int64_t)j * d, xt + (int64_t)j * d, t + j, rate ? rate[j] : 1.0, d, eta, te[e], alpha, alpha_t);
        } else {
            return -(e + 1);
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Observables at a common time t_now >= max_i t_i, on a COPY of the state      */
/* mixed to t_now (the stored state is not modified):                           */
/*   consensus distance ||pi x||_F^2 = sum_i ||x_i - xbar||^2 (appendix,        */
/*   "Notations"), the same for xt, and the per-worker coordinate sums.         */
/* ------------------------------------------------------------------------- */
int a2o_stats(int32_t n, int64_t d, const double *x, const double *xt, const double *t,
              double eta, double t_now,
              double *consensus_x, double *consensus_xt, double *sum_x, double *sum_xt, const double *rate)
{
    double *mx = (double *)malloc(sizeof(double) * (size_t)n * (size_t)d);
    double *mxt = (double *)malloc(sizeof(double) * (size_t)n * (size_t)d);
    if (!mx || !mxt) { free(mx); free(mxt); return -1; }
    memcpy(mx, x, sizeof(double) * (size_t)n * (size_t)d);
    memcpy(mxt, xt, sizeof(double) * (size_t)n * (size_t)d);
    for (int32_t i = 0; i < n; ++i)
        a2o_mix_row(mx + (int64_t)i * d, mxt + (int64_t)i * d, d, eta, (rate ? rate[i] : 1.0) * (t_now - t[i]));

    double cx = 0.0, cxt = 0.0;
    for (int64_t k = 0; k < d; ++k) {
        double bar = 0.0, bart = 0.0;
        for (int32_t i = 0; i < n; ++i) { bar += mx[(int64_t)i * d + k]; bart += mxt[(int64_t)i * d + k]; }
        bar /= n; bart /= n;
        for (int32_t i = 0; i < n; ++i) {
            const double u = mx[(int64_t)i * d + k] - bar;
            const double v = mxt[(int64_t)i * d + k] - bart;
            cx += u * u;
            cxt += v * v;
        }
    }
    for (int32_t i = 0; i < n; ++i) {
        double s = 0.0, st = 0.0;
        for (int64_t k = 0; k < d; ++k) { s += mx[(int64_t)i * d + k]; st += mxt[(int64_t)i * d + k]; }
        sum_x[i] = s; sum_xt[i] = st;
    }
    *consensus_x = cx; *consensus_xt = cxt;
    free(mx); free(mxt);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as      */
/* easy as 1, 2, 3", SC'11): ten rounds of two 32x32->64 multiplies with a      */
/* Weyl-sequence key schedule.  Written from the published description.         */
/* ------------------------------------------------------------------------- */
void a2o_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* ------------------------------------------------------------------------- */
/* Event source: independent Poisson point processes (Assumption 3.1): one per  */
/* node (gradient clock, rate node_rate[i]) and one per edge (communication     */
/* clock, rate edge_rate[e]).  Clock ids: nodes 0..n-1, then edges in edge-list */
/* order.  The k-th inter-arrival of clock c is -log1p(-u)/rate with u the      */
/* 53-bit uniform in [0,1) made of Philox4x32-10(counter = (k_lo, k_hi, c,      */
/* 0x0A2C1D20), key = (seed_lo, seed_hi)) words 0 (high 32 bits) and 1 (top 21  */
/* bits).  Arrival times are running fp64 sums.  The merged stream is built by  */
/* repeatedly taking the clock with the smallest next arrival (a plain linear   */
/* scan; ties go to the lower clock id).  A rate of 0 means the clock never     */
/* fires.  Outputs: te, kind (0 gradient, 1 gossip), wi, wj (-1 for gradient),  */
/* clock id.  Returns the number of events written (< n_events only if every    */
/* clock is dead).                                                              */
/* ------------------------------------------------------------------------- */
static double a2o_interarrival(uint64_t seed, uint32_t clock, uint64_t k, double rate)
{
    uint32_t ctr[4] = { (uint32_t)k, (uint32_t)(k >> 32), clock, 0x0A2C1D20u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t r[4];
    a2o_philox4x32_10(ctr, key, r);
    const uint64_t bits = ((uint64_t)r[0] << 21) | (uint64_t)(r[1] >> 11);
    const double u = (double)bits * 0x1.0p-53;
    return -log1p(-u) / rate;
}

int64_t a2o_generate_events(int32_t n, int32_t n_edges, const int32_t *eu, const int32_t *ev,
                            const double *node_rate, const double *edge_rate, uint64_t seed,
                            int64_t n_events, double *te, int32_t *kind, int32_t *wi, int32_t *wj,
                            int32_t *clock_id)
{
    const int32_t n_clocks = n + n_edges;
    double *next = (double *)malloc(sizeof(double) * (size_t)n_clocks);
    uint64_t *draws = (uint64_t *)calloc((size_t)n_clocks, sizeof(uint64_t));
    if (!next || !draws) { free(next); free(draws); return -1; }
    for (int32_t c = 0; c < n_clocks; ++c) {
        const double rate = c < n ? node_rate[c] : edge_rate[c - n];
        if (rate > 0.0) { next[c] = a2o_interarrival(seed, (uint32_t)c, 0, rate); draws[c] = 1; }
        else next[c] = INFINITY;
    }
    int64_t written = 0;
    while (written < n_events) {
        int32_t best = 0;
        for (int32_t c = 1; c < n_clocks; ++c)
            if (next[c] < next[best]) best = c;
        if (!(next[best] < INFINITY)) break;
        te[written] = next[best];
        clock_id[written] = best;
        if (best < n) { kind[written] = 0; wi[written] = best; wj[written] = -1; }
        else { kind[written] = 1; wi[written] = eu[best - n]; wj[written] = ev[best - n]; }
        ++written;
        const double rate = best < n ? node_rate[best] : edge_rate[best - n];
        next[best] += a2o_interarrival(seed, (uint32_t)best, draws[best], rate);
        ++draws[best];
    }
    free(next); free(draws);
    return written;
}
