// Host side of the A2CiD2 engine: error reporting, graph quantities (Definition 3.1,
// chi_1, chi_2, Proposition 3.2), the batch planner (validation + mixing coefficients of
// Algorithm 1's matrix-exponential step) and the Poisson-clock event scheduler
// (Assumption 3.1) with its level packing.  No GPU code in this file.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstddef>
#include <cstdio>
#include <cstring>
#include <limits>
#include <new>
#include <deque>
#include <queue>
#include <tuple>
#include <utility>

#include "a2cid_internal.h"

namespace a2cid {

static thread_local char g_error[512] = "";

int fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return code;
}

void clear_error() { g_error[0] = '\0'; }

int load_graph(Graph &g, int32_t n, const a2cid_graph *src) {
    if (n < 2 || n > A2CID_MAX_WORKERS)
        return fail(A2CID_EINVAL, "n = %d outside [2, %d]", n, A2CID_MAX_WORKERS);
    if (!src) return fail(A2CID_EINVAL, "graph is NULL");
    if (src->n_edges < 0) return fail(A2CID_EGRAPH, "n_edges = %d is negative", src->n_edges);
    if (src->n_edges > 0 && (!src->u || !src->v || !src->rate))
        return fail(A2CID_EINVAL, "graph arrays are NULL");
    g.n = n;
    g.u.assign(src->u, src->u + src->n_edges);
    g.v.assign(src->v, src->v + src->n_edges);
    g.rate.assign(src->rate, src->rate + src->n_edges);
    g.adj.assign((size_t)n * n, 0);
    for (int32_t e = 0; e < src->n_edges; ++e) {
        const int32_t a = g.u[e], b = g.v[e];
        if (a < 0 || b >= n || a >= b)
            return fail(A2CID_EGRAPH, "edge %d = (%d, %d) must satisfy 0 <= u < v < n", e, a, b);
        if (!(g.rate[e] >= 0.0) || !std::isfinite(g.rate[e]))
            return fail(A2CID_EGRAPH, "edge %d has rate %g (must be finite and >= 0)", e, g.rate[e]);
        if (g.adj[(size_t)a * n + b]) return fail(A2CID_EGRAPH, "edge %d = (%d, %d) is a duplicate", e, a, b);
        g.adj[(size_t)a * n + b] = g.adj[(size_t)b * n + a] = 1;
    }
    return A2CID_OK;
}

double mix_coefficient(double eta, double tau) {
    // (1 - e^{-2 eta tau}) / 2 without cancellation for small eta * tau
    return -0.5 * std::expm1(-2.0 * eta * tau);
}

// ------------------------------------------------------------------------------------------
// Eigenvalues of a symmetric matrix (row-major, destroyed): Householder reduction to tridiagonal
// form followed by the implicit-shift QL iteration (Wilkinson & Reinsch), eigenvalues only.
// O(n^3) once: a second for n = 1024, the largest Laplacian the library accepts.
// Returns false if the QL iteration does not converge.
// ------------------------------------------------------------------------------------------
static bool symmetric_eigenvalues(int n, std::vector<double> &a, std::vector<double> &diag) {
    std::vector<double> off(n, 0.0), p(n);
    diag.assign(n, 0.0);
    auto A = [&](int r, int c) -> double & { return a[(size_t)r * n + c]; };
    // Householder: row i of the (lower triangle of the) leading (i+1) x (i+1) block is reflected onto e_{i-1}
    for (int i = n - 1; i >= 1; --i) {
        const int l = i - 1;
        double scale = 0.0, h = 0.0;
        if (l > 0) {
            for (int k = 0; k <= l; ++k) scale += std::fabs(A(i, k));
            if (scale == 0.0) {
                off[i] = A(i, l);
            } else {
                for (int k = 0; k <= l; ++k) { A(i, k) /= scale; h += A(i, k) * A(i, k); }
                const double f = A(i, l);
                const double g = f >= 0.0 ? -std::sqrt(h) : std::sqrt(h);
                off[i] = scale * g;
                h -= f * g;
                A(i, l) = f - g;                       // row i now holds the Householder vector u, h = |u|^2 / 2
                double dot = 0.0;
                for (int j = 0; j <= l; ++j) {         // p = B u / h with B the leading block (lower triangle stored)
                    double acc = 0.0;
                    for (int k = 0; k <= j; ++k) acc += A(j, k) * A(i, k);
                    for (int k = j + 1; k <= l; ++k) acc += A(k, j) * A(i, k);
                    p[j] = acc / h;
                    dot += p[j] * A(i, j);
                }
                const double kappa = dot / (h + h);
                for (int j = 0; j <= l; ++j) p[j] -= kappa * A(i, j);          // q = p - kappa u
                for (int j = 0; j <= l; ++j) {                                 // B <- B - u q^T - q u^T
                    const double uj = A(i, j), qj = p[j];
                    for (int k = 0; k <= j; ++k) A(j, k) -= uj * p[k] + qj * A(i, k);
                }
            }
        } else {
            off[i] = A(i, l);
        }
    }
    for (int i = 0; i < n; ++i) diag[i] = A(i, i);
    // implicit QL on the tridiagonal (diag, off), off[i] coupling i-1 and i
    for (int i = 1; i < n; ++i) off[i - 1] = off[i];
    off[n - 1] = 0.0;
    for (int l = 0; l < n; ++l) {
        for (int iter = 0;; ++iter) {
            int m = l;
            for (; m < n - 1; ++m) {
                const double dd = std::fabs(diag[m]) + std::fabs(diag[m + 1]);
                if (std::fabs(off[m]) <= 2.3e-16 * dd) break;
            }
            if (m == l) break;
            if (iter == 200) return false;
            double g = (diag[l + 1] - diag[l]) / (2.0 * off[l]);
            double r = std::hypot(g, 1.0);
            g = diag[m] - diag[l] + off[l] / (g + (g >= 0.0 ? std::fabs(r) : -std::fabs(r)));
            double sn = 1.0, cs = 1.0, shift = 0.0;
            int i = m - 1;
            for (; i >= l; --i) {
                double f = sn * off[i];
                const double bb = cs * off[i];
                r = std::hypot(f, g);
                off[i + 1] = r;
                if (r == 0.0) { diag[i + 1] -= shift; off[m] = 0.0; break; }
                sn = f / r;
                cs = g / r;
                g = diag[i + 1] - shift;
                r = (diag[i] - g) * sn + 2.0 * cs * bb;
                shift = sn * r;
                diag[i + 1] = g + shift;
                g = cs * r - bb;
            }
            if (r == 0.0 && i >= l) continue;
            diag[l] -= shift;
            off[l] = g;
            off[m] = 0.0;
        }
    }
    return true;
}

// Inverse of a symmetric positive definite matrix (row-major, overwritten) by Cholesky factorisation.
// Returns false if a pivot is not positive.
static bool spd_inverse(int n, std::vector<double> &a) {
    auto A = [&](int r, int c) -> double & { return a[(size_t)r * n + c]; };
    for (int j = 0; j < n; ++j) {                      // A = G G^T, G lower triangular, stored in place
        double dj = A(j, j);
        for (int k = 0; k < j; ++k) dj -= A(j, k) * A(j, k);
        if (!(dj > 0.0)) return false;
        dj = std::sqrt(dj);
        A(j, j) = dj;
        for (int i = j + 1; i < n; ++i) {
            double v = A(i, j);
            for (int k = 0; k < j; ++k) v -= A(i, k) * A(j, k);
            A(i, j) = v / dj;
        }
    }
    for (int j = 0; j < n; ++j) {                      // G <- G^{-1} (lower triangular), column by column
        A(j, j) = 1.0 / A(j, j);
        for (int i = j + 1; i < n; ++i) {
            double v = 0.0;
            for (int k = j; k < i; ++k) v -= A(i, k) * A(k, j);
            A(i, j) = v / A(i, i);
        }
    }
    for (int i = 0; i < n; ++i)                         // A^{-1} = G^{-T} G^{-1}: upper triangle first, then mirror
        for (int j = i; j < n; ++j) {
            double v = 0.0;
            for (int k = j; k < n; ++k) v += A(k, i) * A(k, j);
            A(i, j) = v;                                // safe: column entries A(k, i), A(k, j) with k >= j >= i, row i < k
        }
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < i; ++j) A(i, j) = A(j, i);
    return true;
}

static bool connected(const Graph &g) {
    std::vector<std::vector<int32_t>> nb(g.n);
    for (size_t e = 0; e < g.u.size(); ++e)
        if (g.rate[e] > 0.0) { nb[g.u[e]].push_back(g.v[e]); nb[g.v[e]].push_back(g.u[e]); }
    std::vector<char> seen(g.n, 0);
    std::vector<int32_t> stack{0};
    seen[0] = 1;
    int32_t count = 1;
    while (!stack.empty()) {
        const int32_t a = stack.back();
        stack.pop_back();
        for (int32_t b : nb[a])
            if (!seen[b]) { seen[b] = 1; ++count; stack.push_back(b); }
    }
    return count == g.n;
}

// ------------------------------------------------------------------------------------------
// Batch planner
// ------------------------------------------------------------------------------------------
int plan_batch(const Graph &g, double eta, const double *t_now, const double *rate_now, const a2cid_event_batch *batch,
               Plan &plan, PlanScratch &scratch) {
    if (!batch) return fail(A2CID_EINVAL, "batch is NULL");
    if (batch->n_ops < 0 || batch->n_levels < 0) return fail(A2CID_EINVAL, "negative batch size");
    if (batch->n_ops > 0 && !batch->ops) return fail(A2CID_EINVAL, "batch->ops is NULL");
    if (!batch->level_off) return fail(A2CID_EINVAL, "batch->level_off is NULL");
    if (batch->level_off[0] != 0 || batch->level_off[batch->n_levels] != batch->n_ops)
        return fail(A2CID_EMATCHING, "level_off must start at 0 and end at n_ops");
    const int32_t n = g.n;
    plan.coef.assign((size_t)batch->n_ops, a2cid_coef{0.f, 0.f, 0.f, 0.f});
    plan.t_after.assign(t_now, t_now + n);
    if (rate_now) plan.rate_after.assign(rate_now, rate_now + n);
    else plan.rate_after.assign(n, 1.0);
    plan.n_gossip = plan.n_grad = plan.n_grad_xi = plan.n_grad_c = plan.n_grad_h = 0;
    scratch.level_stamp.assign(n, 0);
    scratch.last_op.assign(n, -1);
    const bool sync = std::isfinite(batch->t_sync);
    if (!sync && !std::isnan(batch->t_sync)) return fail(A2CID_EINVAL, "t_sync must be finite or NaN");

    for (int32_t l = 0; l < batch->n_levels; ++l) {
        const int64_t lo = batch->level_off[l], hi = batch->level_off[l + 1];
        if (hi < lo || hi > batch->n_ops) return fail(A2CID_EMATCHING, "level_off not monotone at level %d", l);
        for (int64_t k = lo; k < hi; ++k) {
            const a2cid_op &op = batch->ops[k];
            if (!std::isfinite(op.t)) return fail(A2CID_EINVAL, "op %lld: time is not finite", (long long)k);
            if (op.i < 0 || op.i >= n) return fail(A2CID_EINVAL, "op %lld: worker i = %d out of range", (long long)k, op.i);
            int32_t ends[2] = {op.i, -1};
            if (op.kind == A2CID_KIND_GOSSIP) {
                if (op.j < 0 || op.j >= n || op.j == op.i)
                    return fail(A2CID_EINVAL, "op %lld: worker j = %d invalid", (long long)k, op.j);
                if (!g.has_edge(op.i, op.j))
                    return fail(A2CID_EGRAPH, "op %lld: (%d, %d) is not an edge of the graph", (long long)k, op.i, op.j);
                ends[1] = op.j;
                ++plan.n_gossip;
            } else if (op.kind == A2CID_KIND_GRADIENT) {
                if (!std::isfinite(op.gamma) || !std::isfinite(op.gscale))
                    return fail(A2CID_EINVAL, "op %lld: gamma / gscale not finite", (long long)k);
                if (((uintptr_t)op.xi | (uintptr_t)op.c | (uintptr_t)op.h) & 15u)
                    return fail(A2CID_EALIGN, "op %lld: xi / c / h must be 16-byte aligned", (long long)k);
                if (!(op.clock_rate >= 0.f) || !std::isfinite(op.clock_rate))
                    return fail(A2CID_EINVAL, "op %lld: clock_rate must be finite and >= 0", (long long)k);
                ++plan.n_grad;
                if (op.xi) ++plan.n_grad_xi;
                if (op.c && op.gscale != 0.f) ++plan.n_grad_c;
                if (op.h && op.gscale != 0.f) ++plan.n_grad_h;
            } else {
                return fail(A2CID_EINVAL, "op %lld: unknown kind %d", (long long)k, op.kind);
            }
            if (sync && op.t > batch->t_sync)
                return fail(A2CID_EORDER, "op %lld: time %.17g is after t_sync %.17g", (long long)k, op.t, batch->t_sync);
            float *b_pre[2] = {&plan.coef[k].b_pre_i, &plan.coef[k].b_pre_j};
            for (int s = 0; s < 2; ++s) {
                const int32_t w = ends[s];
                if (w < 0) continue;
                if (scratch.level_stamp[w] == (int64_t)l + 1)
                    return fail(A2CID_EMATCHING, "level %d: worker %d appears in two operations", l, w);
                scratch.level_stamp[w] = (int64_t)l + 1;
                const double tau = op.t - plan.t_after[w];
                if (tau < 0.0)
                    return fail(A2CID_EORDER, "op %lld: time %.17g is before worker %d's time %.17g",
                                (long long)k, op.t, w, plan.t_after[w]);
                *b_pre[s] = (float)mix_coefficient(eta, plan.rate_after[w] * tau);
                plan.t_after[w] = op.t;
                scratch.last_op[w] = k;
            }
            // the finished gradient step sets the speed of the worker's clock from here on
            if (op.kind == A2CID_KIND_GRADIENT && op.clock_rate > 0.f) plan.rate_after[op.i] = (double)op.clock_rate;
        }
    }
    if (sync) {
        for (int32_t w = 0; w < n; ++w) {
            const int64_t k = scratch.last_op[w];
            if (k < 0) continue;
            const float b = (float)mix_coefficient(eta, plan.rate_after[w] * (batch->t_sync - plan.t_after[w]));
            if (batch->ops[k].i == w) plan.coef[k].b_post_i = b; else plan.coef[k].b_post_j = b;
            plan.t_after[w] = batch->t_sync;
        }
    }
    return A2CID_OK;
}

// ------------------------------------------------------------------------------------------
// Scheduler
// ------------------------------------------------------------------------------------------
static inline void philox4x32_10(uint32_t c[4], uint32_t k0, uint32_t k1) {
    // Philox4x32-10 of Salmon et al. (SC'11): ten S-P rounds; the key follows a Weyl sequence.
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    for (int round = 0; round < 10; ++round) {
        const uint64_t lo = (uint64_t)M0 * c[0], hi = (uint64_t)M1 * c[2];
        const uint32_t y0 = (uint32_t)(hi >> 32) ^ c[1] ^ k0;
        const uint32_t y2 = (uint32_t)(lo >> 32) ^ c[3] ^ k1;
        c[1] = (uint32_t)hi;
        c[3] = (uint32_t)lo;
        c[0] = y0;
        c[2] = y2;
        k0 += W0;
        k1 += W1;
    }
}

}  // namespace a2cid

using namespace a2cid;

struct a2cid_sched {
    Graph g;
    std::vector<double> rate;        // per clock: workers, then edges
    std::vector<uint64_t> draws;     // waiting times drawn so far, per clock
    std::vector<int64_t> fired;      // events produced so far, per clock
    uint64_t seed = 0;
    int64_t serial = 0;              // serial index of the next event
    using Entry = std::pair<double, int32_t>;   // (arrival time, clock id): ties -> lower id first
    std::priority_queue<Entry, std::vector<Entry>, std::greater<Entry>> heap;
    // storage behind the batch handed out by a2cid_sched_next
    std::vector<a2cid_op> raw, ops;
    std::vector<int32_t> level_of;
    std::vector<int64_t> level_off, cursor;
    std::vector<int32_t> last_level;

    // ---- first-in-first-out pairing source (a2cid_sched_create_fifo) -------------------------------
    bool fifo = false;
    double comm_per_grad = 0.0, comm_time = 0.0, jitter = 0.0;
    std::vector<uint64_t> count_draws;           // uniforms used so far for the Poisson counts, per worker
    std::vector<int64_t> todo;                   // averagings a worker still has to do
    std::vector<char> busy, queued;
    std::vector<int32_t> waiting;                // available workers, oldest first
    std::vector<int32_t> edge_of;                // n x n: index of edge {a, b}, or -1
    using Completion = std::tuple<double, int32_t, int32_t>;   // (time, 0 averaging ends / 1 step ends, worker)
    std::priority_queue<Completion, std::vector<Completion>, std::greater<Completion>> completions;
    std::deque<a2cid_op> emitted;                // events produced by the last completion, not yet handed out
    // normalised clock: time advances by (real time elapsed) / (average duration of the gradient steps completed
    // so far), so that a gradient step takes one unit of it
    bool normalize = false;
    double unit = 1.0, dur_sum = 0.0, t_norm = 0.0, real_last = 0.0;
    int64_t dur_n = 0;
    // the same per worker: stamps stay in real time, every gradient event carries the speed of its worker's own clock,
    // 1 / (average duration of that worker's completed steps)
    bool per_worker = false;
    std::vector<double> own_sum;
    std::vector<int64_t> own_n;
    std::vector<double> running;                 // duration of the gradient step each worker is in

    double uniform(uint64_t k, uint32_t stream, uint32_t tag) const {
        uint32_t c[4] = {(uint32_t)k, (uint32_t)(k >> 32), stream, tag};
        philox4x32_10(c, (uint32_t)seed, (uint32_t)(seed >> 32));
        const uint64_t mantissa = ((uint64_t)c[0] << 21) | (c[1] >> 11);
        return std::ldexp((double)mantissa, -53);
    }

    double waiting_time(int32_t clock) {
        const double u = uniform(draws[clock]++, (uint32_t)clock, 0x0A2C1D20u);
        return -std::log1p(-u) / rate[clock];
    }

    // duration of worker w's next gradient step: mean 1 / rate, uniform within +- jitter of it
    double step_time(int32_t w) {
        const double u = uniform(draws[w]++, (uint32_t)w, 0x0A2C1D21u);
        return (1.0 / rate[w]) * (1.0 + jitter * (2.0 * u - 1.0));
    }

    // Poisson(comm_per_grad) by multiplying uniforms until the product reaches exp(-mean) (Knuth)
    int64_t comm_count(int32_t w) {
        const double limit = std::exp(-comm_per_grad);
        int64_t k = 0;
        double p = 1.0;
        do {
            ++k;
            p *= uniform(count_draws[w]++, (uint32_t)w, 0x0A2C1D22u);
        } while (p > limit);
        return k - 1;
    }

    void emit(double t, int32_t kind, int32_t i, int32_t j, int32_t clock, float clock_rate = 0.f) {
        a2cid_op op;
        std::memset(&op, 0, sizeof(op));
        op.t = t; op.kind = kind; op.i = i; op.j = j;
        op.clock_rate = clock_rate;
        op.id = serial++;
        ++fired[clock];
        emitted.push_back(op);
    }

    // one completion of the FIFO source: may emit a gradient event and any number of pairings
    bool advance_fifo() {
        if (completions.empty()) return false;
        const auto [t, what, w] = completions.top();
        completions.pop();
        t_norm += (t - real_last) / unit;
        real_last = t;
        const double stamp = normalize ? t_norm : t;
        double finished = 0.0;
        if (what == 0) {
            busy[w] = 0;
        } else {
            finished = running[w];
            float speed = 0.f;
            if (per_worker) {
                own_sum[w] += finished;
                ++own_n[w];
                speed = (float)(1.0 / (own_sum[w] / (double)own_n[w]));
            }
            emit(stamp, A2CID_KIND_GRADIENT, w, -1, w, speed);
            todo[w] += comm_count(w);
            running[w] = step_time(w);
            completions.emplace(t + running[w], 1, w);
        }
        if (!busy[w] && todo[w] > 0 && !queued[w]) { waiting.push_back(w); queued[w] = 1; }
        // the coordinator: oldest available worker first, with the oldest available neighbour of it
        for (;;) {
            size_t pa = 0, pb = 0;
            bool found = false;
            for (pa = 0; pa < waiting.size() && !found; ++pa)
                for (pb = pa + 1; pb < waiting.size(); ++pb)
                    if (edge_of[(size_t)waiting[pa] * g.n + waiting[pb]] >= 0) { found = true; break; }
            if (!found) break;
            --pa;   // the outer loop stepped once more after the hit
            const int32_t a = waiting[pa], b = waiting[pb];
            waiting.erase(waiting.begin() + (std::ptrdiff_t)pb);
            waiting.erase(waiting.begin() + (std::ptrdiff_t)pa);
            const int32_t e = edge_of[(size_t)a * g.n + b];
            emit(stamp, A2CID_KIND_GOSSIP, g.u[e], g.v[e], g.n + e);
            for (int32_t m : {a, b}) {
                --todo[m];
                busy[m] = 1;
                queued[m] = 0;
                completions.emplace(t + comm_time, 0, m);
            }
        }
        if (what == 1) {                         // the finished step counts from the next interval on
            dur_sum += finished;
            ++dur_n;
            unit = dur_sum / (double)dur_n;
        }
        return true;
    }

    bool pop(a2cid_op &op) {
        if (fifo) {
            while (emitted.empty())
                if (!advance_fifo()) return false;
            op = emitted.front();
            emitted.pop_front();
            return true;
        }
        if (heap.empty()) return false;
        const Entry e = heap.top();
        heap.pop();
        const int32_t c = e.second;
        std::memset(&op, 0, sizeof(op));
        op.t = e.first;
        if (c < g.n) { op.kind = A2CID_KIND_GRADIENT; op.i = c; op.j = -1; }
        else { op.kind = A2CID_KIND_GOSSIP; op.i = g.u[c - g.n]; op.j = g.v[c - g.n]; }
        op.id = serial++;
        ++fired[c];
        heap.emplace(e.first + waiting_time(c), c);
        return true;
    }
};

namespace a2cid {

static inline int op_endpoints(const a2cid_op &o, int32_t (&w)[2]) {
    w[0] = o.i;
    w[1] = o.j;
    return o.kind == A2CID_KIND_GOSSIP ? 2 : 1;
}

void plan_chain(int32_t n, const a2cid_op *ops, int64_t count, int32_t lds_slots, ChainPlan &s) {
    s.steps.clear();
    s.steps.reserve((size_t)count + (size_t)count / 2 + (size_t)lds_slots);
    s.bytes_per_column = 0.0;
    s.next_op.assign(2 * (size_t)count, -1);
    s.waiting.assign((size_t)count, 0);
    s.emitted.assign((size_t)count, 0);
    s.head.assign(n, -1);
    s.last.assign(n, -1);
    s.where.assign(n, A2CID_LOC_MEMORY);
    s.owner.assign(lds_slots, -1);
    s.recent.clear();
    int32_t w[2];
    for (int64_t k = 0; k < count; ++k) {
        const int ne = op_endpoints(ops[k], w);
        for (int e = 0; e < ne; ++e) {
            const int32_t p = s.last[w[e]];
            if (p >= 0) {
                s.next_op[2 * (size_t)p + (ops[p].i == w[e] ? 0 : 1)] = (int32_t)k;
                ++s.waiting[k];
            } else {
                s.head[w[e]] = (int32_t)k;
            }
            s.last[w[e]] = (int32_t)k;
        }
    }
    const int32_t never = INT32_MAX;
    auto next_use = [&](int32_t worker) { return s.head[worker] >= 0 ? s.head[worker] : never; };

    int64_t scan = 0;
    int64_t prev = -1;                  // index into steps of the last operation step; its dst_* are still open
    int32_t pw[2] = {-1, -1};           // its workers, as (row_i, row_j)
    int npw = 0;

    // Closes the previous operation's step: where its workers' columns go, given the workers of the next one.
    auto close_prev = [&](const int32_t *nw, int nn) {
        if (prev < 0) return;
        auto used_next = [&](int32_t worker) { return (nn > 0 && nw[0] == worker) || (nn > 1 && nw[1] == worker); };
        int32_t carried = -1;
        for (int e = 0; e < npw && carried < 0; ++e)
            if (used_next(pw[e])) carried = pw[e];
        for (int e = 0; e < npw; ++e) {
            const int32_t worker = pw[e];
            const uint8_t at = s.where[worker];             // where the operation found it
            uint8_t dst = A2CID_LOC_MEMORY;
            if (worker == carried) {
                dst = A2CID_LOC_CARRY;
            } else if (next_use(worker) != never) {
                if (at >= A2CID_LOC_SLOT0) {
                    dst = at;                               // stays in its slot
                } else {
                    int32_t slot = -1;
                    for (int32_t q = 0; q < lds_slots && slot < 0; ++q)
                        if (s.owner[q] < 0) slot = q;
                    if (slot < 0) {
                        // the parked worker whose next operation is farthest away makes room if it is farther
                        // than this worker's; workers of the previous and of the next operation stay
                        int32_t far = -1;
                        for (int32_t q = 0; q < lds_slots; ++q) {
                            const int32_t v = s.owner[q];
                            if (v == pw[0] || (npw > 1 && v == pw[1]) || used_next(v)) continue;
                            if (far < 0 || next_use(v) > next_use(s.owner[far])) far = q;
                        }
                        if (far >= 0 && next_use(s.owner[far]) > next_use(worker)) {
                            a2cid_chain_step spill{};
                            spill.op = -1;
                            spill.row_i = s.owner[far];
                            spill.row_j = -1;
                            spill.src_i = (uint8_t)(A2CID_LOC_SLOT0 + far);
                            s.steps.insert(s.steps.begin() + prev, spill);   // before the step that re-uses the slot
                            ++prev;
                            s.bytes_per_column += 8.0;
                            s.where[s.owner[far]] = A2CID_LOC_MEMORY;
                            s.owner[far] = -1;
                            slot = far;
                        }
                    }
                    if (slot >= 0) {
                        dst = (uint8_t)(A2CID_LOC_SLOT0 + slot);
                        s.owner[slot] = worker;
                    }
                }
            }
            if (at >= A2CID_LOC_SLOT0 && dst != at) s.owner[at - A2CID_LOC_SLOT0] = -1;
            if (dst == A2CID_LOC_MEMORY) s.bytes_per_column += 8.0;
            s.where[worker] = dst;
            (e == 0 ? s.steps[prev].dst_i : s.steps[prev].dst_j) = dst;
        }
    };

    for (int64_t out = 0; out < count; ++out) {
        // candidates: pending operations of nearby workers, fewest rows to fetch from memory first
        int32_t pick = -1, pick_miss = 3;
        auto near_by = [&](int32_t worker) {
            return s.where[worker] != A2CID_LOC_MEMORY || (npw > 0 && pw[0] == worker) || (npw > 1 && pw[1] == worker);
        };
        auto consider = [&](int32_t worker) {
            const int32_t k = s.head[worker];
            if (k < 0 || s.waiting[k] != 0) return;
            int32_t v[2];
            const int ne = op_endpoints(ops[k], v);
            int32_t miss = 0;
            for (int e = 0; e < ne; ++e) miss += near_by(v[e]) ? 0 : 1;
            if (miss < pick_miss) { pick = k; pick_miss = miss; }
        };
        for (int e = 0; e < npw; ++e) consider(pw[e]);
        for (size_t r = 0; r < s.recent.size(); ++r) consider(s.recent[r]);
        for (int32_t q = 0; q < lds_slots; ++q)
            if (s.owner[q] >= 0) consider(s.owner[q]);
        if (pick < 0) {
            // the earliest operation not yet emitted: everything it waits for has a smaller index, so it is free
            while (s.emitted[scan]) ++scan;
            pick = (int32_t)scan;
        }
        s.emitted[pick] = 1;
        const int ne = op_endpoints(ops[pick], w);
        close_prev(w, ne);

        a2cid_chain_step step{};
        step.op = pick;
        // the worker that sits in the carry registers, if any, is presented as row_i
        const bool turn = ne == 2 && s.where[w[1]] == A2CID_LOC_CARRY;
        step.row_i = turn ? w[1] : w[0];
        step.row_j = ne == 2 ? (turn ? w[0] : w[1]) : -1;
        step.src_i = s.where[step.row_i];
        step.src_j = ne == 2 ? s.where[step.row_j] : (uint8_t)A2CID_LOC_MEMORY;
        if (step.src_i == A2CID_LOC_MEMORY) s.bytes_per_column += 8.0;
        if (ne == 2 && step.src_j == A2CID_LOC_MEMORY) s.bytes_per_column += 8.0;
        if (ops[pick].kind == A2CID_KIND_GRADIENT)
            s.bytes_per_column += (ops[pick].xi ? 4.0 : 0.0) + ((ops[pick].c && ops[pick].gscale != 0.f) ? 4.0 : 0.0) +
                                  ((ops[pick].h && ops[pick].gscale != 0.f) ? 4.0 : 0.0);
        prev = (int64_t)s.steps.size();
        s.steps.push_back(step);
        pw[0] = step.row_i; pw[1] = step.row_j; npw = ne;

        for (int e = 0; e < ne; ++e) {
            const int32_t nx = s.next_op[2 * (size_t)pick + e];
            s.head[w[e]] = nx;
            if (nx >= 0) --s.waiting[nx];
            auto it = std::find(s.recent.begin(), s.recent.end(), w[e]);
            if (it != s.recent.end()) s.recent.erase(it);
            s.recent.insert(s.recent.begin(), w[e]);
        }
        if (s.recent.size() > kChainRecent) s.recent.resize(kChainRecent);
    }
    close_prev(nullptr, 0);
    // a worker is parked only while an operation of it is pending, and by now none is: the slots are empty
    for (int32_t q = 0; q < lds_slots; ++q) {
        if (s.owner[q] < 0) continue;
        a2cid_chain_step spill{};                // guard: never reached
        spill.op = -1;
        spill.row_i = s.owner[q];
        spill.row_j = -1;
        spill.src_i = (uint8_t)(A2CID_LOC_SLOT0 + q);
        s.steps.push_back(spill);
        s.bytes_per_column += 8.0;
        s.where[s.owner[q]] = A2CID_LOC_MEMORY;
        s.owner[q] = -1;
    }
}


// ---- resident kernel: launch shape and per-wave programmes -------------------------------------------------

void resident_shape(int32_t n, const a2cid_event_batch *batch, int *waves, int *cols) {
    const double per_level = batch->n_levels > 0 ? (double)batch->n_ops / (double)batch->n_levels : 1.0;
    int w = 2;
    while (w < 16 && per_level > 1.6 * w) w *= 2;       // measured break-even between 8 and 16 waves: about 13
    int c = 4;
    while (c > 1 && (size_t)n * 512 * c * (32 / w) > 160 * 1024) c /= 2;
    *waves = w;
    *cols = c;
}

void plan_resident(int32_t n, const a2cid_event_batch *batch, const a2cid_coef *coef, int waves, int cols,
                   bool trailing, int32_t *l, int64_t *k, ResidentPlan &plan) {
    const int W = waves;
    const size_t n_slots = (size_t)resident_slots(W);
    const uint32_t row_bytes = resident_row_bytes(cols);
    const int64_t sub_max = (kResSetMax / 2) * (int64_t)W;  // at most 31 operations (62 slots) per wave and level
    const uint32_t gossip_slots = trailing ? 2u : 1u;
    plan.programme.resize(W);
    for (auto &prog : plan.programme) prog.clear();
    plan.rows.clear();
    plan.grad_op.clear();
    plan.n_xi = plan.n_c = plan.n_h = 0;
    plan.slot_of.assign(n, -1);
    plan.last_grad_slot.assign(W, -1);
    plan.last_grad_level.assign(W, -1);
    plan.wave_load.assign(W, 0);
    plan.wave_slots.assign(W, 0);
    const ResSlot blank = {0u, 0u, 0u, 0u};
    auto f2u = [](float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; };
    int32_t sub_index = 0;                      // running number of the (sub-)levels of this launch
    while (*l < batch->n_levels) {
        const int64_t hi = batch->level_off[*l + 1];
        if (*k >= hi) { ++*l; continue; }
        const int64_t sub = *k, end = std::min(hi, sub + sub_max);
        // Deal the operations to the waves: gradient events first, each to the least loaded wave whose previous
        // gradient event lies furthest back (its inputs are requested when that one is done); then the gossip
        // events to the least loaded waves.
        std::fill(plan.wave_load.begin(), plan.wave_load.end(), 0);
        std::fill(plan.wave_slots.begin(), plan.wave_slots.end(), 0);
        plan.wave_of.assign((size_t)(end - sub), 0);
        for (int pass = 0; pass < 2; ++pass)
            for (int64_t q = sub; q < end; ++q) {
                const bool is_grad = batch->ops[q].kind == A2CID_KIND_GRADIENT;
                if (is_grad != (pass == 0)) continue;
                int best = 0;
                for (int w = 1; w < W; ++w) {
                    if (plan.wave_load[w] != plan.wave_load[best]) {
                        if (plan.wave_load[w] < plan.wave_load[best]) best = w;
                    } else if (is_grad && plan.last_grad_level[w] < plan.last_grad_level[best]) {
                        best = w;
                    }
                }
                plan.wave_of[(size_t)(q - sub)] = best;
                ++plan.wave_load[best];
                plan.wave_slots[best] += is_grad ? 2 : (int32_t)gossip_slots;
                if (is_grad) plan.last_grad_level[best] = sub_index;
            }
        // does every wave's programme take the (sub-)level, and still an end slot after it?
        bool full = false;
        for (int w = 0; w < W && !full; ++w) {
            size_t at = plan.programme[(size_t)w].size();
            const size_t need = 1 + (size_t)plan.wave_slots[w];
            if ((at & 63) + need > 63) at = (at + 64) & ~(size_t)63;      // a jump slot, then the next set
            if (at + need + 1 > n_slots) full = true;
        }
        if (full) break;
        // per wave: control slot, gossip operations, gradient operations; never across a set of 64 slots
        for (int w = 0; w < W; ++w) {
            auto &prog = plan.programme[(size_t)w];
            const size_t need = 1 + (size_t)plan.wave_slots[w];
            if ((prog.size() & 63) + need > 63) {
                ResSlot jump = blank;
                jump.x = kResJump;
                prog.push_back(jump);
                ResSlot pad = blank;
                pad.x = kResEnd;
                while (prog.size() & 63) prog.push_back(pad);
            }
            ResSlot ctl = blank;
            ctl.y = kResNone;
            const size_t ctl_at = prog.size();
            prog.push_back(ctl);
            uint32_t n_gos_w = 0, n_grad_w = 0;
            for (int pass = 0; pass < 2; ++pass)
                for (int64_t q = sub; q < end; ++q) {
                    if (plan.wave_of[(size_t)(q - sub)] != w) continue;
                    const a2cid_op &op = batch->ops[q];
                    const a2cid_coef &cf = coef[q];
                    const bool is_grad = op.kind == A2CID_KIND_GRADIENT;
                    if (is_grad != (pass == 1)) continue;
                    const int32_t row_i = op.i, row_j = is_grad ? op.i : op.j;
                    if (plan.slot_of[row_i] < 0) { plan.slot_of[row_i] = (int32_t)plan.rows.size(); plan.rows.push_back(row_i); }
                    if (plan.slot_of[row_j] < 0) { plan.slot_of[row_j] = (int32_t)plan.rows.size(); plan.rows.push_back(row_j); }
                    ResSlot r = blank;
                    r.x = (uint32_t)plan.slot_of[row_i] * row_bytes;
                    if (!is_grad) {
                        r.y = (uint32_t)plan.slot_of[row_j] * row_bytes;
                        r.z = f2u(cf.b_pre_i); r.w = f2u(cf.b_pre_j);
                        prog.push_back(r);
                        if (trailing) {
                            ResSlot r2 = blank;
                            r2.x = f2u(cf.b_post_i); r2.y = f2u(cf.b_post_j);
                            prog.push_back(r2);
                        }
                        ++n_gos_w;
                    } else {
                        r.y = f2u(cf.b_pre_i); r.z = f2u(op.gamma); r.w = f2u(op.gscale);
                        const uint32_t ordinal = (uint32_t)plan.grad_op.size();
                        const uintptr_t xi = op.xi ? (uintptr_t)op.xi : kResZeros;
                        plan.n_xi += op.xi != nullptr;
                        plan.n_c += op.c && op.gscale != 0.f;
                        plan.n_h += op.h && op.gscale != 0.f;
                        // the slot that names this event: the second slot of the wave's previous gradient
                        // operation, or the first slot of its programme
                        if (plan.last_grad_slot[w] < 0) {
                            prog[0].y = ordinal;
                            prog[0].z = (uint32_t)(xi & 0xffffffffu);
                            prog[0].w = (uint32_t)((uint64_t)xi >> 32);
                        } else {
                            ResSlot &from = prog[(size_t)plan.last_grad_slot[w]];
                            from.x = ordinal;
                            from.z = (uint32_t)(xi & 0xffffffffu);
                            from.w = (uint32_t)((uint64_t)xi >> 32);
                        }
                        prog.push_back(r);
                        ResSlot r2 = blank;
                        r2.x = kResNone;
                        r2.y = f2u(cf.b_post_i);
                        plan.last_grad_slot[w] = (int64_t)prog.size();
                        prog.push_back(r2);
                        plan.grad_op.push_back(q);
                        ++n_grad_w;
                    }
                }
            prog[ctl_at].x = n_gos_w | n_grad_w << 8;
        }
        ++sub_index;
        *k = end;
    }
    ResSlot end_slot = blank;
    end_slot.x = kResEnd;
    end_slot.y = kResNone;                      // also a valid first slot of an empty programme
    for (auto &prog : plan.programme) {
        prog.push_back(end_slot);
        prog.resize(n_slots, end_slot);
    }
}

void plan_regfile(int32_t n, const a2cid_event_batch *batch, const a2cid_coef *coef, int64_t max_slots, bool full,
                  uintptr_t zero_one, int64_t *k, RegPlan &plan) {
    (void)n;
    plan.programme.clear();
    plan.grad_op.clear();
    plan.touched = 0;
    plan.n_xi = plan.n_c = plan.n_h = 0;
    plan.request_at.clear();
    auto f2u = [](float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; };
    const ResSlot filler = {kRegControl << 8, 0u, 0u, 0u};
    const size_t request_slots = full ? 2 * kRegBlock : kRegBlock;
    auto whole_blocks = [](size_t slots) { return (slots + kRegBlock - 1) / kRegBlock * kRegBlock; };
    auto &prog = plan.programme;
    // a request block for the next chunk of inputs (its pointers are filled in at the end), in a block of its own
    auto request = [&](uint32_t code) {
        prog.resize(whole_blocks(prog.size()), filler);
        plan.request_at.push_back(prog.size());
        ResSlot ctl = filler;
        ctl.y = code;
        prog.push_back(ctl);
        prog.resize(prog.size() - 1 + request_slots, filler);
    };
    request(kRegRequest);                       // chunk 0
    request(kRegRequest);                       // chunk 1
    for (; *k < batch->n_ops; ++*k) {
        const a2cid_op &op = batch->ops[*k];
        const a2cid_coef &cf = coef[*k];
        const bool is_grad = op.kind == A2CID_KIND_GRADIENT;
        // a gradient event that opens a chunk of inputs (not the first chunk) comes after a switch block
        const bool opens = is_grad && !plan.grad_op.empty() && plan.grad_op.size() % kRegChunk == 0;
        const size_t at = opens ? whole_blocks(prog.size()) + request_slots : prog.size();
        const size_t need = 1 + (cf.b_post_i != 0.f) + (!is_grad && cf.b_post_j != 0.f);
        if ((int64_t)whole_blocks(at + need + 1) > max_slots) break;        // the end slot still has to fit
        if (opens) request(kRegSwitch);
        ResSlot r = {0u, 0u, 0u, 0u};
        plan.touched |= (uint64_t)1 << op.i;
        if (!is_grad) {
            plan.touched |= (uint64_t)1 << op.j;
            r.x = (uint32_t)op.i | kRegGossip << 8;
            r.y = (uint32_t)op.j;
            r.z = f2u(cf.b_pre_i); r.w = f2u(cf.b_pre_j);
        } else {
            r.x = (uint32_t)op.i | kRegGradient << 8;
            r.y = f2u(cf.b_pre_i); r.z = f2u(op.gamma); r.w = f2u(op.gscale);
            plan.n_xi += op.xi != nullptr;
            plan.n_c += op.c && op.gscale != 0.f;
            plan.n_h += op.h && op.gscale != 0.f;
            plan.grad_op.push_back(*k);
        }
        prog.push_back(r);
        if (cf.b_post_i != 0.f) prog.push_back(ResSlot{(uint32_t)op.i | kRegMix << 8, f2u(cf.b_post_i), 0u, 0u});
        if (!is_grad && cf.b_post_j != 0.f) prog.push_back(ResSlot{(uint32_t)op.j | kRegMix << 8, f2u(cf.b_post_j), 0u, 0u});
    }
    ResSlot end_slot = filler;
    end_slot.y = kRegEnd;
    prog.push_back(end_slot);
    prog.resize(whole_blocks(prog.size()), filler);
    // The pointers: request block q (in programme order) names chunk q, i.e. gradient events 8 q ... 8 q + 7 of the
    // launch; absent inputs and events past the last one: the address of a zero (or one) with bit 0 set.
    const uint64_t zeros = (uint64_t)zero_one | 1u, ones = (uint64_t)(zero_one + sizeof(float)) | 1u;
    auto put = [&](size_t slot, int e, uint64_t p) {         // pointer e (0 ... 7) of the four slots from `slot` on
        ResSlot &r = prog[slot + (size_t)e / 2];
        if (e % 2 == 0) { r.x = (uint32_t)p; r.y = (uint32_t)(p >> 32); }
        else { r.z = (uint32_t)p; r.w = (uint32_t)(p >> 32); }
    };
    for (size_t q = 0; q < plan.request_at.size(); ++q) {
        const size_t base = plan.request_at[q];
        for (int e = 0; e < kRegChunk; ++e) {
            const size_t g = q * kRegChunk + (size_t)e;
            uint64_t xi = zeros, c = zeros, h = ones;
            if (g < plan.grad_op.size()) {
                const a2cid_op &op = batch->ops[plan.grad_op[g]];
                const bool affine = op.gscale != 0.f;
                if (op.xi) xi = (uint64_t)(uintptr_t)op.xi;
                if (op.c && affine) c = (uint64_t)(uintptr_t)op.c;
                if (op.h && affine) h = (uint64_t)(uintptr_t)op.h;
            }
            put(base + 1, e, xi);
            if (full) {
                put(base + kRegBlock, e, c);
                put(base + kRegBlock + 4, e, h);
            }
        }
    }
}

// Walks a register-file programme the way the kernel does and checks everything the kernel relies on without
// testing it: whole blocks, the first request blocks, an end slot, worker indices below n (the kernel adds them to a
// register number: an index past the wave's registers is not harmless), at most kRegChunk gradient events between two
// switch slots, switch slots only at the head of a block and followed by their pointer block(s).
bool regfile_programme_ok(const std::vector<ResSlot> &prog, int32_t n, bool full) {
    const size_t request_slots = full ? 2 * kRegBlock : kRegBlock;
    if (prog.empty() || prog.size() % kRegBlock != 0 || prog.size() < 2 * request_slots + kRegBlock) return false;
    if (n < 1 || n > kRegMaxRows) return false;
    for (size_t q = 0; q < 2; ++q) {
        const ResSlot &ctl = prog[q * request_slots];
        if (ctl.x != kRegControl << 8 || ctl.y != kRegRequest) return false;
    }
    int in_chunk = 0;
    for (size_t at = 2 * request_slots; at < prog.size(); at += kRegBlock) {
        for (int j = 0; j < kRegBlock; ++j) {
            const ResSlot &r = prog[at + (size_t)j];
            const uint32_t kind = r.x >> 8, worker = r.x & 255u;
            if (kind == kRegGossip) {
                if (worker >= (uint32_t)n || r.y >= (uint32_t)n) return false;
            } else if (kind == kRegGradient) {
                if (worker >= (uint32_t)n || ++in_chunk > kRegChunk) return false;
            } else if (kind == kRegMix) {
                if (worker >= (uint32_t)n) return false;
            } else if (kind == kRegControl) {
                if (r.y == kRegEnd) return at + kRegBlock == prog.size();       // nothing after the end slot's block
                if (r.y == kRegSwitch) {
                    if (j != 0 || at + request_slots >= prog.size()) return false;
                    in_chunk = 0;
                    at += request_slots - kRegBlock;                            // the pointers are not operations
                    break;
                }
                if (r.y != 0) return false;
            } else {
                return false;
            }
        }
    }
    return false;                                                               // no end slot
}

}  // namespace a2cid

extern "C" {

const char *a2cid_last_error(void) { return g_error; }
const char *a2cid_version(void) { return "a2cid 0.1 (gfx950)"; }

int a2cid_graph_params(const a2cid_graph *graph, int32_t n, double *chi1, double *chi2,
                       double *eta, double *alpha_tilde) {
    clear_error();
    Graph g;
    if (int rc = load_graph(g, n, graph)) return rc;
    if (!connected(g)) return fail(A2CID_EGRAPH, "graph is not connected (chi_1 is infinite)");
    std::vector<double> lap((size_t)n * n, 0.0);
    double trace = 0.0;
    for (size_t e = 0; e < g.u.size(); ++e) {
        const int32_t a = g.u[e], b = g.v[e];
        lap[(size_t)a * n + a] += g.rate[e];
        lap[(size_t)b * n + b] += g.rate[e];
        lap[(size_t)a * n + b] -= g.rate[e];
        lap[(size_t)b * n + a] -= g.rate[e];
        trace += 2.0 * g.rate[e];
    }
    // chi_2: Lambda + c 1 1^T is positive definite for a connected graph and its inverse differs from the
    // pseudo-inverse only by a multiple of 1 1^T, which (e_a - e_b) does not see
    std::vector<double> inv(lap);
    const double shift = trace / ((double)n * (double)n);
    for (double &v : inv) v += shift;
    if (!spd_inverse(n, inv)) return fail(A2CID_EGRAPH, "Laplacian is not positive definite on the complement of 1");
    double worst = 0.0;
    for (size_t e = 0; e < g.u.size(); ++e) {
        const size_t a = (size_t)g.u[e], b = (size_t)g.v[e];
        worst = std::max(worst, inv[a * n + a] + inv[b * n + b] - 2.0 * inv[a * n + b]);
    }
    // chi_1: the second smallest eigenvalue (the smallest is the 0 of the constant vector)
    std::vector<double> eig;
    if (!symmetric_eigenvalues(n, lap, eig)) return fail(A2CID_EGRAPH, "eigenvalue iteration did not converge");
    std::sort(eig.begin(), eig.end());
    const double smallest = eig[1], top = eig[n - 1];
    if (!(smallest > 1e-13 * top)) return fail(A2CID_EGRAPH, "Laplacian has a second (near-)zero eigenvalue");
    const double c1 = 1.0 / smallest;
    const double c2 = 0.5 * worst;
    if (chi1) *chi1 = c1;
    if (chi2) *chi2 = c2;
    if (eta) *eta = 0.5 / std::sqrt(c1 * c2);
    if (alpha_tilde) *alpha_tilde = 0.5 * std::sqrt(c1 / c2);
    return A2CID_OK;
}

int a2cid_plan_batch_clocks(int32_t n, const a2cid_graph *graph, double eta, double *t, double *rate,
                            const a2cid_event_batch *batch, a2cid_coef *coef) {
    clear_error();
    if (!t) return fail(A2CID_EINVAL, "t is NULL");
    if (!(eta >= 0.0) || !std::isfinite(eta)) return fail(A2CID_EINVAL, "eta = %g must be finite and >= 0", eta);
    if (rate)
        for (int32_t i = 0; i < n; ++i)
            if (!(rate[i] > 0.0) || !std::isfinite(rate[i])) return fail(A2CID_EINVAL, "rate[%d] must be finite and > 0", i);
    try {
        Graph g;
        if (int rc = load_graph(g, n, graph)) return rc;
        Plan plan;
        PlanScratch scratch;
        if (int rc = plan_batch(g, eta, t, rate, batch, plan, scratch)) return rc;
        if (coef && batch->n_ops > 0) std::memcpy(coef, plan.coef.data(), sizeof(a2cid_coef) * (size_t)batch->n_ops);
        std::copy(plan.t_after.begin(), plan.t_after.end(), t);
        if (rate) std::copy(plan.rate_after.begin(), plan.rate_after.end(), rate);
    } catch (const std::bad_alloc &) {
        return fail(A2CID_ENOMEM, "out of host memory");
    }
    return A2CID_OK;
}

int a2cid_plan_batch(int32_t n, const a2cid_graph *graph, double eta, double *t,
                     const a2cid_event_batch *batch, a2cid_coef *coef) {
    return a2cid_plan_batch_clocks(n, graph, eta, t, nullptr, batch, coef);
}

int a2cid_plan_chain(int32_t n, const a2cid_event_batch *batch, int32_t lds_slots, a2cid_chain_step *steps,
                     int64_t capacity, int64_t *n_steps, double *bytes_per_column) {
    clear_error();
    if (n < 1 || n > A2CID_MAX_WORKERS) return fail(A2CID_EINVAL, "n = %d out of range", n);
    if (lds_slots < 0 || lds_slots > kChainMaxSlots) return fail(A2CID_EINVAL, "lds_slots must be in [0, %d]", kChainMaxSlots);
    if (!batch || batch->n_ops < 0 || (batch->n_ops > 0 && !batch->ops)) return fail(A2CID_EINVAL, "batch is NULL or malformed");
    if (batch->n_ops > INT32_MAX / 4) return fail(A2CID_EINVAL, "too many operations");
    if (!n_steps) return fail(A2CID_EINVAL, "n_steps is NULL");
    for (int64_t k = 0; k < batch->n_ops; ++k) {
        const a2cid_op &o = batch->ops[k];
        const bool gossip = o.kind == A2CID_KIND_GOSSIP;
        if ((!gossip && o.kind != A2CID_KIND_GRADIENT) || o.i < 0 || o.i >= n || (gossip && (o.j < 0 || o.j >= n || o.j == o.i)))
            return fail(A2CID_EINVAL, "op %lld: bad kind or worker index", (long long)k);
    }
    try {
        ChainPlan plan;
        plan_chain(n, batch->ops, batch->n_ops, lds_slots, plan);
        *n_steps = (int64_t)plan.steps.size();
        if (bytes_per_column) *bytes_per_column = plan.bytes_per_column;
        if (steps) {
            if ((int64_t)plan.steps.size() > capacity)
                return fail(A2CID_EINVAL, "%zu steps do not fit into %lld entries", plan.steps.size(), (long long)capacity);
            std::copy(plan.steps.begin(), plan.steps.end(), steps);
        }
    } catch (const std::bad_alloc &) {
        return fail(A2CID_ENOMEM, "out of host memory");
    }
    return A2CID_OK;
}

int a2cid_plan_resident(int32_t n, const a2cid_event_batch *batch, const a2cid_coef *coef, int32_t *waves, int32_t *cols,
                        int64_t first_op, a2cid_resident_slot *slots, int32_t *rows, int32_t *n_rows,
                        int64_t *gradient_ops, int32_t *n_gradient_ops, int64_t *next_op) {
    clear_error();
    if (n < 1 || n > A2CID_MAX_WORKERS) return fail(A2CID_EINVAL, "n = %d out of range", n);
    if (!batch || batch->n_ops < 0 || (batch->n_ops > 0 && (!batch->ops || !batch->level_off)) || batch->n_levels < 0)
        return fail(A2CID_EINVAL, "batch is NULL or malformed");
    if (!coef || !waves || !cols || !slots || !rows || !n_rows || !gradient_ops || !n_gradient_ops || !next_op)
        return fail(A2CID_EINVAL, "an output or coef is NULL");
    if (first_op < 0 || first_op > batch->n_ops) return fail(A2CID_EINVAL, "first_op out of range");
    for (int64_t k = 0; k < batch->n_ops; ++k) {
        const a2cid_op &o = batch->ops[k];
        const bool gossip = o.kind == A2CID_KIND_GOSSIP;
        if ((!gossip && o.kind != A2CID_KIND_GRADIENT) || o.i < 0 || o.i >= n || (gossip && (o.j < 0 || o.j >= n || o.j == o.i)))
            return fail(A2CID_EINVAL, "op %lld: bad kind or worker index", (long long)k);
    }
    int64_t at = 0;
    for (int32_t l = 0; l < batch->n_levels; ++l) {
        if (batch->level_off[l] != at || batch->level_off[l + 1] < at) return fail(A2CID_EMATCHING, "level table is not ascending");
        at = batch->level_off[l + 1];
    }
    if (at != batch->n_ops) return fail(A2CID_EMATCHING, "level table does not cover the operations");
    int w = *waves, c = *cols;
    if (w == 0) resident_shape(n, batch, &w, &c);
    if (w != 1 && w != 2 && w != 4 && w != 8 && w != 16) return fail(A2CID_EINVAL, "waves must be 0, 1, 2, 4, 8 or 16");
    if (c != 1 && c != 2 && c != 4) return fail(A2CID_EINVAL, "cols must be 1, 2 or 4");
    try {
        bool trailing = false;
        for (int64_t k = 0; k < batch->n_ops && !trailing; ++k) trailing = coef[k].b_post_i != 0.f || coef[k].b_post_j != 0.f;
        int32_t l = 0;
        while (l < batch->n_levels && batch->level_off[l + 1] <= first_op) ++l;
        int64_t k = first_op;
        ResidentPlan plan;
        plan_resident(n, batch, coef, w, c, trailing, &l, &k, plan);
        const size_t per_wave = (size_t)resident_slots(w);
        for (int q = 0; q < w; ++q)
            std::memcpy(slots + (size_t)q * per_wave, plan.programme[(size_t)q].data(), per_wave * sizeof(ResSlot));
        std::copy(plan.rows.begin(), plan.rows.end(), rows);
        *n_rows = (int32_t)plan.rows.size();
        std::copy(plan.grad_op.begin(), plan.grad_op.end(), gradient_ops);
        *n_gradient_ops = (int32_t)plan.grad_op.size();
        *next_op = k;
        *waves = w;
        *cols = c;
    } catch (const std::bad_alloc &) {
        return fail(A2CID_ENOMEM, "out of host memory");
    }
    return A2CID_OK;
}

int a2cid_plan_registers(int32_t n, const a2cid_event_batch *batch, const a2cid_coef *coef, int64_t first_op,
                         int64_t max_slots, int32_t full, const float *zero_one, a2cid_resident_slot *slots,
                         int64_t *n_slots, int64_t *gradient_ops, int32_t *n_gradient_ops, uint64_t *touched,
                         int64_t *next_op) {
    clear_error();
    if (n < 1 || n > kRegMaxRows) return fail(A2CID_EINVAL, "n = %d out of range (1 ... %d)", n, kRegMaxRows);
    if (!batch || batch->n_ops < 0 || (batch->n_ops > 0 && !batch->ops))
        return fail(A2CID_EINVAL, "batch is NULL or malformed");
    if (!coef || !slots || !n_slots || !gradient_ops || !n_gradient_ops || !touched || !next_op)
        return fail(A2CID_EINVAL, "an output or coef is NULL");
    if (first_op < 0 || first_op > batch->n_ops) return fail(A2CID_EINVAL, "first_op out of range");
    const int64_t least = (full ? 5 : 3) * kRegBlock;       // the two first requests and a block for the end slot
    if (max_slots < least + kRegBlock || max_slots % kRegBlock)
        return fail(A2CID_EINVAL, "max_slots must be a multiple of %d and at least %lld", kRegBlock,
                    (long long)(least + kRegBlock));
    if (((uintptr_t)zero_one & 3) != 0) return fail(A2CID_EINVAL, "zero_one must be 4-byte aligned");
    bool needs_full = false;
    for (int64_t k = 0; k < batch->n_ops; ++k) {
        const a2cid_op &o = batch->ops[k];
        const bool gossip = o.kind == A2CID_KIND_GOSSIP;
        if ((!gossip && o.kind != A2CID_KIND_GRADIENT) || o.i < 0 || o.i >= n || (gossip && (o.j < 0 || o.j >= n || o.j == o.i)))
            return fail(A2CID_EINVAL, "op %lld: bad kind or worker index", (long long)k);
        if (!gossip && o.gscale != 0.f && (o.c || o.h)) needs_full = true;
        if (!gossip && ((((uintptr_t)o.xi | (uintptr_t)o.c | (uintptr_t)o.h) & 3) != 0))
            return fail(A2CID_EINVAL, "op %lld: gradient inputs must be 4-byte aligned", (long long)k);
    }
    if (needs_full && !full) return fail(A2CID_EINVAL, "the batch has centres or curvatures: full must be set");
    try {
        RegPlan plan;
        int64_t k = first_op;
        plan_regfile(n, batch, coef, max_slots, full != 0, (uintptr_t)zero_one, &k, plan);
        if (!regfile_programme_ok(plan.programme, n, full != 0))
            return fail(A2CID_EINVAL, "internal: the register-file programme fails its own check");
        std::memcpy(slots, plan.programme.data(), plan.programme.size() * sizeof(ResSlot));
        *n_slots = (int64_t)plan.programme.size();
        std::copy(plan.grad_op.begin(), plan.grad_op.end(), gradient_ops);
        *n_gradient_ops = (int32_t)plan.grad_op.size();
        *touched = plan.touched;
        *next_op = k;
    } catch (const std::bad_alloc &) {
        return fail(A2CID_ENOMEM, "out of host memory");
    }
    return A2CID_OK;
}

int a2cid_check_registers(int32_t n, int32_t full, const a2cid_resident_slot *slots, int64_t n_slots) {
    clear_error();
    if (!slots || n_slots < 0) return fail(A2CID_EINVAL, "slots is NULL or n_slots negative");
    try {
        std::vector<ResSlot> prog((size_t)n_slots);
        std::memcpy(prog.data(), slots, (size_t)n_slots * sizeof(ResSlot));
        if (!regfile_programme_ok(prog, n, full != 0))
            return fail(A2CID_EINVAL, "not a programme the register-file kernel may run");
    } catch (const std::bad_alloc &) {
        return fail(A2CID_ENOMEM, "out of host memory");
    }
    return A2CID_OK;
}

int a2cid_sched_create(a2cid_sched **out, int32_t n, const a2cid_graph *graph,
                       const double *node_rate, uint64_t seed) {
    clear_error();
    if (!out || !node_rate) return fail(A2CID_EINVAL, "out / node_rate is NULL");
    *out = nullptr;
    a2cid_sched *s = new (std::nothrow) a2cid_sched;
    if (!s) return fail(A2CID_ENOMEM, "out of host memory");
    try {
        if (int rc = load_graph(s->g, n, graph)) { delete s; return rc; }
        const int32_t clocks = n + (int32_t)s->g.u.size();
        s->rate.resize(clocks);
        for (int32_t i = 0; i < n; ++i) {
            if (!(node_rate[i] >= 0.0) || !std::isfinite(node_rate[i])) {
                delete s;
                return fail(A2CID_EINVAL, "node_rate[%d] = %g must be finite and >= 0", i, node_rate[i]);
            }
            s->rate[i] = node_rate[i];
        }
        for (size_t e = 0; e < s->g.u.size(); ++e) s->rate[n + e] = s->g.rate[e];
        s->draws.assign(clocks, 0);
        s->fired.assign(clocks, 0);
        s->seed = seed;
        s->last_level.assign(n, -1);
        for (int32_t c = 0; c < clocks; ++c)
            if (s->rate[c] > 0.0) s->heap.emplace(s->waiting_time(c), c);
    } catch (const std::bad_alloc &) {
        delete s;
        return fail(A2CID_ENOMEM, "out of host memory");
    }
    *out = s;
    return A2CID_OK;
}

int a2cid_sched_create_fifo(a2cid_sched **out, int32_t n, const a2cid_graph *graph, const double *node_rate,
                           double comm_per_grad, double comm_time, double jitter, int32_t normalize, uint64_t seed) {
    clear_error();
    if (!out || !node_rate) return fail(A2CID_EINVAL, "out / node_rate is NULL");
    *out = nullptr;
    if (!(comm_per_grad >= 0.0) || !std::isfinite(comm_per_grad) || comm_per_grad > 700.0)
        return fail(A2CID_EINVAL, "comm_per_grad = %g must be in [0, 700]", comm_per_grad);
    if (!(comm_time >= 0.0) || !std::isfinite(comm_time)) return fail(A2CID_EINVAL, "comm_time = %g must be >= 0", comm_time);
    if (!(jitter >= 0.0) || jitter >= 1.0) return fail(A2CID_EINVAL, "jitter = %g must be in [0, 1)", jitter);
    if (normalize < 0 || normalize > 2) return fail(A2CID_EINVAL, "normalize must be 0, 1 or 2");
    a2cid_sched *s = new (std::nothrow) a2cid_sched;
    if (!s) return fail(A2CID_ENOMEM, "out of host memory");
    try {
        if (int rc = load_graph(s->g, n, graph)) { delete s; return rc; }
        const int32_t clocks = n + (int32_t)s->g.u.size();
        s->fifo = true;
        s->comm_per_grad = comm_per_grad; s->comm_time = comm_time; s->jitter = jitter;
        s->rate.assign(clocks, 0.0);
        for (int32_t i = 0; i < n; ++i) {
            if (!(node_rate[i] >= 0.0) || !std::isfinite(node_rate[i])) {
                delete s;
                return fail(A2CID_EINVAL, "node_rate[%d] = %g must be finite and >= 0", i, node_rate[i]);
            }
            s->rate[i] = node_rate[i];
        }
        s->draws.assign(clocks, 0);
        s->fired.assign(clocks, 0);
        s->count_draws.assign(n, 0);
        s->todo.assign(n, 0);
        s->busy.assign(n, 0);
        s->queued.assign(n, 0);
        s->seed = seed;
        s->last_level.assign(n, -1);
        s->edge_of.assign((size_t)n * n, -1);
        for (size_t e = 0; e < s->g.u.size(); ++e) {
            s->edge_of[(size_t)s->g.u[e] * n + s->g.v[e]] = (int32_t)e;
            s->edge_of[(size_t)s->g.v[e] * n + s->g.u[e]] = (int32_t)e;
        }
        s->normalize = normalize == 1;
        s->per_worker = normalize == 2;
        s->own_sum.assign(n, 0.0);
        s->own_n.assign(n, 0);
        s->running.assign(n, 0.0);
        double nominal = 0.0;
        int32_t active = 0;
        for (int32_t i = 0; i < n; ++i) {
            if (!(s->rate[i] > 0.0)) continue;
            s->running[i] = s->step_time(i);
            s->completions.emplace(s->running[i], 1, i);
            nominal += 1.0 / s->rate[i];
            ++active;
        }
        s->unit = active > 0 ? nominal / (double)active : 1.0;
    } catch (const std::bad_alloc &) {
        delete s;
        return fail(A2CID_ENOMEM, "out of host memory");
    }
    *out = s;
    return A2CID_OK;
}

int a2cid_sched_next(a2cid_sched *s, int64_t max_events, a2cid_event_batch *out) {
    clear_error();
    if (!s || !out) return fail(A2CID_EINVAL, "scheduler / out is NULL");
    if (max_events < 0) return fail(A2CID_EINVAL, "max_events is negative");
    try {
        s->raw.clear();
        s->level_of.clear();
        std::fill(s->last_level.begin(), s->last_level.end(), -1);
        int32_t n_levels = 0;
        a2cid_op op;
        while ((int64_t)s->raw.size() < max_events && s->pop(op)) {
            int32_t lev = s->last_level[op.i];
            if (op.kind == A2CID_KIND_GOSSIP) lev = std::max(lev, s->last_level[op.j]);
            ++lev;
            s->last_level[op.i] = lev;
            if (op.kind == A2CID_KIND_GOSSIP) s->last_level[op.j] = lev;
            n_levels = std::max(n_levels, lev + 1);
            s->raw.push_back(op);
            s->level_of.push_back(lev);
        }
        // stable counting sort by level: serial order survives inside each level
        s->level_off.assign((size_t)n_levels + 1, 0);
        for (int32_t lev : s->level_of) ++s->level_off[(size_t)lev + 1];
        for (int32_t l = 0; l < n_levels; ++l) s->level_off[(size_t)l + 1] += s->level_off[l];
        s->cursor.assign(s->level_off.begin(), s->level_off.end() - (n_levels > 0 ? 1 : 0));
        s->ops.resize(s->raw.size());
        for (size_t k = 0; k < s->raw.size(); ++k) s->ops[(size_t)s->cursor[s->level_of[k]]++] = s->raw[k];
        out->n_ops = (int64_t)s->ops.size();
        out->ops = s->ops.data();
        out->n_levels = n_levels;
        out->level_off = s->level_off.data();
        out->t_sync = std::numeric_limits<double>::quiet_NaN();
    } catch (const std::bad_alloc &) {
        return fail(A2CID_ENOMEM, "out of host memory");
    }
    return A2CID_OK;
}

int a2cid_sched_skip(a2cid_sched *s, int64_t n_events) {
    clear_error();
    if (!s || n_events < 0) return fail(A2CID_EINVAL, "scheduler is NULL or n_events negative");
    a2cid_op op;
    for (int64_t k = 0; k < n_events; ++k)
        if (!s->pop(op)) break;
    return A2CID_OK;
}

int a2cid_sched_counts(const a2cid_sched *s, int64_t *counts) {
    clear_error();
    if (!s || !counts) return fail(A2CID_EINVAL, "scheduler / counts is NULL");
    std::copy(s->fired.begin(), s->fired.end(), counts);
    return A2CID_OK;
}

void a2cid_sched_destroy(a2cid_sched *s) { delete s; }

}  // extern "C"
