// SLO-aware resource scaling on the host (Janus Sec. 3.5, "Fine-Grained Scaling under SLOs"):
// the layer-wise latency model of Eq. 1a-1c, the steady-state batch of Eq. 2 (Little's law)
// found by bisection of the residual, and the enumeration of Alg. 2 over (n_a, n_e).  The MoE
// term is beta * a_max(n_e, B) + c_e with a_max from a caller-supplied table (the Monte-Carlo
// estimate over sampled batches) and beta, c_e from profiling the layer step.  Plain sequential
// C++ on host data: it runs when demand changes, never on the per-layer path.
#include "common.h"

namespace {

struct Table {
    const double *v;
    const int *ne;
    int n_ne;
    const double *B;
    int n_B;
};

bool lookup(const Table &t, int n_e, double B, double *out) {
    int r = -1;
    for (int i = 0; i < t.n_ne; ++i)
        if (t.ne[i] == n_e) { r = i; break; }
    if (r < 0) return false;
    const double *row = t.v + static_cast<size_t>(r) * t.n_B;
    if (B <= t.B[0]) { *out = row[0]; return true; }
    if (B >= t.B[t.n_B - 1]) { *out = row[t.n_B - 1]; return true; }
    for (int i = 0; i + 1 < t.n_B; ++i) {
        if (t.B[i] <= B && B <= t.B[i + 1]) {
            const double f = (B - t.B[i]) / (t.B[i + 1] - t.B[i]);
            *out = row[i] + f * (row[i + 1] - row[i]);
            return true;
        }
    }
    return false;
}

double tpot(const moe_scaling_model &m, double a_max, double B, int n_a) {
    const double b = B / n_a;
    const double lin = m.alpha * b + m.c_kv * b * m.S_ctx;
    const double t_attn = m.c_a > lin ? m.c_a : lin;
    const double t_moe = m.beta * a_max + m.c_e;
    const double t_comm = m.comm0 + m.comm1 * B;
    return m.L * (t_attn + t_moe + t_comm);
}

}  // namespace

extern "C" int moe_scaling_solve(const moe_scaling_model *m, const double *amax_table_host, const int *ne_values_host,
                                 int n_ne, const double *B_values_host, int n_B, double lambda, double slo,
                                 int n_max, int ne_min, double B_max, int *n_a_out, int *n_e_out, double *B_star_out,
                                 double *tpot_out) {
    if (!m || !amax_table_host || !ne_values_host || !B_values_host || !n_a_out || !n_e_out || !B_star_out || !tpot_out)
        return MOE_EINVAL;
    if (n_ne < 1 || n_B < 1 || n_max < 1 || ne_min < 1 || m->L < 1 || !(B_max >= 1.0) || !(lambda > 0.0)) return MOE_EINVAL;
    for (int i = 0; i + 1 < n_B; ++i)
        if (!(B_values_host[i] < B_values_host[i + 1])) return MOE_EINVAL;
    const Table t{amax_table_host, ne_values_host, n_ne, B_values_host, n_B};
    bool found = false;
    int best = 0;
    for (int n_a = 1; n_a <= n_max; ++n_a) {
        for (int n_e = ne_min; n_e <= n_max; ++n_e) {
            double a = 0.0;
            if (!lookup(t, n_e, 1.0, &a)) continue;                        // n_e is not on the grid
            auto f = [&](double B) {
                double am = 0.0;
                lookup(t, n_e, B, &am);
                return B - lambda * tpot(*m, am, B, n_a);
            };
            double Bs;
            if (f(1.0) >= 0.0) {
                Bs = 1.0;                                                  // too light to form a larger batch
            } else if (f(B_max) < 0.0) {
                continue;                                                  // cannot sustain the demand
            } else {
                double lo = 1.0, hi = B_max;
                for (int it = 0; it < 60; ++it) {
                    const double mid = 0.5 * (lo + hi);
                    if (f(mid) < 0.0) lo = mid; else hi = mid;
                }
                Bs = hi;
            }
            lookup(t, n_e, Bs, &a);
            const double T = tpot(*m, a, Bs, n_a);
            if (T > slo) continue;
            if (m->mem_fixed + m->mem_per_token * (Bs / n_a) * m->S_ctx > m->mem_budget) continue;
            if (!found || n_a + n_e < best) {
                found = true;
                best = n_a + n_e;
                *n_a_out = n_a; *n_e_out = n_e; *B_star_out = Bs; *tpot_out = T;
            }
        }
    }
    if (!found) { *n_a_out = 0; *n_e_out = 0; *B_star_out = 0.0; *tpot_out = 0.0; }
    return MOE_OK;
}
