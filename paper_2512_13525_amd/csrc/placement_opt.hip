// Replica management on the host (Janus Appendix B, "Activation-Aware Replica Placement"): the
// window statistics c(e) and a(e, e'), the replica-count rule, and the greedy placement of Alg. 3
// that spreads experts that are activated together over different instances (objective: the
// largest co-activation load I(g) of Eq. 6).  Runs when the layout is rebuilt (minutes apart,
// Sec. 3.4), never on the per-layer path, so it is plain sequential C++ on host arrays; its
// output feeds moe_placement_create.
//
// Choices the appendix leaves open: an expert gets at most one replica per instance, so at most
// n_inst replicas; ties go to the lower expert id / lower instance / earlier position; the penalty
// of a swap is the change of the summed co-activation load.  Sums are fp64 in placement order.
#include <algorithm>
#include <vector>

#include "common.h"

extern "C" int moe_coactivation_counts(const int32_t *ids_host, int n_batches, int batch_pairs, int E,
                                       double *c_host_out, double *a_host_out) {
    if (E < 1 || n_batches < 0 || batch_pairs < 0) return MOE_EINVAL;
    if (!c_host_out || !a_host_out || (static_cast<long long>(n_batches) * batch_pairs > 0 && !ids_host)) return MOE_EINVAL;
    std::fill(c_host_out, c_host_out + E, 0.0);
    std::fill(a_host_out, a_host_out + static_cast<size_t>(E) * E, 0.0);
    std::vector<char> seen(E);
    std::vector<int> act;
    for (int b = 0; b < n_batches; ++b) {
        std::fill(seen.begin(), seen.end(), 0);
        act.clear();
        const int32_t *row = ids_host + static_cast<size_t>(b) * batch_pairs;
        for (int p = 0; p < batch_pairs; ++p) {
            const int e = row[p];
            if (e < 0 || e >= E) return MOE_EINVAL;
            if (!seen[e]) { seen[e] = 1; act.push_back(e); }
        }
        for (size_t i = 0; i < act.size(); ++i) {
            c_host_out[act[i]] += 1.0;
            for (size_t j = i + 1; j < act.size(); ++j) {
                a_host_out[static_cast<size_t>(act[i]) * E + act[j]] += 1.0;
                a_host_out[static_cast<size_t>(act[j]) * E + act[i]] += 1.0;
            }
        }
    }
    return MOE_OK;
}

extern "C" int moe_replica_counts(int E, int n_inst, int C, const double *c_host, int32_t *R_host_out) {
    if (E < 1 || n_inst < 1 || C < 1 || !c_host || !R_host_out) return MOE_EINVAL;
    const long long S = static_cast<long long>(n_inst) * C;
    if (S < E) return MOE_EPLACEMENT;
    for (int e = 0; e < E; ++e) R_host_out[e] = 1;
    for (long long s = E; s < S; ++s) {
        int best = -1;
        for (int e = 0; e < E; ++e) {
            if (R_host_out[e] >= n_inst) continue;
            if (best < 0 || c_host[e] / R_host_out[e] > c_host[best] / R_host_out[best]) best = e;
        }
        if (best < 0) break;                           // every expert is on every instance
        R_host_out[best] += 1;
    }
    return MOE_OK;
}

namespace {

// sum of a(e, m) over the members of an instance in placement order, optionally leaving one out
double penalty(const double *a, int E, int e, const std::vector<int> &members, int skip = -1) {
    double s = 0.0;
    for (size_t pos = 0; pos < members.size(); ++pos)
        if (static_cast<int>(pos) != skip) s += a[static_cast<size_t>(e) * E + members[pos]];
    return s;
}

}  // namespace

extern "C" int moe_place_replicas(int E, int n_inst, int C, const int32_t *R_host, const double *c_host,
                                  const double *a_host, int32_t *slot_to_expert_host_out) {
    if (E < 1 || n_inst < 1 || C < 1 || !R_host || !c_host || !a_host || !slot_to_expert_host_out) return MOE_EINVAL;
    long long total = 0;
    for (int e = 0; e < E; ++e) {
        if (R_host[e] < 1 || R_host[e] > n_inst) return MOE_EPLACEMENT;
        total += R_host[e];
    }
    if (total > static_cast<long long>(n_inst) * C) return MOE_EPLACEMENT;

    struct Replica { int e, r; double load; };
    std::vector<Replica> order;
    order.reserve(static_cast<size_t>(total));
    for (int e = 0; e < E; ++e)
        for (int r = 0; r < R_host[e]; ++r) order.push_back({e, r, c_host[e] / R_host[e]});
    std::stable_sort(order.begin(), order.end(), [](const Replica &x, const Replica &y) {
        if (x.load != y.load) return x.load > y.load;
        if (x.e != y.e) return x.e < y.e;
        return x.r < y.r;
    });

    std::vector<std::vector<int>> P(n_inst);
    std::vector<int> slots(n_inst, C);
    std::vector<char> x(static_cast<size_t>(E) * n_inst, 0);
    auto hosts = [&](int e, int g) -> char & { return x[static_cast<size_t>(e) * n_inst + g]; };

    for (const Replica &rep : order) {
        const int e = rep.e;
        int best_g = -1;
        double best_p = 0.0;
        for (int g = 0; g < n_inst; ++g) {
            if (slots[g] <= 0 || hosts(e, g)) continue;
            const double p = penalty(a_host, E, e, P[g]);
            if (best_g < 0 || p < best_p) { best_g = g; best_p = p; }
        }
        if (best_g >= 0) {
            P[best_g].push_back(e);
            slots[best_g] -= 1;
            hosts(e, best_g) = 1;
            continue;
        }
        // no instance with room is free of e: put e in the place of some j on an instance g without e
        // and move j to an instance h with room that does not host j
        bool found = false;
        double best_d = 0.0;
        int sg = -1, spos = -1, sh = -1;
        for (int g = 0; g < n_inst; ++g) {
            if (hosts(e, g)) continue;
            for (int pos = 0; pos < static_cast<int>(P[g].size()); ++pos) {
                const int ej = P[g][pos];
                for (int h = 0; h < n_inst; ++h) {
                    if (slots[h] <= 0 || hosts(ej, h) || h == g) continue;
                    const double d = (penalty(a_host, E, e, P[g], pos) - penalty(a_host, E, ej, P[g], pos)) +
                                     penalty(a_host, E, ej, P[h]);
                    if (!found || d < best_d) { found = true; best_d = d; sg = g; spos = pos; sh = h; }
                }
            }
        }
        if (!found) return MOE_EPLACEMENT;
        const int ej = P[sg][spos];
        P[sg][spos] = e;
        P[sh].push_back(ej);
        slots[sh] -= 1;
        hosts(ej, sg) = 0;
        hosts(ej, sh) = 1;
        hosts(e, sg) = 1;
    }
    for (int g = 0; g < n_inst; ++g)
        for (int s = 0; s < C; ++s)
            slot_to_expert_host_out[static_cast<size_t>(g) * C + s] = s < static_cast<int>(P[g].size()) ? P[g][s] : -1;
    return MOE_OK;
}
