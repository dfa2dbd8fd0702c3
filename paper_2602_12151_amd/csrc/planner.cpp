// Host-side planners of the serving method (no GPU code): the greedy switch plan of the appendix
// "Greedy Algorithm for Ad Hoc Model Switching" (section 5.2), and the lower-level workload
// assignment of section 4.2 (flow network with normalised replica capacities, constraints C1-C3).
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <numeric>
#include <vector>

#include "oserve.h"

namespace {

// Dense simplex for: maximise c.x subject to A x <= b, x >= 0, with b >= 0 (so the slack basis is
// feasible).  Bland's rule (smallest index enters, smallest index leaves among ties): no cycling.
// The instances here are tiny (replicas x workload types variables).
struct Simplex {
    int m, n;                          // constraints, structural variables
    std::vector<double> t;             // (m + 1) x (n + m + 1) tableau, last row = objective
    std::vector<int> basis;
    Simplex(int m_, int n_) : m(m_), n(n_), t(static_cast<size_t>(m_ + 1) * (n_ + m_ + 1), 0.0), basis(m_) {
        for (int i = 0; i < m; ++i) { at(i, n + i) = 1.0; basis[i] = n + i; }
    }
    double& at(int r, int c) { return t[static_cast<size_t>(r) * (n + m + 1) + c]; }
    bool solve() {
        const int cols = n + m;
        const double eps = 1e-11;
        for (int64_t iter = 0; iter < 1000000; ++iter) {
            int enter = -1;
            for (int c = 0; c < cols; ++c)
                if (at(m, c) < -eps) { enter = c; break; }
            if (enter < 0) return true;
            int leave = -1;
            double best = 0.0;
            for (int r = 0; r < m; ++r) {
                const double a = at(r, enter);
                if (a > eps) {
                    const double ratio = at(r, cols) / a;
                    if (leave < 0 || ratio < best - eps || (ratio < best + eps && basis[r] < basis[leave])) {
                        leave = r;
                        best = ratio;
                    }
                }
            }
            if (leave < 0) return false;   // unbounded: cannot happen with C1
            const double piv = at(leave, enter);
            for (int c = 0; c <= cols; ++c) at(leave, c) /= piv;
            for (int r = 0; r <= m; ++r) {
                if (r == leave) continue;
                const double f = at(r, enter);
                if (f == 0.0) continue;
                for (int c = 0; c <= cols; ++c) at(r, c) -= f * at(leave, c);
            }
            basis[leave] = enter;
        }
        return false;
    }
};

}  // namespace

extern "C" {

oserve_status_t oserve_switch_plan(int32_t num_devices, const int32_t* device_machine, int32_t num_shards,
                                   const int32_t* source_offsets, const int32_t* source_devices,
                                   const int32_t* target_offsets, const int32_t* target_devices,
                                   const int64_t* volumes, int32_t* chosen_source, int64_t* pair_load) {
    if (!device_machine || !source_offsets || !source_devices || !target_offsets || !target_devices || !volumes ||
        !chosen_source)
        return OSERVE_ERR_NULL;
    if (num_devices < 1 || num_devices > 32768 || num_shards < 0) return OSERVE_ERR_SHAPE;
    // C[s][t]: volume already planned from source s to target t
    std::vector<int64_t> load(static_cast<size_t>(num_devices) * num_devices, 0);
    std::vector<char> holds(static_cast<size_t>(num_devices));
    for (int32_t m = 0; m < num_shards; ++m) {
        const int32_t s0 = source_offsets[m], s1 = source_offsets[m + 1];
        const int32_t t0 = target_offsets[m], t1 = target_offsets[m + 1];
        if (s0 > s1 || t0 > t1) return OSERVE_ERR_SHAPE;
        std::fill(holds.begin(), holds.end(), 0);
        for (int32_t i = s0; i < s1; ++i) {
            if (source_devices[i] < 0 || source_devices[i] >= num_devices) return OSERVE_ERR_SHAPE;
            holds[source_devices[i]] = 1;
        }
        for (int32_t i = t0; i < t1; ++i) {
            const int32_t t = target_devices[i];
            if (t < 0 || t >= num_devices || volumes[i] < 0) return OSERVE_ERR_SHAPE;
            if (holds[t]) { chosen_source[i] = -1; continue; }   // the target already holds the shard
            if (s0 == s1) return OSERVE_ERR_SHAPE;                 // nobody holds a shard that is needed
            // sources on the target's machine first; among the candidates the least-loaded pair,
            // the first listed among equals
            int32_t best = -1;
            bool best_intra = false;
            for (int32_t k = s0; k < s1; ++k) {
                const int32_t s = source_devices[k];
                const bool intra = device_machine[s] == device_machine[t];
                const int64_t c = load[static_cast<size_t>(s) * num_devices + t];
                if (best < 0 || (intra && !best_intra) ||
                    (intra == best_intra && c < load[static_cast<size_t>(best) * num_devices + t])) {
                    best = s;
                    best_intra = intra;
                }
            }
            load[static_cast<size_t>(best) * num_devices + t] += volumes[i];
            chosen_source[i] = best;
        }
    }
    if (pair_load) std::copy(load.begin(), load.end(), pair_load);
    return OSERVE_OK;
}

oserve_status_t oserve_capacity_normalise(const int64_t* per_type_capacity, int32_t num_types, int64_t* common,
                                          int64_t* units_per_request) {
    if (!per_type_capacity || !common || !units_per_request) return OSERVE_ERR_NULL;
    if (num_types < 1) return OSERVE_ERR_SHAPE;
    int64_t m = 1;
    for (int32_t j = 0; j < num_types; ++j) {
        const int64_t n = per_type_capacity[j];
        if (n < 0) return OSERVE_ERR_SHAPE;
        if (n == 0) continue;                       // the replica cannot serve this type
        const int64_t g = std::gcd(m, n);
        if (m / g > (INT64_MAX / 4) / n) return OSERVE_ERR_SHAPE;   // least common multiple overflows
        m = m / g * n;
    }
    *common = m;
    for (int32_t j = 0; j < num_types; ++j)
        units_per_request[j] = per_type_capacity[j] > 0 ? m / per_type_capacity[j] : 0;
    return OSERVE_OK;
}

oserve_status_t oserve_assign_workload(int32_t num_replicas, int32_t num_types, const double* arrivals,
                                       const int64_t* node_capacity, const double* edge_capacity,
                                       double* assignment, double* total) {
    if (!arrivals || !node_capacity || !assignment || !total) return OSERVE_ERR_NULL;
    if (num_replicas < 1 || num_types < 1 || static_cast<int64_t>(num_replicas) * num_types > 4096) return OSERVE_ERR_SHAPE;
    const int K = num_replicas, J = num_types;
    std::vector<int> var_of(static_cast<size_t>(K) * J, -1);
    int nv = 0, nc2 = 0;
    for (int k = 0; k < K; ++k)
        for (int j = 0; j < J; ++j) {
            const int64_t n = node_capacity[k * J + j];
            if (n < 0) return OSERVE_ERR_SHAPE;
            if (edge_capacity && !(edge_capacity[k * J + j] >= 0.0)) return OSERVE_ERR_SHAPE;
            if (n > 0) {
                var_of[k * J + j] = nv++;
                if (edge_capacity && std::isfinite(edge_capacity[k * J + j])) ++nc2;
            }
        }
    for (int j = 0; j < J; ++j)
        if (!(arrivals[j] >= 0.0) || !std::isfinite(arrivals[j])) return OSERVE_ERR_SHAPE;
    std::fill(assignment, assignment + static_cast<size_t>(K) * J, 0.0);
    *total = 0.0;
    if (nv == 0) return OSERVE_OK;
    Simplex lp(J + K + nc2, nv);
    const int rhs = nv + lp.m;
    int row = 0;
    for (int j = 0; j < J; ++j, ++row) {            // C1: sum_k x[k][j] <= arrivals[j]
        for (int k = 0; k < K; ++k)
            if (var_of[k * J + j] >= 0) lp.at(row, var_of[k * J + j]) = 1.0;
        lp.at(row, rhs) = arrivals[j];
    }
    for (int k = 0; k < K; ++k, ++row) {            // C3: sum_j x[k][j] * (M_k / n[k][j]) <= M_k, divided by M_k
        for (int j = 0; j < J; ++j)
            if (var_of[k * J + j] >= 0) lp.at(row, var_of[k * J + j]) = 1.0 / static_cast<double>(node_capacity[k * J + j]);
        lp.at(row, rhs) = 1.0;
    }
    for (int k = 0; k < K; ++k)                     // C2: x[k][j] <= e[k][j]
        for (int j = 0; j < J; ++j)
            if (var_of[k * J + j] >= 0 && edge_capacity && std::isfinite(edge_capacity[k * J + j])) {
                lp.at(row, var_of[k * J + j]) = 1.0;
                lp.at(row, rhs) = edge_capacity[k * J + j];
                ++row;
            }
    for (int v = 0; v < nv; ++v) lp.at(lp.m, v) = -1.0;   // maximise the number of requests served
    if (!lp.solve()) return OSERVE_ERR_DEVICE;
    for (int r = 0; r < lp.m; ++r)
        if (lp.basis[r] < nv) {
            const double val = std::max(0.0, lp.at(r, rhs));
            for (int i = 0; i < K * J; ++i)
                if (var_of[i] == lp.basis[r]) assignment[i] = val;
        }
    double sum = 0.0;
    for (int i = 0; i < K * J; ++i) sum += assignment[i];
    *total = sum;
    return OSERVE_OK;
}

}  // extern "C"
