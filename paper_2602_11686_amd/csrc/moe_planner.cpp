// Host-side load-balancing planner (paper section 4 and appendix): replica allocation,
// expert relocation, lite routing, the cost model and the layout search.  Plain C++,
// no device code: the paper runs this on the CPU while the GPU computes the layer.
//
// Floating point is kept to single IEEE double operations in a fixed order (no
// contraction), so that results are reproducible bit for bit.
#pragma STDC FP_CONTRACT OFF

#include <algorithm>
#include <climits>
#include <cstdint>
#include <queue>
#include <utility>
#include <vector>

#include "moe_planner.h"

namespace moe {
void set_error(const char* fmt, ...);
}
using moe::set_error;

namespace {

moe_status check_shape(const moe_plan_shape* s, const char* who) {
    if (!s) {
        set_error("%s: shape is NULL", who);
        return MOE_ERR_INVALID_ARG;
    }
    if (s->N < 1 || s->E < 1 || s->C < 1 || s->D < 1 || s->N % s->D != 0) {
        set_error("%s: N=%d E=%d C=%d D=%d: all must be >= 1 and D must divide N", who, s->N, s->E, s->C, s->D);
        return MOE_ERR_INVALID_ARG;
    }
    return MOE_OK;
}

#define MOE_RETURN_IF(expr)             \
    do {                                \
        moe_status _st = (expr);        \
        if (_st != MOE_OK) return _st;  \
    } while (0)

#define PLAN_NOT_NULL(p, who)                         \
    if (!(p)) {                                       \
        set_error("%s: %s is NULL", who, #p);         \
        return MOE_ERR_INVALID_ARG;                   \
    }

struct SplitMix64 {
    uint64_t state;
    uint64_t next() {
        state += 0x9E3779B97F4A7C15ull;
        uint64_t z = state;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
};

moe_status column_sums(const moe_plan_shape* s, const int64_t* R, std::vector<int64_t>& load, const char* who) {
    load.assign(s->E, 0);
    for (int i = 0; i < s->N; ++i)
        for (int j = 0; j < s->E; ++j) {
            const int64_t v = R[(size_t)i * s->E + j];
            if (v < 0) {
                set_error("%s: R[%d][%d] = %lld is negative", who, i, j, (long long)v);
                return MOE_ERR_INVALID_ARG;
            }
            load[j] += v;
        }
    return MOE_OK;
}

// Appendix, replica allocation: a max-heap on (load per replica, then lower index).
void replica_allocation(const moe_plan_shape* s, const std::vector<int64_t>& load, std::vector<int32_t>& rep) {
    struct Item {
        double avg;
        int32_t e;
        bool operator<(const Item& o) const { return avg < o.avg || (avg == o.avg && e > o.e); }
    };
    rep.assign(s->E, 1);
    std::priority_queue<Item> pq;
    for (int j = 0; j < s->E; ++j) pq.push({(double)load[j] / 1.0, j});
    for (int64_t total = s->E; total < (int64_t)s->N * s->C; ++total) {
        const Item top = pq.top();
        pq.pop();
        rep[top.e] += 1;
        pq.push({(double)load[top.e] / (double)rep[top.e], top.e});
    }
}

void evenly_replicas(const moe_plan_shape* s, std::vector<int32_t>& rep) {
    const int64_t slots = (int64_t)s->N * s->C;
    const int32_t base = (int32_t)(slots / s->E), rem = (int32_t)(slots % s->E);
    rep.resize(s->E);
    for (int j = 0; j < s->E; ++j) rep[j] = base + (j < rem ? 1 : 0);
}

// Alg. 1.  O(sum(rep) * N).
moe_status expert_relocation(const moe_plan_shape* s, const int32_t* rep, const int64_t* load, int32_t* A,
                             const char* who) {
    const int N = s->N, E = s->E, C = s->C, D = s->D, nodes = N / D;
    int64_t total = 0;
    for (int j = 0; j < E; ++j) {
        if (rep[j] < 1) {
            set_error("%s: expert_rep[%d] = %d, every expert needs a replica", who, j, rep[j]);
            return MOE_ERR_INVALID_ARG;
        }
        total += rep[j];
    }
    if (total > (int64_t)N * C) {
        set_error("%s: %lld replicas do not fit N*C = %lld slots", who, (long long)total, (long long)N * C);
        return MOE_ERR_INVALID_ARG;
    }
    std::vector<std::pair<int32_t, double>> lst;
    lst.reserve((size_t)total);
    for (int j = 0; j < E; ++j) {
        const double avg = (double)load[j] / (double)rep[j];
        for (int r = 0; r < rep[j]; ++r) lst.emplace_back(j, avg);
    }
    std::stable_sort(lst.begin(), lst.end(), [](const auto& a, const auto& b) { return a.second > b.second; });
    std::vector<int32_t> expert_count(N, 0), node_cnt(nodes);
    std::vector<double> device_loads(N, 0.0);
    std::fill(A, A + (size_t)N * E, 0);
    for (const auto& item : lst) {
        const int e = item.first;
        // devices with a free slot; those that do not hold the expert yet are preferred
        bool any_fresh = false;
        for (int i = 0; i < N && !any_fresh; ++i) any_fresh = expert_count[i] < C && A[(size_t)i * E + e] == 0;
        std::fill(node_cnt.begin(), node_cnt.end(), 0);
        for (int i = 0; i < N; ++i) node_cnt[i / D] += A[(size_t)i * E + e];
        auto eligible = [&](int i) { return expert_count[i] < C && (!any_fresh || A[(size_t)i * E + e] == 0); };
        int fewest = INT_MAX;
        for (int i = 0; i < N; ++i)
            if (eligible(i) && node_cnt[i / D] < fewest) fewest = node_cnt[i / D];
        int device = -1;
        for (int i = 0; i < N; ++i)
            if (eligible(i) && node_cnt[i / D] == fewest && (device < 0 || device_loads[i] < device_loads[device]))
                device = i;
        A[(size_t)device * E + e] += 1;  // a free slot exists: total <= N*C
        device_loads[device] += item.second;
        expert_count[device] += 1;
    }
    return MOE_OK;
}

// The replicas of every expert in ascending device order (a device with m replicas m times),
// and where each node's replicas start in that list: what the lite routing walks.
struct ReplicaLists {
    std::vector<int32_t> dev;    // concatenated lists
    std::vector<int64_t> begin;  // [E+1]
    std::vector<int64_t> node_begin;  // [E][nodes+1] offsets into dev, relative to begin[j]
    void build(const moe_plan_shape* s, const int32_t* A) {
        const int N = s->N, E = s->E, D = s->D, nodes = N / D;
        begin.assign(E + 1, 0);
        for (int j = 0; j < E; ++j) {
            int64_t c = 0;
            for (int i = 0; i < N; ++i) c += A[(size_t)i * E + j];
            begin[j + 1] = begin[j] + c;
        }
        dev.resize((size_t)begin[E]);
        node_begin.assign((size_t)E * (nodes + 1), 0);
        for (int j = 0; j < E; ++j) {
            int64_t p = begin[j];
            for (int i = 0; i < N; ++i) {
                if (i % D == 0) node_begin[(size_t)j * (nodes + 1) + i / D] = p - begin[j];
                for (int m = 0; m < A[(size_t)i * E + j]; ++m) dev[(size_t)p++] = i;
            }
            node_begin[(size_t)j * (nodes + 1) + nodes] = p - begin[j];
        }
    }
};

// Lite routing of device i's tokens for expert j: calls f(k, share) once per destination device k in
// ascending order with the tokens it receives (shares of replicas on one device are added up first).
template <class F>
bool route_one(const moe_plan_shape* s, const ReplicaLists& rl, int i, int j, int64_t tokens, F&& f) {
    const int nodes = s->N / s->D, node = i / s->D;
    const int64_t* nb = &rl.node_begin[(size_t)j * (nodes + 1)];
    int64_t lo = nb[node], hi = nb[node + 1];
    if (lo == hi) { lo = 0; hi = rl.begin[j + 1] - rl.begin[j]; }  // no replica in the node: all replicas
    const int64_t len = hi - lo;
    if (len == 0) return tokens == 0;
    const int64_t base = tokens / len, rem = tokens % len;
    const int32_t* d = &rl.dev[(size_t)(rl.begin[j] + lo)];
    for (int64_t r = 0; r < len;) {
        const int k = d[r];
        int64_t share = 0;
        for (; r < len && d[r] == k; ++r) share += base + (r < rem ? 1 : 0);
        f(k, share);
    }
    return true;
}

// Cost of a layout under the lite routing, without materialising S.  Same operation order as the
// definition: sum over i, j, k ascending of S / bw, skipping i == k and zeros.
moe_status layout_cost(const moe_plan_shape* s, const moe_plan_cost* c, const int64_t* R, const int32_t* A, double* T,
                       const char* who) {
    ReplicaLists rl;
    rl.build(s, A);
    const int N = s->N, E = s->E, D = s->D;
    std::vector<int64_t> received(N, 0);
    double acc = 0.0;
    for (int i = 0; i < N; ++i)
        for (int j = 0; j < E; ++j) {
            const bool ok = route_one(s, rl, i, j, R[(size_t)i * E + j], [&](int k, int64_t share) {
                received[k] += share;
                if (k != i && share != 0) acc += (double)share / (i / D == k / D ? c->b_intra : c->b_inter);
            });
            if (!ok) {
                set_error("%s: expert %d has tokens on device %d but no replica", who, j, i);
                return MOE_ERR_INVALID_ARG;
            }
        }
    const double t_comm = 4.0 * c->v_comm * acc;
    double worst = 0.0;
    for (int i = 0; i < N; ++i) {
        const double t_i = (c->v_comp * (double)received[i]) / c->b_comp;
        if (t_i > worst) worst = t_i;
    }
    const double t_comp = (double)(3 + c->f_ckpt) * worst;
    T[0] = t_comm + t_comp;
    T[1] = t_comm;
    T[2] = t_comp;
    return MOE_OK;
}

}  // namespace

extern "C" moe_status moe_plan_replica_allocation(const moe_plan_shape* s, const int64_t* R, int32_t* expert_rep) {
    const char* who = "moe_plan_replica_allocation";
    MOE_RETURN_IF(check_shape(s, who));
    PLAN_NOT_NULL(R, who);
    PLAN_NOT_NULL(expert_rep, who);
    if ((int64_t)s->N * s->C < s->E) {
        set_error("%s: N*C = %lld slots cannot hold E = %d experts", who, (long long)s->N * s->C, s->E);
        return MOE_ERR_INVALID_ARG;
    }
    std::vector<int64_t> load;
    MOE_RETURN_IF(column_sums(s, R, load, who));
    std::vector<int32_t> rep;
    replica_allocation(s, load, rep);
    std::copy(rep.begin(), rep.end(), expert_rep);
    return MOE_OK;
}

extern "C" moe_status moe_plan_expert_relocation(const moe_plan_shape* s, const int32_t* expert_rep,
                                                 const int64_t* expert_loads, int32_t* A) {
    const char* who = "moe_plan_expert_relocation";
    MOE_RETURN_IF(check_shape(s, who));
    PLAN_NOT_NULL(expert_rep, who);
    PLAN_NOT_NULL(expert_loads, who);
    PLAN_NOT_NULL(A, who);
    return expert_relocation(s, expert_rep, expert_loads, A, who);
}

extern "C" moe_status moe_plan_lite_routing(const moe_plan_shape* s, const int64_t* R, const int32_t* A, int64_t* S) {
    const char* who = "moe_plan_lite_routing";
    MOE_RETURN_IF(check_shape(s, who));
    PLAN_NOT_NULL(R, who);
    PLAN_NOT_NULL(A, who);
    PLAN_NOT_NULL(S, who);
    const int N = s->N, E = s->E;
    ReplicaLists rl;
    rl.build(s, A);
    std::fill(S, S + (size_t)N * E * N, (int64_t)0);
    for (int i = 0; i < N; ++i)
        for (int j = 0; j < E; ++j) {
            const int64_t tokens = R[(size_t)i * E + j];
            if (tokens < 0) {
                set_error("%s: R[%d][%d] is negative", who, i, j);
                return MOE_ERR_INVALID_ARG;
            }
            int64_t* row = S + ((size_t)i * E + j) * N;
            if (!route_one(s, rl, i, j, tokens, [&](int k, int64_t share) { row[k] = share; })) {
                set_error("%s: expert %d has tokens on device %d but no replica", who, j, i);
                return MOE_ERR_INVALID_ARG;
            }
        }
    return MOE_OK;
}

extern "C" moe_status moe_plan_time_cost(const moe_plan_shape* s, const moe_plan_cost* c, const int64_t* S, double* T) {
    const char* who = "moe_plan_time_cost";
    MOE_RETURN_IF(check_shape(s, who));
    PLAN_NOT_NULL(c, who);
    PLAN_NOT_NULL(S, who);
    PLAN_NOT_NULL(T, who);
    const int N = s->N, E = s->E, D = s->D;
    double acc = 0.0;
    std::vector<int64_t> received(N, 0);
    for (int i = 0; i < N; ++i)
        for (int j = 0; j < E; ++j)
            for (int k = 0; k < N; ++k) {
                const int64_t v = S[((size_t)i * E + j) * N + k];
                received[k] += v;
                if (i == k || v == 0) continue;
                acc += (double)v / (i / D == k / D ? c->b_intra : c->b_inter);
            }
    const double t_comm = 4.0 * c->v_comm * acc;
    double worst = 0.0;
    for (int i = 0; i < N; ++i) {
        const double t_i = (c->v_comp * (double)received[i]) / c->b_comp;
        if (t_i > worst) worst = t_i;
    }
    const double t_comp = (double)(3 + c->f_ckpt) * worst;
    T[0] = t_comm + t_comp;
    T[1] = t_comm;
    T[2] = t_comp;
    return MOE_OK;
}

extern "C" moe_status moe_plan_expert_layout(const moe_plan_shape* s, const moe_plan_cost* c, const int64_t* R, int32_t eps,
                                             uint64_t seed, int32_t* A, double* T, int32_t* best_index,
                                             int32_t* replicas_set) {
    const char* who = "moe_plan_expert_layout";
    MOE_RETURN_IF(check_shape(s, who));
    PLAN_NOT_NULL(c, who);
    PLAN_NOT_NULL(R, who);
    PLAN_NOT_NULL(A, who);
    PLAN_NOT_NULL(T, who);
    PLAN_NOT_NULL(best_index, who);
    if (eps < 1) {
        set_error("%s: eps = %d, at least one candidate is needed", who, eps);
        return MOE_ERR_INVALID_ARG;
    }
    if ((int64_t)s->N * s->C < s->E) {
        set_error("%s: N*C = %lld slots cannot hold E = %d experts", who, (long long)s->N * s->C, s->E);
        return MOE_ERR_INVALID_ARG;
    }
    const int E = s->E;
    std::vector<int64_t> load;
    MOE_RETURN_IF(column_sums(s, R, load, who));
    std::vector<std::vector<int32_t>> set(1);
    replica_allocation(s, load, set[0]);
    if (eps >= 2) {
        set.emplace_back();
        evenly_replicas(s, set.back());
    }
    SplitMix64 rng{seed};
    while ((int)set.size() < eps) {
        std::vector<int32_t> rep = set[(size_t)(rng.next() % set.size())];
        std::vector<int32_t> donors;
        for (int j = 0; j < E; ++j)
            if (rep[j] > 1) donors.push_back(j);
        if (!donors.empty() && E >= 2) {
            const int d = donors[(size_t)(rng.next() % donors.size())];
            int r = (int)(rng.next() % (uint64_t)(E - 1));
            if (r >= d) r += 1;
            rep[d] -= 1;
            rep[r] += 1;
        }
        set.push_back(std::move(rep));
    }
    std::vector<int32_t> cand((size_t)s->N * E);
    double best = 0.0;
    int best_i = -1;
    for (int idx = 0; idx < (int)set.size(); ++idx) {
        MOE_RETURN_IF(expert_relocation(s, set[idx].data(), load.data(), cand.data(), who));
        double t[3];
        MOE_RETURN_IF(layout_cost(s, c, R, cand.data(), t, who));
        if (best_i < 0 || t[0] < best) {
            best = t[0];
            best_i = idx;
            std::copy(cand.begin(), cand.end(), A);
        }
        if (replicas_set) std::copy(set[idx].begin(), set[idx].end(), replicas_set + (size_t)idx * E);
    }
    *T = best;
    *best_index = best_i;
    return MOE_OK;
}

extern "C" moe_status moe_plan_dispatch_table(const moe_plan_shape* s, const int32_t* A, int32_t rank, int32_t* G_out,
                                              int32_t* n_rep_out, int32_t* expert_of_group, int32_t* device_of_group,
                                              int32_t* rep_begin, int32_t* rep_group) {
    const char* who = "moe_plan_dispatch_table";
    MOE_RETURN_IF(check_shape(s, who));
    PLAN_NOT_NULL(A, who);
    PLAN_NOT_NULL(G_out, who);
    PLAN_NOT_NULL(n_rep_out, who);
    PLAN_NOT_NULL(expert_of_group, who);
    PLAN_NOT_NULL(device_of_group, who);
    PLAN_NOT_NULL(rep_begin, who);
    PLAN_NOT_NULL(rep_group, who);
    const int N = s->N, E = s->E, D = s->D;
    if (rank < 0 || rank >= N) {
        set_error("%s: rank %d outside [0, %d)", who, rank, N);
        return MOE_ERR_INVALID_ARG;
    }
    int64_t total = 0;
    for (int64_t q = 0; q < (int64_t)N * E; ++q) {
        if (A[q] < 0) {
            set_error("%s: A has a negative entry", who);
            return MOE_ERR_INVALID_ARG;
        }
        total += A[q];
    }
    if (total > (int64_t)N * s->C) {
        set_error("%s: the layout holds %lld replicas, more than N*C = %lld", who, (long long)total, (long long)N * s->C);
        return MOE_ERR_INVALID_ARG;
    }
    int G = 0;
    for (int i = 0; i < N; ++i)
        for (int j = 0; j < E; ++j)
            for (int m = 0; m < A[(size_t)i * E + j]; ++m) {
                expert_of_group[G] = j;
                device_of_group[G] = i;
                ++G;
            }
    const int node = rank / D;
    int n = 0;
    rep_begin[0] = 0;
    for (int j = 0; j < E; ++j) {
        const int first = n;
        for (int g = 0; g < G; ++g)
            if (expert_of_group[g] == j && device_of_group[g] / D == node) rep_group[n++] = g;
        if (n == first)
            for (int g = 0; g < G; ++g)
                if (expert_of_group[g] == j) rep_group[n++] = g;
        rep_begin[j + 1] = n;
    }
    *G_out = G;
    *n_rep_out = n;
    return MOE_OK;
}
