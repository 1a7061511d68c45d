// Adapter placement and request routing (host only): the steps are described in
// include/lora_placement.h.
#include "../../include/lora_placement.h"

#include <algorithm>
#include <cmath>
#include <limits>
#include <map>
#include <new>
#include <vector>

// No exception crosses the C boundary: every entry point is a function-try-block that ends in this.
#define API_CATCH                                        \
    catch (const std::bad_alloc &) { return LORA_ERR_OOM; } \
    catch (...) { return LORA_ERR_INVALID_ARG; }

namespace {

const double kEps = 1e-12;

// Largest-weight perfect matching of an n x n matrix (rows = new servers, columns = old labels):
// shortest augmenting paths with potentials on cost = -weight.  Returns col_of_row.
std::vector<int> max_weight_assignment(const std::vector<std::vector<double>> &w)
{
    const int n = (int)w.size();
    const double inf = std::numeric_limits<double>::infinity();
    std::vector<double> u(n + 1, 0.0), v(n + 1, 0.0);
    std::vector<int> p(n + 1, 0), way(n + 1, 0);
    for (int i = 1; i <= n; ++i) {
        p[0] = i;
        int j0 = 0;
        std::vector<double> minv(n + 1, inf);
        std::vector<char> used(n + 1, 0);
        do {
            used[j0] = 1;
            const int i0 = p[j0];
            double delta = inf;
            int j1 = 0;
            for (int j = 1; j <= n; ++j) {
                if (used[j]) continue;
                const double cur = -w[i0 - 1][j - 1] - u[i0] - v[j];
                if (cur < minv[j]) {
                    minv[j] = cur;
                    way[j] = j0;
                }
                if (minv[j] < delta) {
                    delta = minv[j];
                    j1 = j;
                }
            }
            for (int j = 0; j <= n; ++j) {
                if (used[j]) {
                    u[p[j]] += delta;
                    v[j] -= delta;
                } else {
                    minv[j] -= delta;
                }
            }
            j0 = j1;
        } while (p[j0] != 0);
        do {
            const int j1 = way[j0];
            p[j0] = p[j1];
            j0 = j1;
        } while (j0);
    }
    std::vector<int> col_of_row(n, 0);
    for (int j = 1; j <= n; ++j) col_of_row[p[j] - 1] = j - 1;
    return col_of_row;
}

}  // namespace

extern "C" lora_status_t lora_place_extrapolate(const double *history, int32_t n, double current, double *demand)
try {
    if (!demand || n < 0 || (n > 0 && !history)) return LORA_ERR_INVALID_ARG;
    const double d = n == 0 ? current : current + (current - history[n - 1]);
    *demand = d > 0.0 ? d : 0.0;
    return LORA_OK;
}
API_CATCH

extern "C" lora_status_t lora_place_assign(const lora_place_problem_t *pr, double *phi, double *server_util,
                                           int32_t *server_max_rank, int32_t *rank_budget, double *target_util)
try {
    if (!pr || pr->n_servers < 1 || pr->n_adapters < 0 || pr->n_ops < 0) return LORA_ERR_INVALID_ARG;
    const int S = pr->n_servers, N = pr->n_adapters;
    if (N > 0 && (!pr->ranks || !pr->demand_tps || !phi)) return LORA_ERR_INVALID_ARG;
    if (pr->n_ops > 0 && (!pr->op_ranks || !pr->op_tps)) return LORA_ERR_INVALID_ARG;
    std::map<int, double> op;
    for (int i = 0; i < pr->n_ops; ++i) {
        if (!(pr->op_tps[i] > 0.0) || op.count(pr->op_ranks[i])) return LORA_ERR_INVALID_ARG;
        op[pr->op_ranks[i]] = pr->op_tps[i];
    }
    std::vector<double> load(N);  // utilisation an adapter asks for
    for (int a = 0; a < N; ++a) {
        if (!op.count(pr->ranks[a]) || !(pr->demand_tps[a] >= 0.0)) return LORA_ERR_INVALID_ARG;
        load[a] = pr->demand_tps[a] / op[pr->ranks[a]];
    }

    // step 1: utilisation per rank (ranks ascending, adapters in id order), target per server
    std::map<int, double> rank_util;
    for (int a = 0; a < N; ++a) rank_util[pr->ranks[a]];
    for (auto &ru : rank_util) {
        double sum = 0.0;
        for (int a = 0; a < N; ++a)
            if (pr->ranks[a] == ru.first) sum += pr->demand_tps[a];
        ru.second = sum / op[ru.first];
    }
    double target = 0.0;
    for (const auto &ru : rank_util) target += ru.second;
    target /= S;

    // step 2: servers per rank
    std::map<int, int> budget;
    for (const auto &ru : rank_util) budget[ru.first] = target > 0.0 ? (int)std::floor(ru.second / target + 0.5) : 0;

    std::vector<std::vector<double>> f(N, std::vector<double>(S, 0.0));
    std::vector<double> util(S, 0.0);
    std::vector<int> max_rank(S, 0);
    std::vector<char> started(N, 0);

    // step 3: fractional bin packing, highest rank first, consecutive servers
    int next_server = 0;
    for (auto it = budget.rbegin(); it != budget.rend(); ++it) {
        const int r = it->first;
        const int first = next_server, last = std::min(S, next_server + it->second);  // [first, last)
        next_server = last;
        if (last <= first) continue;
        std::vector<int> order;
        for (int a = 0; a < N; ++a)
            if (pr->ranks[a] == r && pr->demand_tps[a] > 0.0) order.push_back(a);
        std::stable_sort(order.begin(), order.end(),
                         [&](int x, int y) { return pr->demand_tps[x] > pr->demand_tps[y]; });
        int b = first;
        for (int a : order) {
            if (b >= last) break;
            const double whole = load[a];
            double left = whole;
            started[a] = 1;
            while (left > kEps * std::max(1.0, whole) && b < last) {
                const double take = std::min(left, target - util[b]);
                if (take > 0.0) {
                    f[a][b] += take / whole;
                    util[b] += take;
                    max_rank[b] = std::max(max_rank[b], r);
                    left -= take;
                }
                if (util[b] >= target - kEps * std::max(1.0, target)) ++b;
            }
            if (left > kEps * std::max(1.0, whole)) {
                f[a][last - 1] += left / whole;
                util[last - 1] += left;
            }
            double sum = 0.0;
            for (int s = 0; s < S; ++s) sum += f[a][s];
            for (int s = 0; s < S; ++s) f[a][s] /= sum;
        }
    }

    // step 4: what is left, highest rank first
    std::vector<int> rest;
    for (int a = 0; a < N; ++a)
        if (!started[a]) rest.push_back(a);
    std::stable_sort(rest.begin(), rest.end(), [&](int x, int y) {
        if (pr->ranks[x] != pr->ranks[y]) return pr->ranks[x] > pr->ranks[y];
        return pr->demand_tps[x] > pr->demand_tps[y];
    });
    for (int a : rest) {
        const int r = pr->ranks[a];
        int best = -1;
        for (int s = 0; s < S; ++s) {
            if (!(max_rank[s] == 0 || max_rank[s] >= r)) continue;
            if (best < 0 || util[s] < util[best] || (util[s] == util[best] && max_rank[s] > max_rank[best])) best = s;
        }
        if (best < 0) {
            best = 0;
            for (int s = 1; s < S; ++s)
                if (max_rank[s] > max_rank[best] || (max_rank[s] == max_rank[best] && util[s] < util[best])) best = s;
        }
        f[a][best] = 1.0;
        util[best] += load[a];
        max_rank[best] = std::max(max_rank[best], r);
    }

    // step 5: relabel the servers to keep as much of the previous assignment as possible
    std::vector<int> label(S);
    for (int s = 0; s < S; ++s) label[s] = s;
    if (pr->prev_phi && N > 0) {
        std::vector<std::vector<double>> keep(S, std::vector<double>(S, 0.0));
        for (int a = 0; a < N; ++a)
            for (int i = 0; i < S; ++i) {
                if (!(f[a][i] > 0.0)) continue;
                for (int j = 0; j < S; ++j)
                    if (pr->prev_phi[(size_t)a * S + j] > 0.0) keep[i][j] += (double)pr->ranks[a];
            }
        label = max_weight_assignment(keep);
    }
    for (int a = 0; a < N; ++a)
        for (int i = 0; i < S; ++i) phi[(size_t)a * S + label[i]] = f[a][i];
    for (int i = 0; i < S; ++i) {
        if (server_util) server_util[label[i]] = util[i];
        if (server_max_rank) server_max_rank[label[i]] = max_rank[i];
    }
    if (rank_budget)
        for (int i = 0; i < pr->n_ops; ++i) rank_budget[i] = budget.count(pr->op_ranks[i]) ? budget[pr->op_ranks[i]] : 0;
    if (target_util) *target_util = target;
    return LORA_OK;
}
API_CATCH
