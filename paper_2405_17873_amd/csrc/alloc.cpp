// Bit-width allocation on the host (no GPU work): the integer programme of Sec. 3.3, Eq. 2, and the budget / ratio
// scan of App. A, Alg. 1 around it.
//
// Eq. 2 is a multiple-choice knapsack: one choice per layer, maximise the summed score within a cost budget.  It is
// solved exactly:
//   1. The linear relaxation is solved greedily over the upper convex hulls of the layers' (cost, score) points; the
//      slope at which the budget runs out is the multiplier lambda, and rounding the relaxed solution down gives a
//      first feasible assignment (the incumbent).
//   2. A dynamic programme walks the layers and keeps, per layer, the list of (cost, score) states that are not
//      dominated (no cheaper-or-equal state scores at least as much).  A state is dropped when it cannot be completed
//      within the budget, or when its Lagrangian bound  score + sum_rest max_b(S - lambda*M) + lambda*(B - cost)
//      falls below the incumbent: that bound holds for every lambda >= 0, and with the relaxation's own lambda it is
//      tight enough that only states next to the relaxed optimum survive (a few hundred per layer on a 790-layer
//      UNet table, whatever the size of the costs).
//   3. The best final state is traced back through per-layer parent links.
// Scores are added in layer order in double precision, so the reported objective is reproducible to the last bit.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <map>
#include <vector>

#include "../../include/mixdq.h"

namespace {

struct State {
    int64_t cost;
    double value;
    int32_t parent;  // index into the previous layer's list
    int32_t choice;
};

struct Step {  // one move up a layer's convex hull
    double slope;
    int64_t dcost;
    double dvalue;
    int32_t layer, from, to;  // positions in that layer's hull
};

constexpr size_t kMaxStates = 40u * 1000u * 1000u;  // over all layers (16 bytes each)

// Upper convex hull of one layer's choices in the (cost, score) plane, cheapest first; ties in cost keep the
// higher score.  Returns indices into the layer's choice list.
std::vector<int> hull_of(const double* s, const int64_t* c, int m) {
    std::vector<int> idx(m);
    for (int b = 0; b < m; ++b) idx[b] = b;
    std::sort(idx.begin(), idx.end(), [&](int a, int b) { return c[a] != c[b] ? c[a] < c[b] : s[a] > s[b]; });
    std::vector<int> h;
    for (int b : idx) {
        if (!h.empty() && s[b] <= s[h.back()]) continue;  // costs more (or the same) and scores no more
        while (h.size() >= 2) {
            const int p = h[h.size() - 2], q = h.back();
            // q lies on or under the chord p -> b: drop it
            const long double lhs = (long double)(s[q] - s[p]) * (long double)(c[b] - c[p]);
            const long double rhs = (long double)(s[b] - s[p]) * (long double)(c[q] - c[p]);
            if (lhs <= rhs) h.pop_back(); else break;
        }
        h.push_back(b);
    }
    return h;
}

int solve(int n, int m, const double* sens, const int64_t* cost, int64_t budget, int32_t* choice_out,
          double* objective_out, int64_t* cost_out) {
    // cheapest completion of every suffix (cost and the score that goes with it)
    std::vector<int64_t> rest_cost(n + 1, 0);
    std::vector<int> cheapest(n);
    for (int i = n - 1; i >= 0; --i) {
        const double* s = sens + (size_t)i * m;
        const int64_t* c = cost + (size_t)i * m;
        int best = 0;
        for (int b = 1; b < m; ++b)
            if (c[b] < c[best] || (c[b] == c[best] && s[b] > s[best])) best = b;
        cheapest[i] = best;
        if (rest_cost[i + 1] > std::numeric_limits<int64_t>::max() - c[best]) return MQ_ERR_BAD_ARG;
        rest_cost[i] = rest_cost[i + 1] + c[best];
    }
    if (rest_cost[0] > budget) return MQ_ERR_INFEASIBLE;

    // 1. linear relaxation -> lambda and an incumbent
    std::vector<std::vector<int>> hulls(n);
    std::vector<Step> steps;
    for (int i = 0; i < n; ++i) {
        const double* s = sens + (size_t)i * m;
        const int64_t* c = cost + (size_t)i * m;
        hulls[i] = hull_of(s, c, m);
        for (size_t j = 1; j < hulls[i].size(); ++j) {
            const int p = hulls[i][j - 1], q = hulls[i][j];
            steps.push_back({(s[q] - s[p]) / (double)(c[q] - c[p]), c[q] - c[p], s[q] - s[p], i, (int)j - 1, (int)j});
        }
    }
    std::stable_sort(steps.begin(), steps.end(), [](const Step& a, const Step& b) { return a.slope > b.slope; });
    std::vector<int> at(n, 0);  // hull position per layer
    int64_t left = budget - rest_cost[0];
    double lambda = 0.0;
    bool ran_out = false;
    for (const Step& st : steps) {
        if (at[st.layer] != st.from) continue;  // an earlier step of this layer did not fit
        if (st.dcost <= left) {
            left -= st.dcost;
            at[st.layer] = st.to;
        } else if (!ran_out) {
            ran_out = true;
            lambda = st.slope;  // the relaxation would take a fraction of this step
        }
    }
    std::vector<int32_t> incumbent_choice(n);
    double incumbent = 0.0;
    for (int i = 0; i < n; ++i) {
        incumbent_choice[i] = hulls[i][at[i]];
        incumbent += sens[(size_t)i * m + incumbent_choice[i]];
    }

    // Lagrangian bound of every suffix, and a slack that covers the rounding of the bound's own arithmetic
    std::vector<double> rest_bound(n + 1, 0.0);
    double magnitude = 0.0;
    for (int i = n - 1; i >= 0; --i) {
        double best = -std::numeric_limits<double>::infinity(), big = 0.0;
        for (int b = 0; b < m; ++b) {
            best = std::max(best, sens[(size_t)i * m + b] - lambda * (double)cost[(size_t)i * m + b]);
            big = std::max(big, std::fabs(sens[(size_t)i * m + b]) + lambda * (double)cost[(size_t)i * m + b]);
        }
        rest_bound[i] = rest_bound[i + 1] + best;
        magnitude += big;
    }
    const double slack = 1e-9 * (magnitude + lambda * (double)budget + 1.0);

    // 2. dynamic programme over undominated states
    std::vector<std::vector<State>> lists(n + 1);
    lists[0].push_back({0, 0.0, -1, -1});
    size_t total_states = 1;
    std::vector<State> cand;
    for (int i = 0; i < n; ++i) {
        const double* s = sens + (size_t)i * m;
        const int64_t* c = cost + (size_t)i * m;
        cand.clear();
        const std::vector<State>& prev = lists[i];
        for (int32_t p = 0; p < (int32_t)prev.size(); ++p)
            for (int b = 0; b < m; ++b) {
                const int64_t nc = prev[p].cost + c[b];
                if (nc + rest_cost[i + 1] > budget) continue;
                const double nv = prev[p].value + s[b];
                const double bound = nv + rest_bound[i + 1] + lambda * (double)(budget - nc);
                if (bound < incumbent - slack) continue;
                cand.push_back({nc, nv, p, b});
            }
        std::sort(cand.begin(), cand.end(), [](const State& a, const State& b) {
            return a.cost != b.cost ? a.cost < b.cost : a.value > b.value;
        });
        std::vector<State>& cur = lists[i + 1];
        for (const State& st : cand)
            if (cur.empty() || st.value > cur.back().value) cur.push_back(st);
        if (cur.empty()) {
            // every state fell under the incumbent: the relaxation's rounding is optimal
            break;
        }
        total_states += cur.size();
        if (total_states > kMaxStates) return MQ_ERR_TOO_LARGE;
        // (no incumbent update from partial states: completing one with the cheapest remaining choices is what the
        // relaxation's rounding already explored near the optimum)
    }

    // 3. the best complete state, if the programme reached the last layer with one that beats the incumbent
    std::vector<int32_t> choice = incumbent_choice;
    if (!lists[n].empty()) {
        const State* best = &lists[n][0];
        for (const State& st : lists[n])
            if (st.value > best->value) best = &st;
        if (best->value > incumbent) {
            const State* st = best;
            for (int i = n; i >= 1; --i) {
                choice[i - 1] = st->choice;
                st = &lists[i - 1][st->parent];
            }
        }
    }
    double obj = 0.0;
    int64_t used = 0;
    for (int i = 0; i < n; ++i) {
        obj += sens[(size_t)i * m + choice[i]];
        used += cost[(size_t)i * m + choice[i]];
    }
    if (choice_out) std::memcpy(choice_out, choice.data(), sizeof(int32_t) * (size_t)n);
    if (objective_out) *objective_out = obj;
    if (cost_out) *cost_out = used;
    return MQ_OK;
}

}  // namespace

extern "C" {

int mq_alloc_solve(int n_layers, int n_choices, const double* sens_host, const int64_t* cost_host, int64_t budget,
                   int32_t* choice_host, double* objective_host, int64_t* cost_used_host) {
    if (!sens_host || !cost_host || !choice_host) return MQ_ERR_BAD_ARG;
    if (n_layers <= 0 || n_choices <= 0) return MQ_ERR_BAD_SHAPE;
    for (size_t i = 0; i < (size_t)n_layers * n_choices; ++i)
        if (cost_host[i] < 0 || !std::isfinite(sens_host[i])) return MQ_ERR_BAD_ARG;
    return solve(n_layers, n_choices, sens_host, cost_host, budget, choice_host, objective_host, cost_used_host);
}

int mq_alloc_split_budget(int64_t budget_all, int64_t params_content, int64_t params_quality, double k,
                          int64_t* budget_content_host, int64_t* budget_quality_host) {
    if (!budget_content_host || !budget_quality_host) return MQ_ERR_BAD_ARG;
    if (params_content <= 0 || params_quality <= 0 || !(k > 0.0) || budget_all < 0) return MQ_ERR_BAD_SHAPE;
    const double avg_q = (double)budget_all / (k * (double)params_content + (double)params_quality);
    const int64_t bc = (int64_t)std::floor(k * avg_q * (double)params_content);
    *budget_content_host = bc;
    *budget_quality_host = budget_all - bc;
    return MQ_OK;
}

int mq_alloc_search(int n_content, const double* sens_content_host, const int64_t* params_content_host, int n_quality,
                    const double* sens_quality_host, const int64_t* params_quality_host, int n_choices,
                    const int32_t* bits_host, double avg_bits_target, double delta_avg_bits, int n_budgets, double k_lo,
                    double k_hi, int n_ratios, int64_t* budgets_host, double* k_host, int32_t* feasible_host,
                    double* objectives_host, int32_t* choice_content_host, int32_t* choice_quality_host) {
    if (!sens_content_host || !params_content_host || !sens_quality_host || !params_quality_host || !bits_host ||
        !budgets_host || !k_host || !feasible_host || !objectives_host || !choice_content_host || !choice_quality_host)
        return MQ_ERR_BAD_ARG;
    if (n_content <= 0 || n_quality <= 0 || n_choices <= 0 || n_budgets <= 0 || n_ratios <= 0) return MQ_ERR_BAD_SHAPE;
    if (!(k_lo > 0.0) || !(k_hi >= k_lo) || !(avg_bits_target > 0.0) || !(delta_avg_bits >= 0.0)) return MQ_ERR_BAD_ARG;
    int64_t pc = 0, pq = 0;
    for (int b = 0; b < n_choices; ++b)
        if (bits_host[b] <= 0) return MQ_ERR_UNSUPPORTED_BITS;
    std::vector<int64_t> cost_c((size_t)n_content * n_choices), cost_q((size_t)n_quality * n_choices);
    for (int i = 0; i < n_content; ++i) {
        if (params_content_host[i] <= 0) return MQ_ERR_BAD_SHAPE;
        pc += params_content_host[i];
        for (int b = 0; b < n_choices; ++b) cost_c[(size_t)i * n_choices + b] = params_content_host[i] * bits_host[b];
    }
    for (int i = 0; i < n_quality; ++i) {
        if (params_quality_host[i] <= 0) return MQ_ERR_BAD_SHAPE;
        pq += params_quality_host[i];
        for (int b = 0; b < n_choices; ++b) cost_q[(size_t)i * n_choices + b] = params_quality_host[i] * bits_host[b];
    }
    for (size_t i = 0; i < (size_t)n_content * n_choices; ++i)
        if (!std::isfinite(sens_content_host[i])) return MQ_ERR_BAD_ARG;
    for (size_t i = 0; i < (size_t)n_quality * n_choices; ++i)
        if (!std::isfinite(sens_quality_host[i])) return MQ_ERR_BAD_ARG;
    const int64_t b_all = (int64_t)std::floor(avg_bits_target * (double)(pc + pq));
    const int64_t d_b = (int64_t)std::floor(delta_avg_bits * (double)(pc + pq));

    // the same group budget comes up under several (budget, ratio) pairs: solve each once
    struct Solved {
        int rc;
        double objective;
        std::vector<int32_t> choice;
    };
    std::map<int64_t, Solved> memo_c, memo_q;
    auto solved = [&](std::map<int64_t, Solved>& memo, int n, const double* sens, const std::vector<int64_t>& cost,
                      int64_t budget) -> const Solved& {
        auto it = memo.find(budget);
        if (it != memo.end()) return it->second;
        Solved s;
        s.choice.resize(n);
        s.objective = 0.0;
        s.rc = solve(n, n_choices, sens, cost.data(), budget, s.choice.data(), &s.objective, nullptr);
        return memo.emplace(budget, std::move(s)).first->second;
    };
    for (int j = 0; j < n_budgets; ++j) {
        const double frac = n_budgets > 1 ? (double)j / (double)(n_budgets - 1) : 1.0;
        const int64_t bj = b_all - d_b + (int64_t)std::floor(frac * (double)d_b);
        for (int t = 0; t < n_ratios; ++t) {
            const size_t e = (size_t)j * n_ratios + t;
            const double k = k_lo + (k_hi - k_lo) * (n_ratios > 1 ? (double)t / (double)(n_ratios - 1) : 0.0);
            int64_t bc = 0, bq = 0;
            int rc = mq_alloc_split_budget(bj, pc, pq, k, &bc, &bq);
            if (rc) return rc;
            budgets_host[e * 3 + 0] = bj;
            budgets_host[e * 3 + 1] = bc;
            budgets_host[e * 3 + 2] = bq;
            k_host[e] = k;
            const Solved& sc = solved(memo_c, n_content, sens_content_host, cost_c, bc);
            const Solved& sq = solved(memo_q, n_quality, sens_quality_host, cost_q, bq);
            if ((sc.rc && sc.rc != MQ_ERR_INFEASIBLE) || (sq.rc && sq.rc != MQ_ERR_INFEASIBLE)) return sc.rc ? sc.rc : sq.rc;
            const bool ok = sc.rc == MQ_OK && sq.rc == MQ_OK;
            feasible_host[e] = ok ? 1 : 0;
            objectives_host[e * 2 + 0] = ok ? sc.objective : 0.0;
            objectives_host[e * 2 + 1] = ok ? sq.objective : 0.0;
            for (int i = 0; i < n_content; ++i) choice_content_host[e * n_content + i] = ok ? sc.choice[i] : -1;
            for (int i = 0; i < n_quality; ++i) choice_quality_host[e * n_quality + i] = ok ? sq.choice[i] : -1;
        }
    }
    return MQ_OK;
}

}  // extern "C"
