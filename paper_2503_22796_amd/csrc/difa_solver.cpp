// Head-wise plan selection for one layer (Sec. 3.4.2, Eq. 2): every head takes at most one method, the
// chosen influences add up to at most delta, no chosen influence exceeds (c / heads) * delta, and the
// total latency (full attention for a head without a method) is minimal.
//
// Host code, exact.  The problem is a multiple-choice knapsack with real weights; it is solved by
// sweeping the heads and keeping, after each, the Pareto frontier of (influence spent, latency saved):
// a partial assignment that spends more and saves no more than another can never become optimal.  The
// frontier is kept sorted by influence, so pruning is one pass.  Each frontier entry remembers its
// predecessor and its head's choice, which gives the assignment back at the end.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <new>
#include <vector>

#include "difa.h"

namespace {

struct State {
    double spent;    // sum of the chosen influences
    double saved;    // sum of (latency_full - latency[m]) over the chosen methods
    int32_t prev;    // index into the previous head's frontier
    int32_t choice;  // this head's method, -1 = full attention
};

constexpr size_t kMaxFrontier = (size_t)1 << 20;

}  // namespace

extern "C" difa_status_t difa_plan_solve(const double* influence, const double* latency, double latency_full,
                                         int32_t heads, int32_t n_methods, double delta, double c,
                                         int32_t* choice_out, double* total_latency_out,
                                         double* total_influence_out) {
    if (!influence || !latency || !choice_out || heads < 1 || n_methods < 1) return DIFA_ERR_INVALID_ARG;
    // (this file is compiled with IEEE comparisons: a NaN fails every test below.  An influence of +inf
    // is legal -- the metric of a head whose original output is constant -- and is never chosen;
    // latencies must be finite, or the total would not be a number.)
    if (!(delta >= 0.0) || !(c >= 0.0) || !(latency_full >= 0.0) || std::isinf(latency_full)) return DIFA_ERR_INVALID_ARG;
    for (int64_t i = 0; i < (int64_t)heads * n_methods; ++i)
        if (std::isnan(influence[i]) || !(influence[i] >= 0.0)) return DIFA_ERR_INVALID_ARG;
    for (int32_t m = 0; m < n_methods; ++m)
        if (std::isnan(latency[m]) || !(latency[m] >= 0.0) || std::isinf(latency[m])) return DIFA_ERR_INVALID_ARG;
    const double cap = c / (double)heads * delta;

    try {
        std::vector<std::vector<State>> layers((size_t)heads);
        std::vector<State> cand;
        std::vector<State> start(1, State{0.0, 0.0, -1, -1});
        const std::vector<State>* prev = &start;
        for (int32_t h = 0; h < heads; ++h) {
            cand.clear();
            const double* row = influence + (int64_t)h * n_methods;
            for (int32_t s = 0; s < (int32_t)prev->size(); ++s) {
                const State& st = (*prev)[(size_t)s];
                cand.push_back(State{st.spent, st.saved, s, -1});
                for (int32_t m = 0; m < n_methods; ++m) {
                    const double gain = latency_full - latency[m];
                    if (gain <= 0.0 || row[m] > cap) continue;        // never better than full attention / over the head's cap
                    const double spent = st.spent + row[m];
                    if (spent > delta) continue;
                    cand.push_back(State{spent, st.saved + gain, s, m});
                }
            }
            // cheapest first; among equal spendings the larger saving first, so that the pass below keeps it
            std::sort(cand.begin(), cand.end(), [](const State& a, const State& b) {
                return a.spent != b.spent ? a.spent < b.spent : a.saved > b.saved;
            });
            std::vector<State>& front = layers[(size_t)h];
            double best_saved = -1.0;
            for (const State& st : cand)
                if (st.saved > best_saved) {
                    front.push_back(st);
                    best_saved = st.saved;
                }
            if (front.size() > kMaxFrontier) return DIFA_ERR_UNSUPPORTED;
            prev = &front;
        }
        // the frontier's savings increase with the spending: the last entry is the optimum
        const std::vector<State>& last = layers[(size_t)heads - 1];
        int32_t idx = (int32_t)last.size() - 1;
        const double saved = last[(size_t)idx].saved, spent = last[(size_t)idx].spent;
        for (int32_t h = heads - 1; h >= 0; --h) {
            const State& st = layers[(size_t)h][(size_t)idx];
            choice_out[h] = st.choice;
            idx = st.prev;
        }
        if (total_latency_out) *total_latency_out = (double)heads * latency_full - saved;
        if (total_influence_out) *total_influence_out = spent;
    } catch (const std::bad_alloc&) {
        return DIFA_ERR_ALLOC;
    }
    return DIFA_OK;
}
