// Execution order of offloaded experts (CPM-2 Section 6.2, the part on scheduling offloaded experts).
//
// Expert i needs alpha_i of computation, proportional to its token count n_i, and every expert the same
// beta of parameter loading; the order o_1..o_T should satisfy for every position t
//     sum_{i<t} alpha_{o_i} >= (t - 1) beta         each load is covered by earlier computation
//     sum_{i<t} alpha_{o_i} <= (t + K - 1) beta     loads do not run more than K experts ahead
// and comes from a greedy pass.  The paper does not print the rule; the one used here keeps the
// slack (computation chosen so far minus loads so far) as high as the second constraint allows:
// at every position the remaining expert with the most tokens that keeps it, else the one with the
// fewest.  Everything is expressed in tokens: r = beta / alpha_per_token is the number of tokens whose
// computation lasts as long as one load, so the tests are  sum n >= (t - 1) r  and  sum n <= (t + K - 1) r,
// one integer sum against one product, identical on every machine.
//
// Host code only.
#include "common.h"

#include <vector>

namespace moe {

int schedule_order(const int32_t* counts, int E, double r, int K, int32_t* order, int* n_order, int* satisfiable) {
    std::vector<int> left;
    left.reserve(E);
    for (int e = 0; e < E; ++e)
        if (counts[e] > 0) left.push_back(e);
    const int n = static_cast<int>(left.size());
    long long sum = 0;
    for (int pos = 0; pos < n; ++pos) {
        // after this choice the slack must not exceed K loads: sum + n_e <= (pos + 1 + K) r
        const double cap = static_cast<double>(pos + 1 + K) * r;
        int best = -1, fewest = 0;
        for (int j = 0; j < static_cast<int>(left.size()); ++j) {
            const int e = left[j];
            if (counts[e] < counts[left[fewest]]) fewest = j;          // first of the fewest = lowest id
            if (static_cast<double>(sum + counts[e]) <= cap && (best < 0 || counts[e] > counts[left[best]])) best = j;
        }
        const int take = best >= 0 ? best : fewest;
        order[pos] = left[take];
        sum += counts[left[take]];
        left.erase(left.begin() + take);
    }
    bool ok = true;
    long long prefix = 0;
    for (int t = 1; t <= n; ++t) {
        const double p = static_cast<double>(prefix);
        if (p < static_cast<double>(t - 1) * r || p > static_cast<double>(t + K - 1) * r) ok = false;
        prefix += counts[order[t - 1]];
    }
    *n_order = n;
    if (satisfiable != nullptr) *satisfiable = ok ? 1 : 0;
    return MOE_OK;
}

// Which slot every expert of a call runs from when the K slots keep their experts between calls
// (Section 6.2: K experts reside in GPU memory), and whether it has to be loaded first.  The whole
// order of the call is known before its first load, so the resident expert whose next use in this
// call lies furthest ahead gives way: an empty slot first, else never-used-again before used-later,
// among equals the slot unused for longest, then the lowest slot.  For a known sequence this
// minimises the number of loads.
//   order[n]      experts in execution order
//   slot_expert[K], slot_tick[K]  in/out: expert held by each slot (-1 = none) and when it was last used
//   *tick         in/out: use counter
//   slot_of[n], load[n]  out
int plan_slots(const int32_t* order, int n, int K, int32_t* slot_expert, int64_t* slot_tick, int64_t* tick,
               int32_t* slot_of, int32_t* load) {
    for (int pos = 0; pos < n; ++pos) {
        const int e = order[pos];
        int s = -1;
        for (int i = 0; i < K; ++i)
            if (slot_expert[i] == e) { s = i; break; }
        load[pos] = s < 0 ? 1 : 0;
        if (s < 0) {
            long best_next = -1;
            for (int i = 0; i < K; ++i) {
                long next = 0;                              // empty: better than any held expert
                if (slot_expert[i] >= 0) {
                    next = n + 1;                           // never again in this call
                    for (int j = pos + 1; j < n; ++j)
                        if (order[j] == slot_expert[i]) { next = j; break; }
                }
                const bool empty = slot_expert[i] < 0;
                bool better;
                if (s < 0) better = true;
                else {
                    const bool s_empty = slot_expert[s] < 0;
                    if (empty != s_empty) better = empty;
                    else if (next != best_next) better = next > best_next;
                    else better = slot_tick[i] < slot_tick[s];      // equal ticks: the lower slot stays chosen
                }
                if (better) { s = i; best_next = next; }
            }
            slot_expert[s] = e;
        }
        slot_tick[s] = ++*tick;
        slot_of[pos] = s;
    }
    return MOE_OK;
}

}  // namespace moe
