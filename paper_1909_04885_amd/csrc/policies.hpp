// Host-side scheduling policies (Section 4.5) and the iteration-time projection model of the
// evaluation (Sections 5.3 and 5.4).  Pure functions over plain arrays: they compute chunk -> solver
// tables and normalised times, never touch the device.
#pragma once
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <numeric>
#include <vector>

namespace chicle {

// Iteration time in units of "one task on 1/base_nodes of the data on a fast node".
//   K_tasks > 0 : that many equal micro-tasks, scheduled in waves over the nodes
//   K_tasks = 0 : uni-tasks, one per node, each sized to its node's speed
// n_slow of the nodes take slow_factor times as long per task.
inline double projected_iteration_time(int K_tasks, int nodes, int n_slow, double slow_factor, int base_nodes)
{
    const int n_fast = nodes - n_slow;
    if (K_tasks == 0) {
        // every node finishes at the same moment: capacity is the sum of the relative speeds
        const double capacity = (double)n_fast + (n_slow > 0 ? (double)n_slow / slow_factor : 0.0);
        return (double)base_nodes / capacity;
    }
    const double task = (double)base_nodes / (double)K_tasks;
    if (n_slow == 0) return task * (double)((K_tasks + nodes - 1) / nodes);
    // i tasks on every slow node, the rest spread over the fast ones: shortest such schedule
    double best = std::numeric_limits<double>::infinity();
    for (int i = 0; i <= (K_tasks + n_slow - 1) / n_slow; ++i) {
        const int rest = std::max(K_tasks - i * n_slow, 0);
        if (n_fast == 0 && rest > 0) continue;
        const int j = n_fast ? (rest + n_fast - 1) / n_fast : 0;
        best = std::min(best, std::max((double)i * slow_factor, (double)j) * task);
    }
    return best;
}

// When to scale in (Section 2.2: start with many partitions and reduce them after a few iterations; the
// evaluation's summary: scale in when convergence slows down).  A round has stalled when it left more
// than stall_ratio of the gap it started from; after `patience` stalled rounds in a row, all run with
// the current K, the number of solvers is halved (rounded up, never below K_min).
inline int next_solver_count(const double *gap, int n_gaps, int K, int K_min, double stall_ratio, int patience,
                             int since_change)
{
    if (K <= K_min || since_change < patience || n_gaps < patience + 1) return K;
    for (int t = n_gaps - patience; t < n_gaps; ++t)
        if (!(gap[t] > stall_ratio * gap[t - 1])) return K;
    return std::max(K_min, (K + 1) / 2);
}

// Scale-out: solvers K_old .. K_new-1 are new.  Every old solver hands over
// floor(count * (K_new - K_old) / K_new) of its chunks, those with the smallest draw (ties: smaller
// chunk id); the handed-over chunks, taken old solver by old solver in pick order, are dealt to the
// new solvers in turn.
inline void scale_out_table(int n_chunks, const int32_t *in, int K_old, int K_new, const uint32_t *draw,
                            int32_t *out)
{
    std::vector<std::vector<int32_t>> own(K_old);
    for (int c = 0; c < n_chunks; ++c) {
        out[c] = in[c];
        own[in[c]].push_back(c);
    }
    int turn = 0;
    for (int k = 0; k < K_old; ++k) {
        std::vector<int32_t> &lst = own[k];
        const int64_t give = (int64_t)lst.size() * (K_new - K_old) / K_new;
        std::stable_sort(lst.begin(), lst.end(), [&](int32_t a, int32_t b) { return draw[a] < draw[b]; });
        for (int64_t t = 0; t < give; ++t) {
            out[lst[t]] = K_old + turn;
            turn = (turn + 1) % (K_new - K_old);
        }
    }
}

// Scale-in: solvers K_new .. K_old-1 are freed.  Their chunks, taken freed solver by freed solver in
// ascending chunk id, are dealt to the remaining solvers 0, 1, .., K_new-1, 0, .. in turn.
inline void scale_in_table(int n_chunks, const int32_t *in, int K_old, int K_new, int32_t *out)
{
    std::vector<std::vector<int32_t>> own(K_old);
    for (int c = 0; c < n_chunks; ++c) {
        out[c] = in[c];
        own[in[c]].push_back(c);
    }
    int turn = 0;
    for (int k = K_new; k < K_old; ++k)
        for (int32_t c : own[k]) {
            out[c] = turn;
            turn = (turn + 1) % K_new;
        }
}

inline double median_of(std::vector<double> v)
{
    std::sort(v.begin(), v.end());
    const size_t m = v.size();
    return (m & 1) ? v[m / 2] : 0.5 * (v[m / 2 - 1] + v[m / 2]);
}

// Gradual rebalancing.  unit_time is I x K row-major: runtime per unit of load that solver k showed
// in each of the last I iterations; a solver's rate is the median of its column.  Up to max_moves
// times: the solver with the longest projected time (rate * load) hands its lightest chunk (ties:
// larger id) to the solver with the shortest, unless the difference is no more than what that chunk
// would take on the receiver.  Returns the number of chunks moved.
inline int rebalance_table(const int64_t *load, int n_chunks, int K, const double *unit_time, int I,
                           int max_moves, int32_t *table)
{
    std::vector<double> rate(K);
    std::vector<double> col(I);
    for (int k = 0; k < K; ++k) {
        for (int i = 0; i < I; ++i) col[i] = unit_time[(size_t)i * K + k];
        rate[k] = median_of(col);
    }
    std::vector<int64_t> L(K, 0);
    for (int c = 0; c < n_chunks; ++c) L[table[c]] += load[c];
    int moved = 0;
    while (moved < max_moves) {
        int slow = 0, fast = 0;
        for (int k = 1; k < K; ++k) {
            if (rate[k] * (double)L[k] > rate[slow] * (double)L[slow]) slow = k;
            if (rate[k] * (double)L[k] < rate[fast] * (double)L[fast]) fast = k;
        }
        if (slow == fast) break;
        int pick = -1;
        for (int c = 0; c < n_chunks; ++c)
            if (table[c] == slow && (pick < 0 || load[c] <= load[pick])) pick = c;
        if (pick < 0) break;
        const double t_slow = rate[slow] * (double)L[slow], t_fast = rate[fast] * (double)L[fast];
        const double one = rate[fast] * (double)load[pick];
        if (!(t_slow - t_fast > one)) break;
        table[pick] = fast;
        L[slow] -= load[pick];
        L[fast] += load[pick];
        ++moved;
    }
    return moved;
}

}  // namespace chicle
