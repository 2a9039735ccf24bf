// Length-based load balancing before rollout (paper section 3.1.1): a host-side scheduling step, no GPU work.
// Samples are visited by decreasing predicted length (equal lengths by increasing index) and each goes to the
// worker group with the smallest running total that still has room, the lowest group index on equal totals.
#include <algorithm>
#include <new>
#include <numeric>
#include <queue>
#include <utility>
#include <vector>

#include "moe355.h"

extern "C" int moe_balance_lengths(const int64_t* pred_len, int64_t n, int32_t n_groups, int32_t equal_count,
                                   int32_t* group_of, int64_t* order, int64_t* bounds, int64_t* totals) {
    if (n < 0 || n_groups < 1 || !bounds || !totals) return MOE_EINVAL;
    if (n > 0 && (!pred_len || !group_of || !order)) return MOE_EINVAL;
    for (int64_t i = 0; i < n; ++i)
        if (pred_len[i] < 0) return MOE_EINVAL;
    try {
        std::vector<int64_t> visit((size_t)n);
        std::iota(visit.begin(), visit.end(), (int64_t)0);
        std::stable_sort(visit.begin(), visit.end(),
                         [&](int64_t a, int64_t b) { return pred_len[a] > pred_len[b]; });
        // groups with room, smallest (total, index) on top
        using Entry = std::pair<int64_t, int32_t>;
        std::priority_queue<Entry, std::vector<Entry>, std::greater<Entry>> open;
        std::vector<int64_t> room((size_t)n_groups), count((size_t)n_groups, 0);
        for (int32_t g = 0; g < n_groups; ++g) {
            room[g] = equal_count ? n / n_groups + (g < n % n_groups ? 1 : 0) : n;
            totals[g] = 0;
            if (room[g] > 0) open.push({0, g});
        }
        for (int64_t i : visit) {
            const int32_t g = open.top().second;
            open.pop();
            group_of[i] = g;
            totals[g] += pred_len[i];
            if (++count[g] < room[g]) open.push({totals[g], g});
        }
        // list the samples group after group, inside a group in the order they were handed out
        bounds[0] = 0;
        for (int32_t g = 0; g < n_groups; ++g) bounds[g + 1] = bounds[g] + count[g];
        std::vector<int64_t> cursor(bounds, bounds + n_groups);
        for (int64_t i : visit) order[cursor[group_of[i]]++] = i;
    } catch (const std::bad_alloc&) {
        return MOE_ENOMEM;
    }
    return MOE_OK;
}
