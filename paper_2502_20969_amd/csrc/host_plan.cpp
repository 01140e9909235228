// Host-side planning of the lookahead path (see host_plan.h).
#include "host_plan.h"

#include <algorithm>
#include <utility>

namespace ivf {

// The plan of one prefetch call (Sec. 4.3 "Prefetching target"; several queries: Sec. 4.2 "Batching"):
// every query gets an equal share of the budget and walks its ranked clusters nearest first; a
// cluster that is resident (also: taken for an earlier query of the call) costs nothing, one that
// fits the query's remaining share and the remaining buffer is taken whole at the buffer's fill
// mark, any other is skipped and the walk goes on.  Pure host arithmetic: res_off (row offset in
// the buffer or -1) and buf_used are updated, `taken` lists the clusters to copy, in order.
void plan_prefetch(const int32_t* ranked, int nq, int nprobe, const int64_t* off, size_t row_bytes,
                          size_t budget_bytes, size_t buf_bytes, size_t& buf_used, int64_t* res_off,
                          std::vector<int32_t>& taken, ivf_prefetch_stats& st) {
    const size_t per_query = budget_bytes / (size_t)nq;
    for (int qi = 0; qi < nq; ++qi) {
        size_t remaining = per_query;
        for (int i = 0; i < nprobe; ++i) {
            const int32_t c = ranked[(size_t)qi * nprobe + i];
            st.n_ranked += 1;
            if (res_off[c] >= 0) { st.n_resident += 1; continue; }
            const size_t bytes = (size_t)(off[c + 1] - off[c]) * row_bytes;
            if (bytes <= remaining && bytes <= buf_bytes - buf_used) {
                res_off[c] = (int64_t)(buf_used / row_bytes);
                buf_used += bytes;
                remaining -= bytes;
                st.bytes += bytes;
                st.n_taken += 1;
                taken.push_back(c);
            } else {
                st.n_skipped += 1;
            }
        }
    }
    st.buffer_used = buf_used;
}

// The host part of a cache round (Sec. 4.2 "Cache design"), after the hotness update.
// Eviction: while the cached bytes exceed fraction x buffer, the cached cluster of lowest hotness
// leaves (equal hotness: the larger index first); its hotness becomes -1.  Consolidation: the
// survivors move to the front of the buffer in their current order.  A cluster only ever moves
// towards lower addresses and never onto a later cluster's old place; it can overlap its own old
// place, and then goes through a staging buffer (need_tmp: the largest such cluster).
void plan_cache_round(float* hot, const int64_t* off, int nlist, size_t rb, int64_t* res_off,
                             size_t& buf_used, size_t buf_bytes, float fraction, std::vector<int32_t>& evicted,
                             std::vector<ivf_cache_move>& moves, size_t& need_tmp, ivf_cache_stats& st) {
    struct Item { float h; int32_t c; };
    std::vector<Item> cached;
    for (int c = 0; c < nlist; ++c)
        if (res_off[c] >= 0) cached.push_back(Item{hot[c], (int32_t)c});
    st.n_cached = (int32_t)cached.size();
    st.bytes_cached = buf_used;
    const uint64_t limit = (uint64_t)((double)fraction * (double)buf_bytes);
    std::sort(cached.begin(), cached.end(), [](const Item& x, const Item& y) {
        return x.h < y.h || (x.h == y.h && x.c > y.c);
    });
    uint64_t in_use = buf_used;
    for (size_t i = 0; i < cached.size() && in_use > limit; ++i) {
        const int c = cached[i].c;
        in_use -= (uint64_t)(off[c + 1] - off[c]) * rb;
        res_off[c] = -1;
        hot[c] = -1.f;
        st.n_evicted += 1;
        evicted.push_back(c);
    }
    std::vector<std::pair<int64_t, int32_t>> order;
    for (int c = 0; c < nlist; ++c)
        if (res_off[c] >= 0) order.push_back({res_off[c], (int32_t)c});
    std::sort(order.begin(), order.end());
    need_tmp = 0;
    uint64_t at = 0;
    for (auto& oc : order) {
        const int c = oc.second;
        const uint64_t bytes = (uint64_t)(off[c + 1] - off[c]) * rb, old = (uint64_t)oc.first * rb;
        if (old != at && bytes > 0) {
            const bool overlap = old - at < bytes;
            if (overlap) need_tmp = std::max<size_t>(need_tmp, bytes);
            moves.push_back(ivf_cache_move{(int32_t)c, overlap ? 1 : 0, old, at, bytes});
            st.bytes_moved += bytes;
        }
        res_off[c] = (int64_t)(at / rb);
        at += bytes;
    }
    buf_used = at;
}

std::vector<MoveGroup> group_moves(const std::vector<ivf_cache_move>& moves) {
    std::vector<MoveGroup> groups;
    for (size_t g0 = 0; g0 < moves.size();) {
        if (moves[g0].via_staging) { groups.push_back(MoveGroup{g0, g0 + 1, true}); g0 += 1; continue; }
        const uint64_t first_src = moves[g0].from_byte;
        size_t g1 = g0;
        // the first move of a group always fits (it does not overlap itself), so the group is not empty
        while (g1 < moves.size() && !moves[g1].via_staging && moves[g1].to_byte + moves[g1].bytes <= first_src) ++g1;
        groups.push_back(MoveGroup{g0, g1, false});
        g0 = g1;
    }
    return groups;
}

PrefetchAmount plan_prefetch_amount(double bandwidth, double t_llm, int nprobe, double t_cc,
                                    const double* budgets, const double* miss_rates, int n) {
    const double window = bandwidth * t_llm;            // what the link moves while the generation runs
    const double per_miss = (double)nprobe * t_cc;      // host seconds if every selected cluster were missed
    // miss rate at the window: between two measured points, or the first / last one outside them
    double r = miss_rates[n - 1];
    if (window <= budgets[0]) r = miss_rates[0];
    else {
        for (int i = 1; i < n; ++i) {
            if (window <= budgets[i]) {
                const double x = (window - budgets[i - 1]) / (budgets[i] - budgets[i - 1]);
                r = x >= 1.0 ? miss_rates[i] : miss_rates[i - 1] + (miss_rates[i] - miss_rates[i - 1]) * x;
                break;
            }
        }
    }
    PrefetchAmount best{window, t_llm + r * per_miss, 1};
    for (int i = 0; i < n; ++i) {
        if (budgets[i] <= window) continue;
        const double t = budgets[i] / bandwidth + miss_rates[i] * per_miss;
        if (t < best.seconds) best = PrefetchAmount{budgets[i], t, 2};       // of equal points the first, nearest to the window
    }
    return best;
}

}  // namespace ivf
