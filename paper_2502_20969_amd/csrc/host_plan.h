// Host-side planning of the lookahead path: pure functions over plain arrays (no GPU, no HIP
// headers), shared by the C entry points, which run them next to the device work, and by the
// stage-level entry points and the sanitizer build, which run them on their own.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "../../include/ivf.h"

namespace ivf {

// The budget walk of one prefetch call (Sec. 4.3 "Prefetching target"; several queries: Sec. 4.2
// "Batching"): res_off (row offset in the buffer or -1) and buf_used are updated, `taken` lists
// the clusters to copy, in order.
void plan_prefetch(const int32_t* ranked, int nq, int nprobe, const int64_t* off, size_t row_bytes,
                   size_t budget_bytes, size_t buf_bytes, size_t& buf_used, int64_t* res_off,
                   std::vector<int32_t>& taken, ivf_prefetch_stats& st);

// How much to prefetch (App. C "Finding Prefetching Amount"): the byte budget that minimises
// t_1 + t_2 for a measured miss-rate curve (n points, budgets increasing, linear between the points,
// constant outside).  t_1 + t_2 is piecewise linear in the budget, with corners at bandwidth * t_llm
// and at the measured points, and cannot fall below bandwidth * t_llm while the miss rate does not
// rise: only that amount (case 1) and the measured points beyond it (case 2) are looked at.
struct PrefetchAmount { double amount, seconds; int which; };
PrefetchAmount plan_prefetch_amount(double bandwidth, double t_llm, int nprobe, double t_cc,
                                    const double* budgets, const double* miss_rates, int n);

// Eviction and consolidation of a cache round (Sec. 4.2 "Cache design"), after the hotness update.
void plan_cache_round(float* hot, const int64_t* off, int nlist, size_t rb, int64_t* res_off,
                      size_t& buf_used, size_t buf_bytes, float fraction, std::vector<int32_t>& evicted,
                      std::vector<ivf_cache_move>& moves, size_t& need_tmp, ivf_cache_stats& st);

// Groups of consecutive moves that one launch can carry out together: no destination of a group
// overlaps a source of the group (all moves go towards lower addresses, so a group ends where the
// next destination would reach the group's first source).  A move that overlaps its own old place
// is a group of its own (through_staging).
struct MoveGroup { size_t first, last; bool through_staging; };
std::vector<MoveGroup> group_moves(const std::vector<ivf_cache_move>& moves);

}  // namespace ivf
