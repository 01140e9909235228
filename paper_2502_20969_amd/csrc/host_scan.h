// Host side of the hybrid search (TeleRAG Sec. 4.1 step 3: the clusters of q_out that were not
// prefetched are searched by CPU threads while the GPU searches the resident ones).
#pragma once
#include <stdint.h>

#include <atomic>
#include <condition_variable>
#include <functional>
#include <mutex>
#include <thread>
#include <vector>

#include "ivf_host_types.h"

namespace ivf {

// A fixed set of worker threads that run one indexed job at a time.
class ThreadPool {
public:
    explicit ThreadPool(int n);
    ~ThreadPool();
    int size() const { return (int)workers_.size() + 1; }
    // Calls fn(worker, item) for item in [0, n_items), items handed out dynamically; the calling
    // thread takes part as worker 0.  Returns when every item is done.
    void run(int64_t n_items, const std::function<void(int, int64_t)>& fn);

private:
    void worker_loop(int id);
    std::vector<std::thread> workers_;
    std::mutex mu_;
    std::condition_variable cv_start_, cv_done_;
    const std::function<void(int, int64_t)>* fn_ = nullptr;
    std::atomic<int64_t> next_{0};
    int64_t n_items_ = 0;
    uint64_t generation_ = 0;
    int active_ = 0;
    bool stop_ = false;
};

struct HostScanArgs {
    const void* lists;      // cluster-major rows in host memory
    const int64_t* off;     // [nlist+1]
    const int64_t* ids;     // [n] or nullptr
    int d, dtype, metric;
    const float* q;         // [d]
    const int32_t* clusters;  // lists to scan
    int n_clusters;
    int kprime;
    int k;                  // results wanted (k <= kprime)
    float row_norm_max;     // an upper bound of the Euclidean norm of the rows; <= 0: measured over the listed clusters
};

// Scans the listed clusters for one query: fp32 accumulation over all rows, the kprime best kept
// per thread, their union cut to kprime and re-scored in fp64.  When the fp32 rounding could have
// kept a row of the k nearest out of those kprime (the k-th fp64 score found is within the rounding
// bound of the last fp32 score kept), the clusters are scanned again in fp64 and the exact kprime
// best by (score, id) are returned instead (*exact_pass, nullable, tells).  Writes up to kprime
// candidates (unordered) to out and returns how many.  *rows_scanned receives the rows covered.
int host_scan_query(const HostScanArgs& a, ThreadPool& pool, HostCand* out, uint64_t* rows_scanned,
                    bool* exact_pass = nullptr);

// The largest Euclidean norm over n stored rows (fp32 sums), with the pool's threads.
float host_row_norm_max(const void* lists, int dtype, int64_t n, int d, ThreadPool& pool);

}  // namespace ivf
