// Host scan of the missed clusters (TeleRAG Sec. 4.1 step 3) and its thread pool.
// Compiled for x86-64 with AVX2 + FMA + F16C; the loops are plain C++ written so that the
// compiler vectorises them (16 independent partial sums per row).
#include "host_scan.h"

#include <math.h>

#include <cmath>
#include <string.h>

#include <algorithm>
#include <functional>

namespace ivf {

// ---- thread pool -------------------------------------------------------------------------
ThreadPool::ThreadPool(int n) {
    for (int i = 1; i < n; ++i) workers_.emplace_back([this, i] { worker_loop(i); });
}

ThreadPool::~ThreadPool() {
    {
        std::lock_guard<std::mutex> lk(mu_);
        stop_ = true;
    }
    cv_start_.notify_all();
    for (auto& t : workers_) t.join();
}

void ThreadPool::worker_loop(int id) {
    uint64_t seen = 0;
    for (;;) {
        const std::function<void(int, int64_t)>* fn;
        int64_t n;
        {
            std::unique_lock<std::mutex> lk(mu_);
            cv_start_.wait(lk, [&] { return stop_ || generation_ != seen; });
            if (stop_) return;
            seen = generation_;
            fn = fn_;
            n = n_items_;
        }
        for (;;) {
            int64_t i = next_.fetch_add(1, std::memory_order_relaxed);
            if (i >= n) break;
            (*fn)(id, i);
        }
        {
            std::lock_guard<std::mutex> lk(mu_);
            if (--active_ == 0) cv_done_.notify_one();
        }
    }
}

void ThreadPool::run(int64_t n_items, const std::function<void(int, int64_t)>& fn) {
    if (n_items <= 0) return;
    {
        std::lock_guard<std::mutex> lk(mu_);
        fn_ = &fn;
        n_items_ = n_items;
        next_.store(0, std::memory_order_relaxed);
        active_ = (int)workers_.size();
        ++generation_;
    }
    cv_start_.notify_all();
    for (;;) {
        int64_t i = next_.fetch_add(1, std::memory_order_relaxed);
        if (i >= n_items) break;
        fn(0, i);
    }
    std::unique_lock<std::mutex> lk(mu_);
    cv_done_.wait(lk, [&] { return active_ == 0; });
}

// ---- row scoring ---------------------------------------------------------------------------
namespace {

constexpr int kLanes = 16;

inline float load_elem(const float* p, int t) { return p[t]; }
inline float load_elem(const _Float16* p, int t) { return (float)p[t]; }
struct bf16_t { uint16_t bits; };
inline float load_elem(const bf16_t* p, int t) {
    uint32_t u = (uint32_t)p[t].bits << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

// key of one row: inner product, or minus the squared distance (larger = nearer)
template <typename T, int METRIC>
inline float row_key(const float* q, const T* y, int d) {
    float acc[kLanes];
    for (int j = 0; j < kLanes; ++j) acc[j] = 0.f;
    int t = 0;
    for (; t + kLanes <= d; t += kLanes) {
        for (int j = 0; j < kLanes; ++j) {
            float x = load_elem(y, t + j);
            if (METRIC == 0) acc[j] += q[t + j] * x;
            else { float df = q[t + j] - x; acc[j] += df * df; }
        }
    }
    float s = 0.f;
    for (; t < d; ++t) {
        float x = load_elem(y, t);
        if (METRIC == 0) s += q[t] * x;
        else { float df = q[t] - x; s += df * df; }
    }
    for (int j = 0; j < kLanes; ++j) s += acc[j];
    return METRIC == 0 ? s : -s;
}

// fp64 key of one row in the order of operations the device's re-score uses, so that a row
// scanned here and an identical row scanned on the GPU get bit-identical scores: 32
// accumulators; accumulator s takes the 16-byte chunks s, s + 32, ... of the row in that order
// (elements in memory order, one fused multiply-add each; single elements instead of chunks when
// the row is not a whole number of chunks); the accumulators are added by a butterfly over the
// distances 1, 2, 4, 8, 16, of which entry 0 is the result.
template <typename T>
inline double row_key_f64(const float* q, const T* y, int d, int metric) {
    constexpr int kLanes = 32;
    double acc[kLanes];
    for (int s = 0; s < kLanes; ++s) acc[s] = 0.0;
    auto add = [&](double& a, int t) {
        const double x = (double)q[t], v = (double)load_elem(y, t);
        if (metric == 0) a = std::fma(x, v, a);
        else { const double df = x - v; a = std::fma(df, df, a); }
    };
    const int epl = (int)(16 / sizeof(T));
    if (((size_t)d * sizeof(T)) % 16 == 0) {
        const int chunks = d / epl;
        for (int c = 0; c < chunks; ++c)
            for (int e = 0; e < epl; ++e) add(acc[c % kLanes], c * epl + e);
    } else {
        for (int t = 0; t < d; ++t) add(acc[t % kLanes], t);
    }
    for (int o = 1; o < kLanes; o <<= 1) {
        double next[kLanes];
        for (int s = 0; s < kLanes; ++s) next[s] = acc[s] + acc[s ^ o];
        for (int s = 0; s < kLanes; ++s) acc[s] = next[s];
    }
    return metric == 0 ? acc[0] : -acc[0];
}

struct Cand { float key; int64_t id; int64_t row; };

inline bool better(const Cand& a, const Cand& b) {
    return a.key > b.key || (a.key == b.key && a.id < b.id);
}

// the kprime best candidates seen so far, best first
struct LocalTop {
    std::vector<Cand> v;
    int cap = 0;
    float thr = -INFINITY;
    void init(int kprime) { cap = kprime; v.clear(); v.reserve(kprime + 1); thr = -INFINITY; }
    void offer(const Cand& c) {
        if ((int)v.size() == cap && !better(c, v.back())) return;
        auto it = std::upper_bound(v.begin(), v.end(), c, better);
        v.insert(it, c);
        if ((int)v.size() > cap) v.pop_back();
        if ((int)v.size() == cap) thr = v.back().key;
    }
};

template <typename T, int METRIC>
void scan_rows(const HostScanArgs& a, int64_t r0, int64_t r1, LocalTop& top) {
    const T* base = (const T*)a.lists;
    for (int64_t r = r0; r < r1; ++r) {
        float key = row_key<T, METRIC>(a.q, base + (size_t)r * a.d, a.d);
        if (key >= top.thr) top.offer(Cand{key, a.ids ? a.ids[r] : r, r});
    }
}

using ScanFn = void (*)(const HostScanArgs&, int64_t, int64_t, LocalTop&);

ScanFn pick_scan(int dtype, int metric) {
    if (dtype == 0) return metric == 0 ? scan_rows<float, 0> : scan_rows<float, 1>;
    if (dtype == 1) return metric == 0 ? scan_rows<_Float16, 0> : scan_rows<_Float16, 1>;
    return metric == 0 ? scan_rows<bf16_t, 0> : scan_rows<bf16_t, 1>;
}

template <typename T>
float norm_sq_max_rows(const T* base, int64_t r0, int64_t r1, int d) {
    float best = 0.f;
    for (int64_t r = r0; r < r1; ++r) {
        const T* y = base + (size_t)r * d;
        float acc[kLanes];
        for (int j = 0; j < kLanes; ++j) acc[j] = 0.f;
        int t = 0;
        for (; t + kLanes <= d; t += kLanes)
            for (int j = 0; j < kLanes; ++j) { const float x = load_elem(y, t + j); acc[j] += x * x; }
        float s = 0.f;
        for (; t < d; ++t) { const float x = load_elem(y, t); s += x * x; }
        for (int j = 0; j < kLanes; ++j) s += acc[j];
        best = std::max(best, s);
    }
    return best;
}

float norm_sq_max(const void* lists, int dtype, int64_t r0, int64_t r1, int d) {
    if (dtype == 0) return norm_sq_max_rows((const float*)lists, r0, r1, d);
    if (dtype == 1) return norm_sq_max_rows((const _Float16*)lists, r0, r1, d);
    return norm_sq_max_rows((const bf16_t*)lists, r0, r1, d);
}

double key_f64(const HostScanArgs& a, int64_t row) {
    if (a.dtype == 0) return row_key_f64(a.q, (const float*)a.lists + (size_t)row * a.d, a.d, a.metric);
    if (a.dtype == 1) return row_key_f64(a.q, (const _Float16*)a.lists + (size_t)row * a.d, a.d, a.metric);
    return row_key_f64(a.q, (const bf16_t*)a.lists + (size_t)row * a.d, a.d, a.metric);
}

// the kprime best seen so far by (fp64 key, id), best first
struct ExactTop {
    struct E { double key; int64_t id; };
    std::vector<E> v;
    int cap = 0;
    static bool better(const E& x, const E& y) { return x.key > y.key || (x.key == y.key && x.id < y.id); }
    void init(int kprime) { cap = kprime; v.clear(); v.reserve(kprime + 1); }
    void offer(const E& e) {
        if ((int)v.size() == cap && !better(e, v.back())) return;
        v.insert(std::upper_bound(v.begin(), v.end(), e, better), e);
        if ((int)v.size() > cap) v.pop_back();
    }
};

}  // namespace

float host_row_norm_max(const void* lists, int dtype, int64_t n, int d, ThreadPool& pool) {
    if (n <= 0) return 0.f;
    constexpr int64_t kChunk = 4096;
    const int64_t items = (n + kChunk - 1) / kChunk;
    std::vector<float> best(pool.size(), 0.f);
    pool.run(items, [&](int worker, int64_t i) {
        best[worker] = std::max(best[worker], norm_sq_max(lists, dtype, i * kChunk, std::min(n, (i + 1) * kChunk), d));
    });
    float b = 0.f;
    for (float x : best) b = std::max(b, x);
    return std::sqrt(b);
}

int host_scan_query(const HostScanArgs& a, ThreadPool& pool, HostCand* out, uint64_t* rows_scanned, bool* exact_pass) {
    // work items: row chunks of the listed clusters
    constexpr int64_t kChunk = 512;
    struct Item { int64_t r0, r1; };
    std::vector<Item> items;
    uint64_t rows = 0;
    for (int i = 0; i < a.n_clusters; ++i) {
        int64_t lo = a.off[a.clusters[i]], hi = a.off[a.clusters[i] + 1];
        rows += (uint64_t)(hi - lo);
        for (int64_t r = lo; r < hi; r += kChunk) items.push_back(Item{r, std::min(hi, r + kChunk)});
    }
    if (rows_scanned) *rows_scanned = rows;
    if (exact_pass) *exact_pass = false;
    if (items.empty()) return 0;
    std::vector<LocalTop> tops(pool.size());
    for (auto& t : tops) t.init(a.kprime);
    ScanFn fn = pick_scan(a.dtype, a.metric);
    pool.run((int64_t)items.size(), [&](int worker, int64_t i) {
        fn(a, items[i].r0, items[i].r1, tops[worker]);
    });
    LocalTop all;
    all.init(a.kprime);
    for (auto& t : tops)
        for (auto& c : t.v) all.offer(c);
    int m = 0;
    for (auto& c : all.v) {
        out[m].key = key_f64(a, c.row);
        out[m].id = c.id;
        ++m;
    }
    // Is every row of the k nearest among the kprime kept?  A row that was not kept has an fp32 key
    // of at most f_last (the last one kept) and so an exact score of at most f_last + E, E bounding
    // the rounding of the fp32 sums above (inner product: g |q| |y|; squared distance: g times the
    // sum); the k-th best exact score found is a lower bound of the true one.
    if (m == a.kprime && a.k >= 1 && a.k <= m) {
        std::vector<double> keys(m);
        for (int i = 0; i < m; ++i) keys[i] = out[i].key;
        std::nth_element(keys.begin(), keys.begin() + (a.k - 1), keys.end(), std::greater<double>());
        const double s_k = keys[a.k - 1];
        const double f_last = (double)all.v.back().key;
        // roundings on the longest path of a row's sum: a product and an addition per element of a
        // partial sum, then the partial sums and the tail
        const double terms = 2.0 * (a.d / kLanes + 1) + kLanes + 2.0 * (a.d % kLanes) + 4.0;
        const double g = 1.05 * terms * 0x1p-24;
        double e;
        if (a.metric == 0) {
            double qq = 0.0;
            for (int t = 0; t < a.d; ++t) qq += (double)a.q[t] * (double)a.q[t];
            float ymax = a.row_norm_max;
            if (!(ymax > 0.f)) {
                std::vector<float> best(pool.size(), 0.f);
                pool.run((int64_t)items.size(), [&](int worker, int64_t i) {
                    best[worker] = std::max(best[worker], norm_sq_max(a.lists, a.dtype, items[i].r0, items[i].r1, a.d));
                });
                float b = 0.f;
                for (float x : best) b = std::max(b, x);
                ymax = std::sqrt(b) * 1.0001f;
            }
            e = g * std::sqrt(qq) * (double)ymax;
        } else {
            e = g * std::fabs(f_last);
        }
        if (!(s_k > f_last + e)) {
            // exact pass: every row scored in fp64, the kprime best by (score, id) kept
            std::vector<ExactTop> ex(pool.size());
            for (auto& t : ex) t.init(a.kprime);
            pool.run((int64_t)items.size(), [&](int worker, int64_t i) {
                for (int64_t r = items[i].r0; r < items[i].r1; ++r)
                    ex[worker].offer(ExactTop::E{key_f64(a, r), a.ids ? a.ids[r] : r});
            });
            ExactTop fin;
            fin.init(a.kprime);
            for (auto& t : ex)
                for (auto& c : t.v) fin.offer(c);
            m = 0;
            for (auto& c : fin.v) { out[m].key = c.key; out[m].id = c.id; ++m; }
            if (exact_pass) *exact_pass = true;
        }
    }
    return m;
}

}  // namespace ivf
