// CPU-only driver for the sanitizer builds (address + undefined behaviour, and thread): runs the
// host scan of the missed clusters, the prefetch and cache planners, the prefetch-amount model and
// the grouping of the consolidation moves on seeded inputs and checks them against the CPU oracle, so that every line
// of the host side executes under the sanitizers.  Built by paper_2502_20969_amd/build.py --sanitize.
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <random>
#include <vector>

#include "../../paper_2502_20969_amd/csrc/host_plan.h"
#include "../../paper_2502_20969_amd/csrc/host_scan.h"

extern "C" {
int orc_search_clusters(const void* lists, int dtype, const int64_t* off, const int64_t* ids, int32_t d, int metric,
                        const float* x, const int32_t* clusters, int32_t nclusters, int32_t k, int64_t* out_ids,
                        double* out_scores);
int32_t orc_probe(const float* centroids, int32_t nlist, int32_t d, int metric, const float* x, int32_t L,
                  int32_t* out_clusters, double* out_scores);
int32_t orc_prefetch(const float* centroids, int32_t nlist, int32_t d, int metric, const int64_t* off, int dtype,
                     const float* x_in, int32_t L, uint64_t budget, uint64_t cap, uint8_t* resident, uint64_t* used,
                     int32_t* chosen, int32_t* n_skipped, uint64_t* bytes_taken);
double orc_prefetch_amount(double B, double t_llm, int32_t nprobe, double t_cc, const double* bs, const double* rs,
                           int32_t n, double step, double* t_total);
}

using namespace ivf;

static int g_failed = 0;
#define CHECK(cond, ...) do { if (!(cond)) { printf("FAILED %s:%d: ", __FILE__, __LINE__); printf(__VA_ARGS__); printf("\n"); g_failed = 1; } } while (0)

static uint16_t to_bf16(float f) {
    uint32_t u; memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

static int kprime_of(int k) { int s = k / 8 > 8 ? k / 8 : 8; return k + s > 128 ? 128 : k + s; }

struct Store {
    int64_t n; int d, nlist, dtype;
    std::vector<float> f32; std::vector<uint16_t> b16;
    std::vector<int64_t> off, ids;
    std::vector<float> cent;
    const void* rows() const { return dtype == 0 ? (const void*)f32.data() : (const void*)b16.data(); }
};

static Store make_store(uint32_t seed, int64_t n, int d, int nlist, int dtype, int dup) {
    std::mt19937 rng(seed);
    std::normal_distribution<float> g(0.f, 1.f);
    Store s; s.n = n; s.d = d; s.nlist = nlist; s.dtype = dtype;
    s.cent.resize((size_t)nlist * d);
    for (auto& x : s.cent) x = g(rng);
    std::vector<int64_t> sizes(nlist, n / nlist);
    sizes[0] += n - (n / nlist) * nlist;
    sizes[nlist / 2] += sizes[nlist - 1]; sizes[nlist - 1] = 0;           // one empty list
    s.off.assign(nlist + 1, 0);
    for (int c = 0; c < nlist; ++c) s.off[c + 1] = s.off[c] + sizes[c];
    std::vector<float> rows((size_t)n * d);
    for (int c = 0; c < nlist; ++c)
        for (int64_t r = s.off[c]; r < s.off[c + 1]; ++r) {
            double nn = 0;
            for (int t = 0; t < d; ++t) { float v = s.cent[(size_t)c * d + t] + 0.5f * g(rng); rows[(size_t)r * d + t] = v; nn += (double)v * v; }
            for (int t = 0; t < d; ++t) rows[(size_t)r * d + t] /= (float)sqrt(nn);
        }
    for (int i = 0; i < dup; ++i) {                                          // identical rows, possibly across lists
        int64_t a = rng() % n, b = rng() % n;
        memcpy(&rows[(size_t)b * d], &rows[(size_t)a * d], sizeof(float) * d);
    }
    if (dtype == 0) s.f32 = rows;
    else {
        s.b16.resize(rows.size());
        for (size_t i = 0; i < rows.size(); ++i) {
            if (dtype == 1) { _Float16 h = (_Float16)rows[i]; memcpy(&s.b16[i], &h, 2); }
            else s.b16[i] = to_bf16(rows[i]);
        }
    }
    s.ids.resize(n);
    for (int64_t i = 0; i < n; ++i) s.ids[i] = (n - i) * 3 + 1;               // ids fall as positions grow
    return s;
}

static void check_host_scan(const Store& s, int metric, int k, ThreadPool& pool, uint32_t seed, int* exact_passes) {
    std::mt19937 rng(seed);
    std::normal_distribution<float> g(0.f, 1.f);
    std::vector<float> q(s.d);
    const int c0 = rng() % s.nlist;
    for (int t = 0; t < s.d; ++t) q[t] = s.cent[(size_t)c0 * s.d + t] + 0.3f * g(rng);
    std::vector<int32_t> cl;
    for (int c = 0; c < s.nlist; ++c) if (rng() % 3 != 0) cl.push_back(c);
    const int kp = kprime_of(k);
    std::vector<HostCand> out(kp);
    uint64_t rows = 0; bool exact = false;
    HostScanArgs a{s.rows(), s.off.data(), s.ids.data(), s.d, s.dtype, metric, q.data(), cl.data(), (int)cl.size(), kp, k, 0.f};
    const int m = host_scan_query(a, pool, out.data(), &rows, &exact);
    *exact_passes += exact ? 1 : 0;
    std::vector<int64_t> oi(k); std::vector<double> os(k);
    orc_search_clusters(s.rows(), s.dtype, s.off.data(), s.ids.data(), s.d, metric, q.data(), cl.data(), (int)cl.size(), k, oi.data(), os.data());
    std::sort(out.begin(), out.begin() + m, [](const HostCand& x, const HostCand& y) { return x.key > y.key || (x.key == y.key && x.id < y.id); });
    for (int i = 0; i < k; ++i) {
        if (oi[i] < 0) { CHECK(i >= m, "oracle has %d results, the host scan %d", i, m); break; }
        CHECK(i < m && out[i].id == oi[i], "metric %d dtype %d k %d: result %d is id %lld, the oracle's %lld", metric, s.dtype, k, i,
              i < m ? (long long)out[i].id : -1ll, (long long)oi[i]);
        if (i < m) {
            const double got = metric == 0 ? out[i].key : -out[i].key;
            CHECK(fabs(got - os[i]) <= 1e-9 * fmax(fabs(os[i]), 1e-30) + 1e-300, "score %g vs %g", got, os[i]);
        }
    }
}

static void check_prefetch_plan(const Store& s, uint32_t seed) {
    std::mt19937 rng(seed);
    std::normal_distribution<float> g(0.f, 1.f);
    const int L = 12;
    const size_t rb = (size_t)s.d * (s.dtype == 0 ? 4 : 2);
    const uint64_t total = (uint64_t)s.n * rb, cap = total / 2;
    std::vector<uint8_t> resident(s.nlist, 0);
    uint64_t used = 0;
    std::vector<int64_t> res_off(s.nlist, -1);
    size_t buf_used = 0;
    for (int round = 0; round < 6; ++round) {
        std::vector<float> q(s.d);
        for (auto& x : q) x = g(rng);
        const uint64_t budget = round == 0 ? 0 : (round == 5 ? ~0ull >> 1 : total / (4 + round));
        std::vector<int32_t> ranked(L), chosen(L);
        std::vector<double> sc(L);
        orc_probe(s.cent.data(), s.nlist, s.d, 0, q.data(), L, ranked.data(), sc.data());
        int32_t skipped = 0; uint64_t bytes = 0;
        const int32_t n_chosen = orc_prefetch(s.cent.data(), s.nlist, s.d, 0, s.off.data(), s.dtype, q.data(), L, budget, cap,
                                              resident.data(), &used, chosen.data(), &skipped, &bytes);
        std::vector<int32_t> taken; ivf_prefetch_stats st{};
        plan_prefetch(ranked.data(), 1, L, s.off.data(), rb, (size_t)budget, (size_t)cap, buf_used, res_off.data(), taken, st);
        CHECK((int)taken.size() == n_chosen && st.n_skipped == skipped && st.bytes == bytes && buf_used == used,
              "round %d: %zu taken vs %d, skipped %d vs %d", round, taken.size(), n_chosen, st.n_skipped, skipped);
        for (int i = 0; i < n_chosen && i < (int)taken.size(); ++i) CHECK(taken[i] == chosen[i], "order differs at %d", i);
        for (int c = 0; c < s.nlist; ++c) CHECK((res_off[c] >= 0) == (resident[c] != 0), "residency of %d differs", c);
    }
}

// Eviction + consolidation on a byte buffer: every group of moves is carried out the way one
// launch would (all sources of the group read before any destination is written).
static void check_cache_rounds(uint32_t seed) {
    std::mt19937 rng(seed);
    const int nlist = 60; const size_t rb = 24;
    std::vector<int64_t> off(nlist + 1, 0);
    for (int c = 0; c < nlist; ++c) off[c + 1] = off[c] + (int64_t)(rng() % 40);
    const size_t buf_bytes = (size_t)off[nlist] * rb * 2 / 3;
    std::vector<unsigned char> buf(buf_bytes, 0);
    std::vector<int64_t> res_off(nlist, -1);
    std::vector<float> hot(nlist, -1.f);
    size_t used = 0;
    auto fill = [&](int c) {        // byte pattern of cluster c's rows
        const size_t bytes = (size_t)(off[c + 1] - off[c]) * rb;
        for (size_t i = 0; i < bytes; ++i) buf[(size_t)res_off[c] * rb + i] = (unsigned char)(c * 7 + i * 13);
    };
    for (int round = 0; round < 25; ++round) {
        for (int tries = 0; tries < 30; ++tries) {      // admit random clusters while they fit
            const int c = rng() % nlist;
            const size_t bytes = (size_t)(off[c + 1] - off[c]) * rb;
            if (res_off[c] >= 0 || bytes > buf_bytes - used) continue;
            res_off[c] = (int64_t)(used / rb); used += bytes; hot[c] = (float)(rng() % 5) * 0.5f;
            fill(c);
        }
        std::vector<int32_t> evicted; std::vector<ivf_cache_move> moves; size_t need_tmp = 0; ivf_cache_stats st{};
        const float fraction = (float)(rng() % 5) / 4.f;
        plan_cache_round(hot.data(), off.data(), nlist, rb, res_off.data(), used, buf_bytes, fraction, evicted, moves, need_tmp, st);
        for (const MoveGroup& g : group_moves(moves)) {
            std::vector<std::vector<unsigned char>> held;
            for (size_t m = g.first; m < g.last; ++m) held.emplace_back(buf.begin() + moves[m].from_byte, buf.begin() + moves[m].from_byte + moves[m].bytes);
            for (size_t m = g.first; m < g.last; ++m) std::copy(held[m - g.first].begin(), held[m - g.first].end(), buf.begin() + moves[m].to_byte);
            CHECK(g.through_staging == (moves[g.first].via_staging != 0), "staging flag of a group");
        }
        CHECK(used <= (size_t)((double)fraction * (double)buf_bytes) || st.n_cached == st.n_evicted, "kept bytes above the fraction");
        size_t at = 0;
        std::vector<std::pair<int64_t, int>> order;
        for (int c = 0; c < nlist; ++c) if (res_off[c] >= 0) order.push_back({res_off[c], c});
        std::sort(order.begin(), order.end());
        for (auto& oc : order) {
            const int c = oc.second;
            const size_t bytes = (size_t)(off[c + 1] - off[c]) * rb;
            if (bytes == 0) continue;                      // an empty cluster takes no place
            CHECK((size_t)oc.first * rb == at, "cluster %d not packed", c);
            for (size_t i = 0; i < bytes; ++i)
                if (buf[at + i] != (unsigned char)(c * 7 + i * 13)) { CHECK(false, "round %d: cluster %d damaged at byte %zu", round, c, i); break; }
            at += bytes;
        }
        CHECK(at == used, "buffer mark");
    }
}

// the prefetch amount on random non-increasing miss-rate curves whose points lie on the oracle's grid
static void check_prefetch_amount(uint32_t seed) {
    std::mt19937 rng(seed);
    std::uniform_real_distribution<double> u(0.0, 1.0);
    for (int trial = 0; trial < 40; ++trial) {
        const int n = 1 + (int)(rng() % 12);
        std::vector<double> bs(n), rs(n);
        double b = (double)(rng() % 3) * 1e8, r = 0.3 + 0.7 * u(rng);
        for (int i = 0; i < n; ++i) {
            bs[i] = b; rs[i] = r;
            b += (double)(1 + rng() % 30) * 1e8;
            r *= u(rng) < 0.3 ? 1.0 : u(rng);
        }
        const double bw = (rng() % 2) ? 52e9 : 400e9, t_llm = 0.05 * u(rng), t_cc = 2e-3 * u(rng) * u(rng);
        const int nprobe = 1 + (int)(rng() % 400);
        const PrefetchAmount got = plan_prefetch_amount(bw, t_llm, nprobe, t_cc, bs.data(), rs.data(), n);
        double ot = 0.0;
        const double ob = orc_prefetch_amount(bw, t_llm, nprobe, t_cc, bs.data(), rs.data(), n, 1e7, &ot);
        CHECK(got.amount == ob, "prefetch amount: seed %u trial %d: %.17g, oracle %.17g", seed, trial, got.amount, ob);
        CHECK(fabs(got.seconds - ot) <= 1e-12 * fabs(ot), "prefetch amount: time %.17g, oracle %.17g", got.seconds, ot);
    }
}

int main() {
    int exact = 0;
    {
        ThreadPool pool(6);
        for (int dtype = 0; dtype < 3; ++dtype) {
            Store s = make_store(11 + dtype, 9000, dtype == 0 ? 96 : (dtype == 1 ? 100 : 64), 24, dtype, 40);
            for (int metric = 0; metric < 2; ++metric)
                for (int k : {1, 10, 100})
                    for (int rep = 0; rep < 3; ++rep) check_host_scan(s, metric, k, pool, 100 * dtype + 10 * metric + rep + k, &exact);
            check_prefetch_plan(s, 5 + dtype);
            CHECK(host_row_norm_max(s.rows(), s.dtype, s.n, s.d, pool) > 0.99f, "row norms");
        }
        // many identical rows: the fp32 pass cannot prove its result, the exact pass must run
        Store s = make_store(77, 4000, 128, 8, 0, 0);
        for (int64_t r = 0; r < 600; ++r) memcpy(&s.f32[(size_t)(r * 5) * 128], &s.f32[0], sizeof(float) * 128);
        std::vector<float> q(s.f32.begin(), s.f32.begin() + 128);
        std::vector<int32_t> cl = {0, 1, 2, 3, 4, 5, 6};
        std::vector<HostCand> out(18);
        bool ex = false;
        HostScanArgs a{s.rows(), s.off.data(), s.ids.data(), s.d, 0, 0, q.data(), cl.data(), (int)cl.size(), 18, 10, 0.f};
        const int m = host_scan_query(a, pool, out.data(), nullptr, &ex);
        CHECK(ex && m == 18, "identical rows: exact pass %d, %d candidates", (int)ex, m);
        std::vector<int64_t> oi(10); std::vector<double> os(10);
        orc_search_clusters(s.rows(), 0, s.off.data(), s.ids.data(), s.d, 0, q.data(), cl.data(), (int)cl.size(), 10, oi.data(), os.data());
        std::sort(out.begin(), out.begin() + m, [](const HostCand& x, const HostCand& y) { return x.key > y.key || (x.key == y.key && x.id < y.id); });
        for (int i = 0; i < 10; ++i) CHECK(out[i].id == oi[i], "identical rows: result %d", i);
    }
    for (uint32_t seed = 1; seed <= 8; ++seed) check_cache_rounds(seed);
    for (uint32_t seed = 1; seed <= 4; ++seed) check_prefetch_amount(seed);
    printf("%s (%d exact passes of the host scan)\n", g_failed ? "FAILED" : "host sanitizer driver ok", exact);
    return g_failed;
}
