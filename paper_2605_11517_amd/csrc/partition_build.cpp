// Host-side construction of the partition metadata: assignment rules, library vertex order,
// boundary lists, per-partition local topology T_p and its transpose, normalisation factors.
//
// Paper passages this follows:
//   - a partition's input GA_p is the union of the sources of its destinations
//     (Cache-(Re)Gather-Bypass section, "(Re)gather");
//   - neighbours are ordered by partition id, then vertex id, so that a gather touches each
//     source partition as one ascending run (appendix "In-Partition Vertex Ordering for
//     Sequential Accesses");
//   - label propagation towards the partition holding most neighbours, with the size penalty
//     |P_j| / (1.1 |V| / k) and a capacity limit per partition (partitioning section and its
//     appendix).
#include <algorithm>
#include <atomic>
#include <cstdio>
#include <chrono>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <new>
#include <thread>

#include "gnn_internal.h"

namespace gnnmi {
namespace {

int worker_count()
{
    int t = (int)std::thread::hardware_concurrency();
    if (const char* e = std::getenv("GNNMI_THREADS")) t = std::atoi(e);
    return std::max(1, std::min(t, 16));
}

// Calls fn(tid, index) for every index in [0, count), handing out chunks dynamically.
void parallel_for(int64_t count, int64_t chunk, const std::function<void(int, int64_t)>& fn)
{
    int nt = (int)std::min<int64_t>(worker_count(), std::max<int64_t>(1, (count + chunk - 1) / chunk));
    if (nt <= 1) {
        for (int64_t i = 0; i < count; ++i) fn(0, i);
        return;
    }
    std::atomic<int64_t> next{0};
    std::atomic<int> failed{0};  // an allocation failure in a worker is re-raised by the caller
    std::vector<std::thread> pool;
    for (int t = 0; t < nt; ++t)
        pool.emplace_back([&, t] {
            try {
                for (;;) {
                    int64_t lo = next.fetch_add(chunk);
                    if (lo >= count || failed.load(std::memory_order_relaxed)) break;
                    int64_t hi = std::min(count, lo + chunk);
                    for (int64_t i = lo; i < hi; ++i) fn(t, i);
                }
            } catch (...) {
                failed.store(1);
            }
        });
    for (auto& th : pool) th.join();
    if (failed.load()) throw std::bad_alloc();
}

inline uint64_t splitmix64(uint64_t x)
{
    uint64_t z = x + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Rank vertices by (hash, id); rank r goes to partition r mod k.
void assign_random(int64_t n, int32_t k, uint64_t seed, std::vector<int32_t>& part)
{
    std::vector<std::pair<uint64_t, int32_t>> keys((size_t)n);
    parallel_for(n, 1 << 16, [&](int, int64_t v) {
        keys[(size_t)v] = {splitmix64(seed ^ splitmix64((uint64_t)v)), (int32_t)v};
    });
    std::sort(keys.begin(), keys.end());
    part.resize((size_t)n);
    for (int64_t r = 0; r < n; ++r) part[(size_t)keys[(size_t)r].second] = (int32_t)(r % k);
}

// One synchronous label-propagation round: targets from the frozen state, then an ascending
// sweep that honours the capacity at the moment of each move.
void lp_round(int64_t n, const int64_t* rowptr, const int32_t* colidx, int32_t k,
              std::vector<int32_t>& part)
{
    std::vector<int64_t> sizes((size_t)k, 0);
    for (int64_t v = 0; v < n; ++v) sizes[(size_t)part[(size_t)v]]++;
    // smallest partition, lowest id among equals: the best of all partitions holding no
    // neighbour of a vertex
    int32_t jmin = 0;
    for (int32_t j = 1; j < k; ++j)
        if (sizes[(size_t)j] < sizes[(size_t)jmin]) jmin = j;

    std::vector<int32_t> target((size_t)n);
    int nt = worker_count();
    std::vector<std::vector<int64_t>> cnt((size_t)nt, std::vector<int64_t>((size_t)k, 0));
    std::vector<std::vector<int32_t>> touched((size_t)nt);
    parallel_for(n, 4096, [&](int tid, int64_t v) {
        auto& c = cnt[(size_t)tid];
        auto& tl = touched[(size_t)tid];
        tl.clear();
        int64_t deg = 0;
        for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
            int32_t u = colidx[e];
            if (u == v) continue;
            int32_t j = part[(size_t)u];
            if (c[(size_t)j]++ == 0) tl.push_back(j);
            ++deg;
        }
        int32_t cur = part[(size_t)v];
        auto key = [&](int32_t j) {
            return (int64_t)11 * n * c[(size_t)j] - (int64_t)10 * k * deg * sizes[(size_t)j];
        };
        int64_t best = key(jmin);
        int32_t arg = jmin;
        for (int32_t j : tl) {
            int64_t kj = key(j);
            if (kj > best || (kj == best && j < arg)) {
                best = kj;
                arg = j;
            }
        }
        if (key(cur) == best) arg = cur;
        target[(size_t)v] = arg;
        for (int32_t j : tl) c[(size_t)j] = 0;
    });

    const int64_t cap = ((int64_t)11 * n) / ((int64_t)10 * k);
    for (int64_t v = 0; v < n; ++v) {
        int32_t j = target[(size_t)v], cur = part[(size_t)v];
        if (j != cur && sizes[(size_t)j] < cap) {
            sizes[(size_t)cur]--;
            sizes[(size_t)j]++;
            part[(size_t)v] = j;
        }
    }
}

// ---- the complete switching-aware partitioner (partitioning section; appendix with its
// insights and details) ------------------------------------------------------------------
//
// One iteration, from the frozen state S_i:
//   1. source-level parallelism: every vertex ranks the partitions that occur among its
//      neighbours, plus its own, by the score 1 + #N(v,j)/#N(v,.) - |P_j|/(1.1 |V|/k) (as the
//      exact integer key 11 |V| #N(v,j) - 10 k #N(v,.) |P_j|; equal keys: own partition first,
//      then the lower id) and keeps the first and the second preference;
//   2. the vertices are split into kSwitchingWorkers contiguous ranges.  Each range keeps, per
//      partition j, its candidates (first preference j, currently elsewhere), groups them by
//      second preference and relocates the largest group (ties: lower second preference, "none"
//      lowest) in ascending vertex id, at most its share of the relocation capacity
//      RC_j = floor(1.1 |V|/k) - |P_j| (equal split, remainder to the first ranges);
//   3. the objective sum_v Score(v, partition_v) of the new state is evaluated exactly (scaled
//      by 11 |V| 2^20, neighbour fraction rounded down to 20 bits); the loop halts when it has
//      improved by less than 0.1 % of its previous value in 5 consecutive iterations, or after
//      50 iterations.
// The number of ranges is a constant of the rule, not the number of threads, so the result
// does not depend on the machine.  The paper's "Dst's Partition" mirror of the adjacency is
// not materialised: the assignment array it would cache is itself cache-resident here.
constexpr int32_t kSwitchingWorkers = 16;
constexpr int32_t kSwitchingMaxIters = 50;
constexpr int32_t kSwitchingWindow = 5;
constexpr int64_t kFracOne = 1 << 20;

struct SwitchingInfo {
    int32_t iterations = 0;
    std::vector<double> objective;   // mean score per vertex, initial state first
};

// Device buffers of the device variant of step 1; freed on every path out of the partitioner.
struct PrefDevice {
    int64_t* rowptr = nullptr;
    int32_t* colidx = nullptr;
    int32_t *part = nullptr, *first = nullptr, *second = nullptr;
    int64_t* sizes = nullptr;
    unsigned long long* frac = nullptr;
    // pinned host mirrors of the three per-vertex arrays that cross the link every iteration
    int32_t *host_part = nullptr, *host_first = nullptr, *host_second = nullptr;
    ~PrefDevice()
    {
        for (void* p : {(void*)rowptr, (void*)colidx, (void*)part, (void*)first, (void*)second,
                        (void*)sizes, (void*)frac})
            if (p) (void)hipFree(p);
        for (void* p : {(void*)host_part, (void*)host_first, (void*)host_second})
            if (p) (void)hipHostFree(p);
    }
};
struct HipFailure {
    std::string what;
};
#define PART_HIP(call)                                                                       \
    do {                                                                                     \
        hipError_t e_ = (call);                                                              \
        if (e_ != hipSuccess) {                                                              \
            (void)hipGetLastError();                                                         \
            throw HipFailure{std::string(#call) + ": " + hipGetErrorString(e_)};             \
        }                                                                                    \
    } while (0)

void assign_switching(int64_t n, const int64_t* rowptr, const int32_t* colidx, int32_t k,
                      uint64_t seed, bool on_device, std::vector<int32_t>& part, SwitchingInfo& info)
{
    assign_random(n, k, seed, part);
    PrefDevice D;
    if (on_device) {
        const int64_t nnz = rowptr[n];
        PART_HIP(hipMalloc((void**)&D.rowptr, (size_t)(n + 1) * 8));
        PART_HIP(hipMalloc((void**)&D.colidx, (size_t)std::max<int64_t>(1, nnz) * 4));
        PART_HIP(hipMalloc((void**)&D.part, (size_t)n * 4));
        PART_HIP(hipMalloc((void**)&D.first, (size_t)n * 4));
        PART_HIP(hipMalloc((void**)&D.second, (size_t)n * 4));
        PART_HIP(hipMalloc((void**)&D.sizes, (size_t)k * 8));
        PART_HIP(hipMalloc((void**)&D.frac, 8));
        const size_t vbytes = (size_t)std::max<int64_t>(1, n) * 4;
        PART_HIP(hipHostMalloc((void**)&D.host_part, vbytes, hipHostMallocDefault));
        PART_HIP(hipHostMalloc((void**)&D.host_first, vbytes, hipHostMallocDefault));
        PART_HIP(hipHostMalloc((void**)&D.host_second, vbytes, hipHostMallocDefault));
        PART_HIP(hipMemcpy(D.rowptr, rowptr, (size_t)(n + 1) * 8, hipMemcpyHostToDevice));
        if (nnz > 0) PART_HIP(hipMemcpy(D.colidx, colidx, (size_t)nnz * 4, hipMemcpyHostToDevice));
    }
    const int nt = worker_count();
    const int64_t cap = ((int64_t)11 * n) / ((int64_t)10 * k);
    // preferences of every vertex: pinned when the device writes them, plain vectors otherwise
    std::vector<int32_t> first_store((size_t)(on_device ? 0 : n)), second_store((size_t)(on_device ? 0 : n));
    int32_t* const first = on_device ? D.host_first : first_store.data();
    int32_t* const second = on_device ? D.host_second : second_store.data();
    if (on_device)
        parallel_for(n, 1 << 16, [&](int, int64_t v) { D.host_part[v] = part[(size_t)v]; });
    std::vector<int64_t> sizes((size_t)k);
    std::vector<std::vector<int64_t>> cnt((size_t)nt, std::vector<int64_t>((size_t)k, 0));
    std::vector<std::vector<int32_t>> touched((size_t)nt);
    constexpr int64_t kChunk = 4096;
    const int64_t nchunks = (n + kChunk - 1) / kChunk;
    std::vector<int64_t> frac_sum((size_t)nchunks);
    struct Cand { int32_t first, second, v; };
    std::vector<std::vector<Cand>> cands((size_t)kSwitchingWorkers);
    __int128 prev_q = 0;
    int32_t streak = 0;

    // GNNMI_PART_TIMING=1: seconds spent per phase, summed over the iterations, on stderr
    const bool timing = std::getenv("GNNMI_PART_TIMING") && std::atoi(std::getenv("GNNMI_PART_TIMING")) != 0;
    double t_sizes = 0, t_pref = 0, t_select = 0, t_apply = 0;
    auto now = [] { return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count(); };
    struct Report {
        const bool on; const double &a, &b, &c, &d; const SwitchingInfo& info;
        ~Report()
        {
            if (on)
                std::fprintf(stderr, "switching partitioner: %d iterations; sizes %.3f s, preferences %.3f s, "
                                     "selection %.3f s, moves %.3f s\n", info.iterations, a, b, c, d);
        }
    } report{timing, t_sizes, t_pref, t_select, t_apply, info};

    for (int32_t it = 0;; ++it) {
        double t0 = now();
        std::fill(sizes.begin(), sizes.end(), 0);
        if ((int64_t)k <= 4096 && n >= ((int64_t)1 << 20)) {
            std::vector<std::vector<int64_t>> part_sizes((size_t)nt, std::vector<int64_t>((size_t)k, 0));
            parallel_for(nchunks, 16, [&](int tid, int64_t ch) {
                auto& ps = part_sizes[(size_t)tid];
                const int64_t hi = std::min(n, (ch + 1) * kChunk);
                for (int64_t v = ch * kChunk; v < hi; ++v) ps[(size_t)part[(size_t)v]]++;
            });
            for (auto& ps : part_sizes)
                for (int32_t j = 0; j < k; ++j) sizes[(size_t)j] += ps[(size_t)j];
        } else {
            for (int64_t v = 0; v < n; ++v) sizes[(size_t)part[(size_t)v]]++;
        }
        t_sizes += now() - t0;
        t0 = now();
        // step 1 on the current state, together with the objective of that state
        unsigned long long device_frac = 0;
        if (on_device) {
            PART_HIP(hipMemcpy(D.part, D.host_part, (size_t)n * 4, hipMemcpyHostToDevice));
            PART_HIP(hipMemcpy(D.sizes, sizes.data(), (size_t)k * 8, hipMemcpyHostToDevice));
            PART_HIP(hipMemset(D.frac, 0, 8));
            launch_switch_pref(n, D.rowptr, D.colidx, D.part, D.sizes, k, D.first, D.second, D.frac, nullptr);
            PART_HIP(hipGetLastError());
            PART_HIP(hipMemcpy(first, D.first, (size_t)n * 4, hipMemcpyDeviceToHost));
            PART_HIP(hipMemcpy(second, D.second, (size_t)n * 4, hipMemcpyDeviceToHost));
            PART_HIP(hipMemcpy(&device_frac, D.frac, 8, hipMemcpyDeviceToHost));
            std::fill(frac_sum.begin(), frac_sum.end(), 0);
        } else {
        parallel_for(nchunks, 1, [&](int tid, int64_t ch) {
            auto& c = cnt[(size_t)tid];
            auto& tl = touched[(size_t)tid];
            int64_t fsum = 0;
            const int64_t hi = std::min(n, (ch + 1) * kChunk);
            for (int64_t v = ch * kChunk; v < hi; ++v) {
                tl.clear();
                int64_t deg = 0;
                for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
                    const int32_t u = colidx[e];
                    if (u == v) continue;
                    const int32_t j = part[(size_t)u];
                    if (c[(size_t)j]++ == 0) tl.push_back(j);
                    ++deg;
                }
                const int32_t cur = part[(size_t)v];
                if (deg > 0) fsum += kFracOne * c[(size_t)cur] / deg;
                if (c[(size_t)cur] == 0) tl.push_back(cur);
                auto key = [&](int32_t j) {
                    return (int64_t)11 * n * c[(size_t)j] - (int64_t)10 * k * deg * sizes[(size_t)j];
                };
                // better(a, b): a ranks before b
                auto better = [&](int32_t a, int64_t ka, int32_t b, int64_t kb) {
                    if (ka != kb) return ka > kb;
                    if ((a == cur) != (b == cur)) return a == cur;
                    return a < b;
                };
                int32_t b1 = -1, b2 = -1;
                int64_t k1 = 0, k2 = 0;
                for (int32_t j : tl) {
                    const int64_t kj = key(j);
                    if (b1 < 0 || better(j, kj, b1, k1)) {
                        b2 = b1; k2 = k1;
                        b1 = j; k1 = kj;
                    } else if (b2 < 0 || better(j, kj, b2, k2)) {
                        b2 = j; k2 = kj;
                    }
                }
                first[(size_t)v] = b1;
                second[(size_t)v] = b2;
                for (int32_t j : tl) c[(size_t)j] = 0;
            }
            frac_sum[(size_t)ch] = fsum;
        });
        }
        t_pref += now() - t0;
        t0 = now();
        __int128 total = (__int128)n * kFracOne + device_frac;
        for (int64_t ch = 0; ch < nchunks; ++ch) total += frac_sum[(size_t)ch];
        __int128 sq = 0;
        for (int32_t j = 0; j < k; ++j) sq += (__int128)sizes[(size_t)j] * sizes[(size_t)j];
        const __int128 q = (__int128)11 * n * total - (__int128)10 * k * kFracOne * sq;
        info.objective.push_back((double)q / ((double)11 * (double)n * (double)kFracOne * (double)n));
        if (it > 0) {
            const __int128 mag = prev_q < 0 ? -prev_q : prev_q;
            const bool small = (__int128)1000 * (q - prev_q) < mag;
            streak = small ? streak + 1 : 0;
        }
        prev_q = q;
        info.iterations = it;
        if (streak == kSwitchingWindow || it == kSwitchingMaxIters) break;

        // step 2: per range, per target partition, the largest second-preference group moves
        std::atomic<int64_t> moved{0};
        // Group sizes come from a (first, second) histogram per range when k is small enough for
        // one (k x (k + 1) counters per range); otherwise the candidates are sorted.  Both pick
        // the same group and the same vertices.
        const char* force_sort = std::getenv("GNNMI_SWITCH_SORT");
        const bool by_histogram = (int64_t)k * (k + 1) <= ((int64_t)1 << 20) &&
                                  !(force_sort && std::atoi(force_sort) != 0);
        parallel_for(kSwitchingWorkers, 1, [&](int, int64_t w) {
            const int64_t lo = (w * n) / kSwitchingWorkers, hi = ((w + 1) * n) / kSwitchingWorkers;
            auto room_of = [&](int32_t j) {
                const int64_t rc = std::max<int64_t>(0, cap - sizes[(size_t)j]);
                return rc / kSwitchingWorkers + (w < rc % kSwitchingWorkers ? 1 : 0);
            };
            int64_t local_moved = 0;
            if (by_histogram) {
                const int64_t k1 = (int64_t)k + 1;                 // second preference -1 ("none") .. k-1
                std::vector<int64_t> hist((size_t)(k * k1), 0);
                for (int64_t v = lo; v < hi; ++v)
                    if (first[(size_t)v] != part[(size_t)v])
                        ++hist[(size_t)(first[(size_t)v] * k1 + second[(size_t)v] + 1)];
                std::vector<int32_t> chosen((size_t)k, -3);        // second preference of the moving group
                std::vector<int64_t> take((size_t)k, 0);
                for (int32_t j = 0; j < k; ++j) {
                    int64_t best_len = 0;
                    int32_t best_second = -3;
                    for (int64_t t = 0; t < k1; ++t)                 // ascending second: first wins ties
                        if (hist[(size_t)(j * k1 + t)] > best_len) {
                            best_len = hist[(size_t)(j * k1 + t)];
                            best_second = (int32_t)t - 1;
                        }
                    chosen[(size_t)j] = best_second;
                    take[(size_t)j] = std::min(best_len, room_of(j));
                }
                // first[] of a mover is its new home; the assignment itself changes below
                for (int64_t v = lo; v < hi; ++v) {
                    const int32_t j = first[(size_t)v];
                    if (j == part[(size_t)v] || second[(size_t)v] != chosen[(size_t)j] || take[(size_t)j] == 0)
                        continue;
                    second[(size_t)v] = -2;
                    --take[(size_t)j];
                    ++local_moved;
                }
                moved += local_moved;
                return;
            }
            auto& L = cands[(size_t)w];
            L.clear();
            for (int64_t v = lo; v < hi; ++v)
                if (first[(size_t)v] != part[(size_t)v])
                    L.push_back({first[(size_t)v], second[(size_t)v], (int32_t)v});
            std::sort(L.begin(), L.end(), [](const Cand& a, const Cand& b) {
                if (a.first != b.first) return a.first < b.first;
                if (a.second != b.second) return a.second < b.second;
                return a.v < b.v;
            });
            size_t i = 0;
            while (i < L.size()) {
                const int32_t j = L[i].first;
                size_t best_lo = i, best_len = 0;
                size_t g = i;
                while (g < L.size() && L[g].first == j) {
                    size_t e = g;
                    while (e < L.size() && L[e].first == j && L[e].second == L[g].second) ++e;
                    if (e - g > best_len) { best_len = e - g; best_lo = g; }   // ascending second: first wins ties
                    g = e;
                }
                const size_t take = (size_t)std::min<int64_t>((int64_t)best_len, room_of(j));
                // first[] of a mover is its new home; the assignment itself changes below
                for (size_t t = best_lo; t < best_lo + take; ++t) second[(size_t)L[t].v] = -2;
                local_moved += (int64_t)take;
                i = g;
            }
            moved += local_moved;
        });
        t_select += now() - t0;
        t0 = now();
        if (moved.load() == 0) break;   // a fixed point: every further iteration repeats it
        parallel_for(n, 1 << 16, [&](int, int64_t v) {
            if (second[(size_t)v] == -2) {
                part[(size_t)v] = first[(size_t)v];
                if (on_device) D.host_part[v] = first[(size_t)v];
            }
        });
        t_apply += now() - t0;
    }
}

// Cuts the rows [0, nrows) of one partition (row pointers rp[0..nrows], absolute positions)
// into work items: rows longer than kSpmmSegment become segments of that many entries; the
// others are grouped into consecutive ranges holding at most kSpmmSegment entries and
// kSpmmRangeRows rows (a long row closes the range before it and is skipped by range items).
struct PlanPart {
    std::vector<int32_t> range_rows, seg_row, seg_len, long_row, long_first, long_nseg, rows_sorted;
    std::vector<int64_t> seg_begin;
};
void plan_partition(const int64_t* rp, int64_t nrows, PlanPart& P)
{
    P.range_rows.push_back(0);
    int64_t acc = 0;
    int32_t start = 0;
    for (int64_t r = 0; r < nrows; ++r) {
        const int64_t deg = rp[r + 1] - rp[r];
        if (deg > kSpmmSegment) {
            P.long_row.push_back((int32_t)r);
            P.long_first.push_back((int32_t)P.seg_row.size());
            int32_t ns = 0;
            for (int64_t e = rp[r]; e < rp[r + 1]; e += kSpmmSegment) {
                P.seg_row.push_back((int32_t)r);
                P.seg_begin.push_back(e);
                P.seg_len.push_back((int32_t)std::min<int64_t>(kSpmmSegment, rp[r + 1] - e));
                ++ns;
            }
            P.long_nseg.push_back(ns);
            continue;  // costs a range nothing
        }
        if (r > start && (acc + deg > kSpmmSegment || r - start >= kSpmmRangeRows)) {
            P.range_rows.push_back((int32_t)r);
            start = (int32_t)r;
            acc = 0;
        }
        acc += deg;
    }
    if (nrows > start) P.range_rows.push_back((int32_t)nrows);
    // short rows by entry count, longest first, ascending row id among equals (counting sort)
    std::vector<int64_t> bucket((size_t)kSpmmSegment + 2, 0);
    for (int64_t r = 0; r < nrows; ++r) {
        const int64_t deg = rp[r + 1] - rp[r];
        if (deg <= kSpmmSegment) bucket[(size_t)(kSpmmSegment - deg) + 1]++;
    }
    for (size_t i = 1; i < bucket.size(); ++i) bucket[i] += bucket[i - 1];
    P.rows_sorted.resize((size_t)bucket.back());
    for (int64_t r = 0; r < nrows; ++r) {
        const int64_t deg = rp[r + 1] - rp[r];
        if (deg <= kSpmmSegment) P.rows_sorted[(size_t)bucket[(size_t)(kSpmmSegment - deg)]++] = (int32_t)r;
    }
}

void append_plan(HostMeta::Plan& G, int32_t k, std::vector<PlanPart>& parts)
{
    G.range_off.assign((size_t)k + 1, 0);
    G.seg_off.assign((size_t)k + 1, 0);
    G.long_off.assign((size_t)k + 1, 0);
    G.rows_off.assign((size_t)k + 1, 0);
    for (int32_t p = 0; p < k; ++p) {
        PlanPart& P = parts[(size_t)p];
        G.rows_off[(size_t)p + 1] = G.rows_off[(size_t)p] + (int64_t)P.rows_sorted.size();
        G.rows_sorted.insert(G.rows_sorted.end(), P.rows_sorted.begin(), P.rows_sorted.end());
        G.range_off[(size_t)p + 1] = G.range_off[(size_t)p] + (int64_t)P.range_rows.size();
        G.seg_off[(size_t)p + 1] = G.seg_off[(size_t)p] + (int64_t)P.seg_row.size();
        G.long_off[(size_t)p + 1] = G.long_off[(size_t)p] + (int64_t)P.long_row.size();
        G.max_segs = std::max<int64_t>(G.max_segs, (int64_t)P.seg_row.size());
        G.range_rows.insert(G.range_rows.end(), P.range_rows.begin(), P.range_rows.end());
        G.seg_row.insert(G.seg_row.end(), P.seg_row.begin(), P.seg_row.end());
        G.seg_begin.insert(G.seg_begin.end(), P.seg_begin.begin(), P.seg_begin.end());
        G.seg_len.insert(G.seg_len.end(), P.seg_len.begin(), P.seg_len.end());
        G.long_row.insert(G.long_row.end(), P.long_row.begin(), P.long_row.end());
        G.long_first.insert(G.long_first.end(), P.long_first.begin(), P.long_first.end());
        G.long_nseg.insert(G.long_nseg.end(), P.long_nseg.begin(), P.long_nseg.end());
        P = PlanPart{};
    }
}

}  // namespace

void build_masked_transpose(HostMeta& M, const uint8_t* mask)
{
    HostMeta::MaskedTranspose& T = M.masked_t;
    T = HostMeta::MaskedTranspose{};
    const int32_t k = (int32_t)M.off.size() - 1;
    struct Part {
        std::vector<int64_t> len;       // kept entries of every kept row
        std::vector<int32_t> tcol, out_row;
        std::vector<float> tw;
    };
    std::vector<Part> parts((size_t)k);
    parallel_for(k, 1, [&](int, int64_t p) {
        Part& P = parts[(size_t)p];
        const int64_t r0 = M.off[(size_t)p], np = M.off[(size_t)p + 1] - r0;
        const int64_t t0 = M.toff[(size_t)p], nR = M.toff[(size_t)p + 1] - t0;
        const int64_t b0 = M.boff[(size_t)p];
        const uint8_t* m = mask + r0;
        for (int64_t i = 0; i < nR; ++i) {
            int64_t kept = 0;
            for (int64_t e = M.trp[(size_t)(t0 + i)]; e < M.trp[(size_t)(t0 + i) + 1]; ++e) {
                const int32_t v = M.tcol[(size_t)e];
                if (!m[v]) continue;
                P.tcol.push_back(v);
                P.tw.push_back(M.tw[(size_t)e]);
                ++kept;
            }
            if (kept) {
                P.len.push_back(kept);
                P.out_row.push_back(i < np ? (int32_t)(r0 + i) : M.bnd[(size_t)(b0 + i - np)]);
            }
        }
    });
    T.toff.assign((size_t)k + 1, 0);
    int64_t entries = 0;
    for (int32_t p = 0; p < k; ++p) {
        T.toff[(size_t)p + 1] = T.toff[(size_t)p] + (int64_t)parts[(size_t)p].len.size();
        entries += (int64_t)parts[(size_t)p].tcol.size();
    }
    T.trp.reserve((size_t)T.toff[(size_t)k] + 1);
    T.tcol.reserve((size_t)entries);
    T.tw.reserve((size_t)entries);
    T.out_row.reserve((size_t)T.toff[(size_t)k]);
    T.trp.push_back(0);
    for (int32_t p = 0; p < k; ++p) {
        Part& P = parts[(size_t)p];
        for (int64_t len : P.len) T.trp.push_back(T.trp.back() + len);
        T.tcol.insert(T.tcol.end(), P.tcol.begin(), P.tcol.end());
        T.tw.insert(T.tw.end(), P.tw.begin(), P.tw.end());
        T.out_row.insert(T.out_row.end(), P.out_row.begin(), P.out_row.end());
        P = Part{};
    }
    std::vector<PlanPart> plan((size_t)k);
    parallel_for(k, 1, [&](int, int64_t p) {
        const int64_t t0 = T.toff[(size_t)p];
        plan_partition(T.trp.data() + t0, T.toff[(size_t)p + 1] - t0, plan[(size_t)p]);
    });
    append_plan(T.plan, k, plan);
    T.ready = true;
}

gnn_status build_host_meta(int model, int64_t n, const int64_t* rowptr, const int32_t* colidx,
                           int32_t k, int32_t mode, uint64_t seed, const int32_t* user_part,
                           bool want_runs, HostMeta& M, std::string& err)
{
    if (!rowptr || n < 1) { err = "n must be >= 1 and rowptr non-null"; return GNN_EINVAL; }
    if (n > 0x7FFFFFF0ll) { err = "n exceeds the int32 vertex id range"; return GNN_EINVAL; }
    if (k < 1 || (int64_t)k > n) { err = "k must satisfy 1 <= k <= n"; return GNN_EINVAL; }
    if (mode != GNN_PART_USER && mode != GNN_PART_RANDOM && mode != GNN_PART_LP &&
        mode != GNN_PART_SWITCHING && mode != GNN_PART_SWITCHING_DEVICE) {
        err = "unknown partition mode"; return GNN_EINVAL;
    }
    if (mode == GNN_PART_USER && !user_part) { err = "user_part is null"; return GNN_EINVAL; }
    if (rowptr[0] != 0) { err = "rowptr[0] must be 0"; return GNN_EINVAL; }
    for (int64_t v = 0; v < n; ++v)
        if (rowptr[v + 1] < rowptr[v]) { err = "rowptr is not monotone"; return GNN_EINVAL; }
    const int64_t nnz_in = rowptr[n];
    if (nnz_in > 0 && !colidx) { err = "colidx is null"; return GNN_EINVAL; }
    {
        std::atomic<int> bad{0};
        parallel_for(n, 8192, [&](int, int64_t v) {
            int64_t prev = -1;
            for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
                int64_t u = colidx[e];
                if (u < 0 || u >= n || u <= prev) bad.store(1, std::memory_order_relaxed);
                prev = u;
            }
        });
        if (bad.load()) {
            err = "colidx must lie in [0, n) and ascend strictly inside every row";
            return GNN_EINVAL;
        }
    }

    try {
        M = HostMeta{};
        M.n = n;
        M.k = k;
        M.model = model;

        // ---- assignment ----------------------------------------------------------------
        if (mode == GNN_PART_USER) {
            M.part.assign(user_part, user_part + n);
            for (int64_t v = 0; v < n; ++v)
                if (M.part[(size_t)v] < 0 || M.part[(size_t)v] >= k) {
                    err = "user_part entry outside [0, k)";
                    return GNN_EINVAL;
                }
        } else if (mode == GNN_PART_SWITCHING || mode == GNN_PART_SWITCHING_DEVICE) {
            if (mode == GNN_PART_SWITCHING_DEVICE && k > switch_pref_max_k()) {
                err = "GNN_PART_SWITCHING_DEVICE supports at most " + std::to_string(switch_pref_max_k()) +
                      " partitions";
                return GNN_EUNSUPPORTED;
            }
            SwitchingInfo info;
            assign_switching(n, rowptr, colidx, k, seed, mode == GNN_PART_SWITCHING_DEVICE, M.part, info);
            M.part_iterations = info.iterations;
            M.part_objective = std::move(info.objective);
        } else {
            assign_random(n, k, seed, M.part);
            if (mode == GNN_PART_LP)
                for (int round = 0; round < 10; ++round) lp_round(n, rowptr, colidx, k, M.part);
        }

        // ---- library order: partition-major, ascending original id inside ----------------
        M.off.assign((size_t)k + 1, 0);
        for (int64_t v = 0; v < n; ++v) M.off[(size_t)M.part[(size_t)v] + 1]++;
        for (int32_t p = 0; p < k; ++p) M.off[(size_t)p + 1] += M.off[(size_t)p];
        M.order.resize((size_t)n);
        M.newid.resize((size_t)n);
        {
            std::vector<int64_t> cur(M.off.begin(), M.off.end() - 1);
            for (int64_t v = 0; v < n; ++v) {
                int64_t r = cur[(size_t)M.part[(size_t)v]]++;
                M.order[(size_t)r] = (int32_t)v;
                M.newid[(size_t)v] = (int32_t)r;
            }
        }

        // ---- operator rows: A + I for GCN (one self-loop each), A for SAGE ----------------
        // GCN: A + I with symmetric-normalisation weights; GAT: the structure of A + I, weights
        // come from the attention at run time; SAGE: A with 1/in-degree row scales
        const bool gat = (model == GNN_GAT);
        const bool self_loops = (model == GNN_GCN) || gat;
        const bool gcn = (model == GNN_GCN);
        std::vector<int32_t> opdeg((size_t)n);       // by original id
        std::vector<uint8_t> add_self((size_t)n, 0);  // by original id
        parallel_for(n, 8192, [&](int, int64_t v) {
            int64_t len = rowptr[v + 1] - rowptr[v];
            if (self_loops) {
                const int32_t* b = colidx + rowptr[v];
                bool has = std::binary_search(b, b + len, (int32_t)v);
                add_self[(size_t)v] = has ? 0 : 1;
                len += has ? 0 : 1;
            }
            opdeg[(size_t)v] = (int32_t)len;
        });
        M.rp.assign((size_t)n + 1, 0);
        for (int64_t r = 0; r < n; ++r)
            M.rp[(size_t)r + 1] = M.rp[(size_t)r] + opdeg[(size_t)M.order[(size_t)r]];
        const int64_t nnz = M.rp[(size_t)n];
        M.lcol.resize((size_t)nnz);
        if (gcn) M.ew.resize((size_t)nnz);
        else if (!gat) {
            M.rscale.resize((size_t)n);
            for (int64_t r = 0; r < n; ++r) {
                int32_t dg = opdeg[(size_t)M.order[(size_t)r]];
                M.rscale[(size_t)r] = dg > 0 ? (float)(1.0 / (double)dg) : 0.0f;
            }
        }

        // ---- phase A: boundary lists and local columns, partitions in parallel -----------
        std::vector<std::vector<int32_t>> bnd_p((size_t)k);
        const int nt = worker_count();
        std::vector<std::vector<int32_t>> lmap((size_t)nt);  // row -> index in B_p, or -1
        parallel_for(k, 1, [&](int tid, int64_t p) {
            auto& map = lmap[(size_t)tid];
            if (map.empty()) map.assign((size_t)n, -1);
            const int64_t r0 = M.off[(size_t)p], r1 = M.off[(size_t)p + 1];
            auto& B = bnd_p[(size_t)p];
            for (int64_t r = r0; r < r1; ++r) {
                int64_t v = M.order[(size_t)r];
                for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
                    int32_t ur = M.newid[(size_t)colidx[e]];
                    if ((ur < r0 || ur >= r1) && map[(size_t)ur] < 0) {
                        map[(size_t)ur] = 0;
                        B.push_back(ur);
                    }
                }
            }
            std::sort(B.begin(), B.end());  // ascending row == (partition id, original id)
            for (size_t i = 0; i < B.size(); ++i) map[(size_t)B[i]] = (int32_t)i;
            const int32_t np = (int32_t)(r1 - r0);
            std::vector<std::pair<int32_t, float>> row;
            for (int64_t r = r0; r < r1; ++r) {
                int64_t v = M.order[(size_t)r];
                row.clear();
                const double dv = (double)opdeg[(size_t)v];
                auto push = [&](int64_t u) {
                    int32_t ur = M.newid[(size_t)u];
                    int32_t lc = (ur >= r0 && ur < r1) ? (int32_t)(ur - r0)
                                                       : np + map[(size_t)ur];
                    float w = gcn ? (float)(1.0 / std::sqrt((double)opdeg[(size_t)u] * dv)) : 1.0f;
                    row.emplace_back(lc, w);
                };
                for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) push(colidx[e]);
                if (self_loops && add_self[(size_t)v]) push(v);
                std::sort(row.begin(), row.end(),
                          [](const std::pair<int32_t, float>& a, const std::pair<int32_t, float>& b) {
                              return a.first < b.first;
                          });
                int64_t o = M.rp[(size_t)r];
                for (auto& pr : row) {
                    M.lcol[(size_t)o] = pr.first;
                    if (gcn) M.ew[(size_t)o] = pr.second;
                    ++o;
                }
            }
            for (int32_t ur : B) map[(size_t)ur] = -1;
        });
        lmap.clear();
        lmap.shrink_to_fit();

        // ---- phase B: offsets --------------------------------------------------------------
        M.boff.assign((size_t)k + 1, 0);
        M.toff.assign((size_t)k + 1, 0);
        for (int32_t p = 0; p < k; ++p) {
            int64_t np = M.off[(size_t)p + 1] - M.off[(size_t)p];
            M.boff[(size_t)p + 1] = M.boff[(size_t)p] + (int64_t)bnd_p[(size_t)p].size();
            M.toff[(size_t)p + 1] = M.toff[(size_t)p] + np + (int64_t)bnd_p[(size_t)p].size();
        }
        M.bnd.resize((size_t)M.boff[(size_t)k]);
        M.bnd_orig.resize((size_t)M.boff[(size_t)k]);
        for (int32_t p = 0; p < k; ++p) {
            int64_t o = M.boff[(size_t)p];
            for (int32_t ur : bnd_p[(size_t)p]) {
                M.bnd[(size_t)o] = ur;
                M.bnd_orig[(size_t)o] = M.order[(size_t)ur];
                ++o;
            }
            std::vector<int32_t>().swap(bnd_p[(size_t)p]);
        }

        if (want_runs) {
            // B_p is ascending in library row, i.e. grouped by source partition: record where
            // each group starts and the row number inside the source partition's block
            M.brun.assign((size_t)k * ((size_t)k + 1), 0);
            M.bnd_local.resize(M.bnd.size());
            parallel_for(k, 1, [&](int, int64_t p) {
                const int32_t* b0 = M.bnd.data() + M.boff[(size_t)p];
                const int32_t* b1 = M.bnd.data() + M.boff[(size_t)p + 1];
                int64_t* run = M.brun.data() + (size_t)p * ((size_t)k + 1);
                for (int32_t q = 0; q <= k; ++q)
                    run[q] = std::lower_bound(b0, b1, (int32_t)M.off[(size_t)q]) - b0;
                for (int32_t q = 0; q < k; ++q)
                    for (int64_t i = run[q]; i < run[q + 1]; ++i)
                        M.bnd_local[(size_t)(M.boff[(size_t)p] + i)] = b0[i] - (int32_t)M.off[(size_t)q];
            });
            int64_t max_own = 0;
            for (int32_t p = 0; p < k; ++p) max_own = std::max(max_own, M.off[(size_t)p + 1] - M.off[(size_t)p]);
            if ((int64_t)k * max_own < 0x7FFFFFF0ll) {
                M.bnd_flat.resize(M.bnd.size());
                parallel_for(k, 1, [&](int, int64_t p) {
                    const int64_t* run = M.brun.data() + (size_t)p * ((size_t)k + 1);
                    for (int32_t q = 0; q < k; ++q)
                        for (int64_t i = run[q]; i < run[q + 1]; ++i) {
                            const size_t at = (size_t)(M.boff[(size_t)p] + i);
                            M.bnd_flat[at] = (int32_t)((int64_t)q * max_own + M.bnd_local[at]);
                        }
                });
            }
        }

        // ---- order in which an epoch walks the partitions -------------------------------------
        // The next partition is the one that shares most blocks with the one just processed
        // (its own block and the owners of its boundary rows), so that blocks already in the
        // cache are reused before they are evicted; the 1-hop topology is fixed, so the order
        // is too (appendix on I/O optimisations, overlap of cache management and computation).
        // Starts at partition 0; equal overlaps go to the lower id.
        {
            const size_t words = ((size_t)k + 63) / 64;
            std::vector<uint64_t> dep((size_t)k * words, 0);
            parallel_for(k, 1, [&](int, int64_t p) {
                uint64_t* d = dep.data() + (size_t)p * words;
                d[(size_t)p / 64] |= 1ull << (p % 64);
                const int32_t* b0 = M.bnd.data() + M.boff[(size_t)p];
                const int32_t* b1 = M.bnd.data() + M.boff[(size_t)p + 1];
                int32_t q = 0;
                for (const int32_t* b = b0; b < b1;) {      // ascending rows: one hop per owner
                    while (M.off[(size_t)q + 1] <= *b) ++q;
                    d[(size_t)q / 64] |= 1ull << (q % 64);
                    b = std::lower_bound(b, b1, (int32_t)M.off[(size_t)q + 1]);
                }
            });
            M.sched.assign((size_t)k, 0);
            std::vector<uint8_t> used((size_t)k, 0);
            used[0] = 1;
            const char* fixed = std::getenv("GNNMI_SCHEDULE");
            const bool identity = fixed && std::strcmp(fixed, "identity") == 0;
            for (int32_t t = 1; t < k; ++t) {
                if (identity) { M.sched[(size_t)t] = t; continue; }
                const uint64_t* dc = dep.data() + (size_t)M.sched[(size_t)t - 1] * words;
                int32_t best = -1;
                int64_t best_common = -1;
                for (int32_t q = 0; q < k; ++q) {
                    if (used[(size_t)q]) continue;
                    const uint64_t* dq = dep.data() + (size_t)q * words;
                    int64_t common = 0;
                    for (size_t w = 0; w < words; ++w) common += __builtin_popcountll(dc[w] & dq[w]);
                    if (common > best_common) { best_common = common; best = q; }
                }
                M.sched[(size_t)t] = best;
                used[(size_t)best] = 1;
            }
        }

        // ---- phase C: transpose of every T_p ------------------------------------------------
        M.trp.assign((size_t)M.toff[(size_t)k] + 1, 0);
        M.tcol.resize((size_t)nnz);
        if (gat) M.tperm.resize((size_t)nnz);
        else M.tw.resize((size_t)nnz);
        std::vector<int64_t> required((size_t)k, 0);
        parallel_for(k, 1, [&](int, int64_t p) {
            const int64_t r0 = M.off[(size_t)p], r1 = M.off[(size_t)p + 1];
            const int64_t nR = M.toff[(size_t)p + 1] - M.toff[(size_t)p];
            const int64_t e0 = M.rp[(size_t)r0], e1 = M.rp[(size_t)r1];
            int64_t* trp = M.trp.data() + M.toff[(size_t)p];
            std::vector<int64_t> cursor((size_t)nR + 1, 0);
            for (int64_t e = e0; e < e1; ++e) cursor[(size_t)M.lcol[(size_t)e] + 1]++;
            int64_t req = 0;
            for (int64_t i = 0; i < nR; ++i) {
                if (cursor[(size_t)i + 1] > 0) ++req;
                cursor[(size_t)i + 1] += cursor[(size_t)i];
            }
            required[(size_t)p] = req;
            for (int64_t i = 0; i < nR; ++i) trp[i] = e0 + cursor[(size_t)i];
            if (p == k - 1) trp[nR] = e1;
            for (int64_t r = r0; r < r1; ++r) {
                const float rs = (gcn || gat) ? 1.0f : M.rscale[(size_t)r];
                for (int64_t e = M.rp[(size_t)r]; e < M.rp[(size_t)r + 1]; ++e) {
                    int64_t pos = e0 + cursor[(size_t)M.lcol[(size_t)e]]++;
                    M.tcol[(size_t)pos] = (int32_t)(r - r0);
                    if (gat) M.tperm[(size_t)pos] = (int32_t)(e - e0);
                    else M.tw[(size_t)pos] = gcn ? M.ew[(size_t)e] : rs;
                }
            }
        });

        // ---- phase D: work items of the aggregation kernels -------------------------------------
        {
            std::vector<PlanPart> fw((size_t)k), bw((size_t)k);
            parallel_for(k, 1, [&](int, int64_t p) {
                const int64_t r0 = M.off[(size_t)p], np = M.off[(size_t)p + 1] - r0;
                plan_partition(M.rp.data() + r0, np, fw[(size_t)p]);
                const int64_t t0 = M.toff[(size_t)p], nR = M.toff[(size_t)p + 1] - t0;
                plan_partition(M.trp.data() + t0, nR, bw[(size_t)p]);
            });
            append_plan(M.plan_fwd, k, fw);
            append_plan(M.plan_bwd, k, bw);
        }

        // ---- stats ---------------------------------------------------------------------------
        gnn_stats& S = M.stats;
        S.n = n;
        S.nnz = nnz;
        S.k = k;
        S.sum_boundary = M.boff[(size_t)k];
        for (int32_t p = 0; p < k; ++p) {
            S.sum_required += required[(size_t)p];
            S.max_own = std::max(S.max_own, M.off[(size_t)p + 1] - M.off[(size_t)p]);
            S.max_boundary = std::max(S.max_boundary, M.boff[(size_t)p + 1] - M.boff[(size_t)p]);
            S.max_nnz = std::max(S.max_nnz,
                                 M.rp[(size_t)M.off[(size_t)p + 1]] - M.rp[(size_t)M.off[(size_t)p]]);
        }
    } catch (const std::bad_alloc&) {
        err = "out of host memory while building partitions";
        return GNN_ENOMEM;
    } catch (const HipFailure& f) {
        err = f.what;
        return GNN_EHIP;
    }
    return GNN_OK;
}

}  // namespace gnnmi
