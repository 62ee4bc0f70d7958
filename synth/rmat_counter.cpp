// Counter-based R-MAT generator for the large synthetic inputs (50 M vertices and more), where
// the numpy generator's single-threaded draws and sort take minutes.  Input data only: nothing
// of the method's arithmetic lives here.
//
// Recipe (every step a pure function of the seed and a counter, so it runs on any number of
// threads with the same result):
//   * draw e in [0, m): level pair q = 0, 1, .. uses r = splitmix64(key_e + q) with
//     key_e = splitmix64(seed ^ splitmix64(e)); the high and the low 32 bits of r pick the
//     quadrant of two successive levels: x < A -> (0,0), x < A+B -> (0,1), x < A+B+C -> (1,0),
//     else (1,1), with A, B, C the quadrant probabilities scaled to 2^32;
//   * ids are squeezed from [0, 2^scale) to [0, n) by id * n >> scale;
//   * ids pass through the permutation that sorts the vertices by
//     (splitmix64(seed ^ 0x5bd1e995 ^ splitmix64(v)), v);
//   * self-draws are dropped, duplicates removed (of the unordered pair when symmetric), every
//     edge is mirrored when symmetric, one self-loop per vertex is added on request;
//   * output: CSR by destination, columns ascending.
#include <algorithm>
#include <cstdint>
#include <cstdlib>
#include <new>
#include <parallel/algorithm>
#include <vector>
#include <chrono>
#include <cstdio>

namespace {

inline uint64_t splitmix64(uint64_t x)
{
    uint64_t z = x + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

struct Graph {
    std::vector<int64_t> rowptr;
    std::vector<int32_t> colidx;
};

}  // namespace

extern "C" {

// Returns a handle (or null when out of memory) and the number of CSR entries in *nnz.
void* rmat_counter_generate(int64_t n, int64_t m, uint64_t seed, int scale, double a, double b, double c,
                            int symmetric, int self_loops, int64_t* nnz)
{
    try {
        auto T0 = std::chrono::steady_clock::now();
        auto lap = [&](const char* what) {
            if (!std::getenv("SYNTH_TIMING")) return;
            auto t = std::chrono::steady_clock::now();
            std::fprintf(stderr, "  rmat_counter %s: %.2f s\n", what, std::chrono::duration<double>(t - T0).count());
            T0 = t;
        };
        const uint64_t A = (uint64_t)(a * 4294967296.0), B = (uint64_t)((a + b) * 4294967296.0),
                       Cq = (uint64_t)((a + b + c) * 4294967296.0);
        // permutation: position -> vertex
        std::vector<uint64_t> pk((size_t)n);
        std::vector<int32_t> perm((size_t)n);
#pragma omp parallel for schedule(static)
        for (int64_t v = 0; v < n; ++v) {
            pk[(size_t)v] = splitmix64(seed ^ 0x5bd1e995ull ^ splitmix64((uint64_t)v));
            perm[(size_t)v] = (int32_t)v;
        }
        __gnu_parallel::sort(perm.begin(), perm.end(), [&](int32_t x, int32_t y) {
            return pk[(size_t)x] != pk[(size_t)y] ? pk[(size_t)x] < pk[(size_t)y] : x < y;
        });
        std::vector<uint64_t>().swap(pk);
        lap("permutation");

        const uint64_t none = ~0ull;
        std::vector<uint64_t> keys((size_t)m + (self_loops ? (size_t)n : 0));
#pragma omp parallel for schedule(static)
        for (int64_t e = 0; e < m; ++e) {
            const uint64_t key = splitmix64(seed ^ splitmix64((uint64_t)e));
            uint64_t s = 0, t = 0;
            uint64_t r = 0;
            for (int l = 0; l < scale; ++l) {
                if ((l & 1) == 0) r = splitmix64(key + (uint64_t)(l >> 1));
                const uint64_t x = (l & 1) == 0 ? (r >> 32) : (r & 0xFFFFFFFFull);
                const uint64_t sbit = x >= B ? 1 : 0;
                const uint64_t tbit = ((x >= A && x < B) || x >= Cq) ? 1 : 0;
                s = (s << 1) | sbit;
                t = (t << 1) | tbit;
            }
            s = (uint64_t)(((unsigned __int128)s * (uint64_t)n) >> scale);
            t = (uint64_t)(((unsigned __int128)t * (uint64_t)n) >> scale);
            s = (uint64_t)perm[(size_t)s];
            t = (uint64_t)perm[(size_t)t];
            if (s == t) {
                keys[(size_t)e] = none;
            } else if (symmetric) {
                const uint64_t lo = s < t ? s : t, hi = s < t ? t : s;
                keys[(size_t)e] = lo * (uint64_t)n + hi;
            } else {
                keys[(size_t)e] = t * (uint64_t)n + s;      // (destination, source)
            }
        }
        std::vector<int32_t>().swap(perm);
        lap("draws");
        if (self_loops && !symmetric) {
#pragma omp parallel for schedule(static)
            for (int64_t v = 0; v < n; ++v) keys[(size_t)m + (size_t)v] = (uint64_t)v * (uint64_t)n + (uint64_t)v;
        } else if (self_loops) {
            keys.resize((size_t)m);
        }
        __gnu_parallel::sort(keys.begin(), keys.end());
        keys.erase(std::unique(keys.begin(), keys.end()), keys.end());
        while (!keys.empty() && keys.back() == none) keys.pop_back();
        lap("sort + unique");
        if (symmetric) {
            const size_t u = keys.size();
            keys.resize(2 * u + (self_loops ? (size_t)n : 0));
#pragma omp parallel for schedule(static)
            for (int64_t i = 0; i < (int64_t)u; ++i) {
                const uint64_t lo = keys[(size_t)i] / (uint64_t)n, hi = keys[(size_t)i] % (uint64_t)n;
                keys[(size_t)i] = lo * (uint64_t)n + hi;          // row lo lists hi
                keys[u + (size_t)i] = hi * (uint64_t)n + lo;
            }
            if (self_loops) {
#pragma omp parallel for schedule(static)
                for (int64_t v = 0; v < n; ++v) keys[2 * u + (size_t)v] = (uint64_t)v * (uint64_t)n + (uint64_t)v;
            }
            __gnu_parallel::sort(keys.begin(), keys.end());
        }
        Graph* g = new Graph();
        const int64_t cnt = (int64_t)keys.size();
        g->rowptr.assign((size_t)n + 1, 0);
        g->colidx.resize((size_t)cnt);
        std::vector<int64_t>& rp = g->rowptr;
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < cnt; ++i) {
            const uint64_t d = keys[(size_t)i] / (uint64_t)n;
            g->colidx[(size_t)i] = (int32_t)(keys[(size_t)i] - d * (uint64_t)n);
            // first entry of a row: every row between the previous entry's row and this one starts here
            const uint64_t dprev = i == 0 ? 0 : keys[(size_t)i - 1] / (uint64_t)n;
            if (i == 0) for (uint64_t r = 0; r <= d; ++r) rp[(size_t)r] = 0;
            else for (uint64_t r = dprev + 1; r <= d; ++r) rp[(size_t)r] = i;
        }
        const uint64_t dlast = cnt ? keys[(size_t)cnt - 1] / (uint64_t)n : 0;
        for (uint64_t r = (cnt ? dlast + 1 : 0); r <= (uint64_t)n; ++r) rp[(size_t)r] = cnt;
        lap("csr");
        *nnz = cnt;
        return g;
    } catch (const std::bad_alloc&) {
        return nullptr;
    }
}

void rmat_counter_fetch(void* handle, int64_t* rowptr, int32_t* colidx)
{
    Graph* g = static_cast<Graph*>(handle);
    std::copy(g->rowptr.begin(), g->rowptr.end(), rowptr);
    std::copy(g->colidx.begin(), g->colidx.end(), colidx);
    delete g;
}

// out[i] = standard normal number i of the stream `seed` for i in [0, count): numbers 2j and
// 2j + 1 are the two outputs of one Box-Muller transform of the halves of splitmix64(key + j).
void normal_counter_fill(float* out, int64_t first, int64_t count, uint64_t seed)
{
    const uint64_t key = splitmix64(seed ^ 0xA0761D6478BD642Full);
    const int64_t p0 = first >> 1, p1 = (first + count + 1) >> 1;
#pragma omp parallel for schedule(static)
    for (int64_t p = p0; p < p1; ++p) {
        const uint64_t r = splitmix64(key + (uint64_t)p);
        // two uniforms from the halves of r; u1 in (0, 1]
        const float u1 = ((float)(r >> 40) + 1.0f) * (1.0f / 16777216.0f);
        const float u2 = (float)((r >> 8) & 0xFFFFFFull) * (1.0f / 16777216.0f);
        const float rad = __builtin_sqrtf(-2.0f * __builtin_logf(u1));
        const float ang = 6.2831853071795864f * u2;
        const int64_t i0 = 2 * p - first, i1 = i0 + 1;
        if (i0 >= 0 && i0 < count) out[i0] = rad * __builtin_cosf(ang);
        if (i1 >= 0 && i1 < count) out[i1] = rad * __builtin_sinf(ang);
    }
}

}  // extern "C"
