// Preference counting of the switching-aware partitioner on the device (partitioning section
// and its appendix: "source-level parallelism").  One wavefront per source vertex: the
// partitions of its neighbours are counted in a per-wavefront histogram in LDS, the first and
// second preference are the two best partitions by the exact integer score key, and the
// vertex's share of the objective is added to an integer sum (integer adds commute, so the
// result does not depend on the order of the waves).
#include "gnn_internal.h"

namespace gnnmi {
namespace {

constexpr int kWave = 64;
constexpr int kPrefWaves = 4;
constexpr long long kFracOne = 1 << 20;

struct Pref {
    long long key;
    int j;   // -1: none
};

// a ranks before b: higher key, then the vertex's own partition, then the lower id
__device__ inline bool ranks_before(const Pref& a, const Pref& b, int cur)
{
    if (b.j < 0) return a.j >= 0;
    if (a.j < 0) return false;
    if (a.key != b.key) return a.key > b.key;
    if ((a.j == cur) != (b.j == cur)) return a.j == cur;
    return a.j < b.j;
}

__device__ inline Pref wave_best(Pref a, int cur)
{
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) {
        Pref o;
        o.key = __shfl_xor(a.key, m, kWave);
        o.j = __shfl_xor(a.j, m, kWave);
        if (ranks_before(o, a, cur)) a = o;
    }
    return a;
}

__global__ __launch_bounds__(kPrefWaves* kWave) void k_switch_pref(
    long long n, const int64_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
    const int32_t* __restrict__ part, const int64_t* __restrict__ sizes, int k,
    int32_t* __restrict__ first, int32_t* __restrict__ second, unsigned long long* __restrict__ frac_sum)
{
    extern __shared__ int hist_all[];
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    int* h = hist_all + (size_t)wave * k;
    for (int j = lane; j < k; j += kWave) h[j] = 0;
    __threadfence_block();

    unsigned long long local = 0;
    const long long stride = (long long)gridDim.x * kPrefWaves;
    for (long long v = (long long)blockIdx.x * kPrefWaves + wave; v < n; v += stride) {
        const long long b = rowptr[v], e = rowptr[v + 1];
        const int cur = part[v];
        int degl = 0;
        for (long long i = b + lane; i < e; i += kWave) {
            const int u = colidx[i];
            if (u != v) {
                atomicAdd(&h[part[u]], 1);
                ++degl;
            }
        }
#pragma unroll
        for (int m = 1; m < kWave; m <<= 1) degl += __shfl_xor(degl, m, kWave);
        const long long deg = degl;
        __threadfence_block();

        // the two best distinct partitions this lane has seen
        Pref p1{0, -1}, p2{0, -1};
        auto offer = [&](int j) {
            if (j == p1.j || j == p2.j) return;
            Pref c;
            c.key = 11ll * n * h[j] - 10ll * k * deg * (long long)sizes[j];
            c.j = j;
            if (ranks_before(c, p1, cur)) {
                p2 = p1;
                p1 = c;
            } else if (ranks_before(c, p2, cur)) {
                p2 = c;
            }
        };
        for (long long i = b + lane; i < e; i += kWave) {
            const int u = colidx[i];
            if (u != v) offer(part[u]);
        }
        if (lane == 0) offer(cur);
        const Pref f = wave_best(p1, cur);
        const Pref s = wave_best(p1.j == f.j ? p2 : p1, cur);
        if (lane == 0) {
            first[v] = f.j;
            second[v] = s.j;
            if (deg > 0) local += (unsigned long long)(kFracOne * h[cur] / deg);
        }
        __threadfence_block();
        for (long long i = b + lane; i < e; i += kWave) {
            const int u = colidx[i];
            if (u != v) h[part[u]] = 0;
        }
        __threadfence_block();
    }
    if (lane == 0 && local) atomicAdd(frac_sum, local);
}

}  // namespace

int switch_pref_max_k() { return 65536 / (kPrefWaves * 4); }

void launch_switch_pref(int64_t n, const int64_t* rowptr, const int32_t* colidx, const int32_t* part,
                        const int64_t* sizes, int32_t k, int32_t* first, int32_t* second,
                        unsigned long long* frac_sum, hipStream_t s)
{
    if (n <= 0) return;
    int64_t blocks = (n + kPrefWaves - 1) / kPrefWaves;
    if (blocks > 4096) blocks = 4096;
    const size_t lds = (size_t)kPrefWaves * (size_t)k * sizeof(int);
    hipLaunchKernelGGL(k_switch_pref, dim3((unsigned)blocks), dim3(kPrefWaves * kWave), lds, s,
                       (long long)n, rowptr, colidx, part, sizes, (int)k, first, second, frac_sum);
}

}  // namespace gnnmi
