// Small dense kernels of the path (plain fp32 ALU work): softmax cross-entropy with its
// gradient, and the activation backward with the bias gradient.
#include "gnn_internal.h"

namespace gnnmi {
namespace {

constexpr int kBlock = 256;
constexpr int kWave = 64;
constexpr int kRowsPerBlockAct = 64;

__device__ inline float wave_max(float v)
{
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) v = fmaxf(v, __shfl_xor(v, m, kWave));
    return v;
}
__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) v += __shfl_xor(v, m, kWave);
    return v;
}

// One wavefront per vertex.  Masked rows: max-subtracted softmax, loss term, gradient
// (softmax - onehot) / |M|.  Other rows: zero gradient.  Each block writes the sum of its
// rows' loss terms to partial[blockIdx.x]; a second kernel adds the partials in order.
__global__ __launch_bounds__(kBlock) void k_loss(const float* __restrict__ logits,
                                                 const int32_t* __restrict__ labels,
                                                 const uint8_t* __restrict__ mask,
                                                 float* __restrict__ grad, int64_t n, int32_t c,
                                                 const unsigned long long* __restrict__ count,
                                                 float* __restrict__ partial)
{
    __shared__ float wsum[kBlock / kWave];
    const unsigned long long cnt = *count;
    const float inv_count = cnt ? 1.f / (float)cnt : 0.f;
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int64_t v = (int64_t)blockIdx.x * (kBlock / kWave) + wave;
    float term = 0.f;
    if (v < n) {
        const float* x = logits + v * c;
        float* g = grad + v * c;
        if (mask[v]) {
            float mx = -INFINITY;
            for (int j = lane; j < c; j += kWave) mx = fmaxf(mx, x[j]);
            mx = wave_max(mx);
            float se = 0.f;
            for (int j = lane; j < c; j += kWave) se += expf(x[j] - mx);
            se = wave_sum(se);
            const float lse = mx + logf(se);
            const int32_t y = labels[v];
            term = lse - x[y];
            for (int j = lane; j < c; j += kWave)
                g[j] = (expf(x[j] - lse) - (j == y ? 1.f : 0.f)) * inv_count;
        } else {
            for (int j = lane; j < c; j += kWave) g[j] = 0.f;
        }
    }
    if (lane == 0) wsum[wave] = term;
    __syncthreads();
    if (threadIdx.x == 0) {
        float s = 0.f;
        for (int i = 0; i < kBlock / kWave; ++i) s += wsum[i];
        partial[blockIdx.x] = s;
    }
}

// |M|: integer block counts added with one integer atomic per block (order-independent).
__global__ __launch_bounds__(kBlock) void k_count_mask(const uint8_t* __restrict__ mask, int64_t n,
                                                       unsigned long long* __restrict__ count)
{
    __shared__ unsigned int sm[kBlock];
    unsigned int c = 0;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * kBlock)
        c += mask[i] ? 1u : 0u;
    sm[threadIdx.x] = c;
    __syncthreads();
    for (int w = kBlock / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) sm[threadIdx.x] += sm[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0 && sm[0]) atomicAdd(count, (unsigned long long)sm[0]);
}

// Single block: fixed-order tree over the block partials.
__global__ __launch_bounds__(kBlock) void k_loss_finish(const float* __restrict__ partial,
                                                        int64_t nparts,
                                                        const unsigned long long* __restrict__ count,
                                                        float* __restrict__ loss)
{
    __shared__ float sm[kBlock];
    const unsigned long long cnt = *count;
    const float inv_count = cnt ? 1.f / (float)cnt : 0.f;
    float s = 0.f;
    for (int64_t i = threadIdx.x; i < nparts; i += kBlock) s += partial[i];
    sm[threadIdx.x] = s;
    __syncthreads();
    for (int w = kBlock / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) sm[threadIdx.x] += sm[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss = sm[0] * inv_count;
}

// dy = g * [act > 0] (act == null: dy aliases g, nothing is written) and per-block column
// sums of dy into partial[block][d].  A block covers 64 rows; thread t walks columns
// t, t + 256, ... so that a row segment is read coalesced.
__global__ __launch_bounds__(kBlock) void k_act_bwd(const float* __restrict__ g,
                                                    const float* __restrict__ act,
                                                    float* __restrict__ dy, int64_t rows,
                                                    int32_t d, float* __restrict__ partial)
{
    const int64_t r0 = (int64_t)blockIdx.x * kRowsPerBlockAct;
    const int64_t r1 = r0 + kRowsPerBlockAct < rows ? r0 + kRowsPerBlockAct : rows;
    for (int32_t c = threadIdx.x; c < d; c += kBlock) {
        float s = 0.f;
        for (int64_t r = r0; r < r1; ++r) {
            float v = g[r * d + c];
            if (act) {
                v = act[r * d + c] > 0.f ? v : 0.f;
                dy[r * d + c] = v;
            }
            s += v;
        }
        partial[(int64_t)blockIdx.x * d + c] = s;
    }
}

__global__ __launch_bounds__(kBlock) void k_colsum_finish(const float* __restrict__ partial,
                                                          int64_t nblocks, int32_t d,
                                                          float* __restrict__ gb)
{
    const int32_t c = blockIdx.x * kBlock + threadIdx.x;
    if (c >= d) return;
    float s = 0.f;
    for (int64_t b = 0; b < nblocks; ++b) s += partial[b * d + c];
    gb[c] += s;
}

}  // namespace

int64_t loss_partial_floats(int64_t n) { return (n + 3) / 4 + 1; }

void launch_loss(const float* logits, const int32_t* labels, const uint8_t* mask, float* grad,
                 int64_t n, int32_t c, unsigned long long* count_dev, float* partial,
                 float* loss_dev, hipStream_t s)
{
    launch_fill_zero(count_dev, sizeof(unsigned long long), s);
    int64_t cb = (n + kBlock * 64 - 1) / (kBlock * 64);
    hipLaunchKernelGGL(k_count_mask, dim3((unsigned)(cb < 1 ? 1 : cb)), dim3(kBlock), 0, s, mask, n,
                       count_dev);
    const int64_t blocks = (n + (kBlock / kWave) - 1) / (kBlock / kWave);
    hipLaunchKernelGGL(k_loss, dim3((unsigned)blocks), dim3(kBlock), 0, s, logits, labels, mask,
                       grad, n, c, (const unsigned long long*)count_dev, partial);
    hipLaunchKernelGGL(k_loss_finish, dim3(1), dim3(kBlock), 0, s, (const float*)partial, blocks,
                       (const unsigned long long*)count_dev, loss_dev);
}

int64_t act_bwd_partial_floats(int64_t rows, int32_t d)
{
    return ((rows + kRowsPerBlockAct - 1) / kRowsPerBlockAct) * (int64_t)d;
}

void launch_act_bwd(const float* g, const float* act, float* dy, int64_t rows, int32_t d,
                    float* gb, float* partial, hipStream_t s)
{
    if (rows <= 0) return;
    const int64_t blocks = (rows + kRowsPerBlockAct - 1) / kRowsPerBlockAct;
    if (!act && !gb) return;
    hipLaunchKernelGGL(k_act_bwd, dim3((unsigned)blocks), dim3(kBlock), 0, s, g, act, dy, rows, d,
                       partial);
    if (gb)
        hipLaunchKernelGGL(k_colsum_finish, dim3((unsigned)((d + kBlock - 1) / kBlock)), dim3(kBlock),
                           0, s, (const float*)partial, blocks, d, gb);
}

}  // namespace gnnmi
