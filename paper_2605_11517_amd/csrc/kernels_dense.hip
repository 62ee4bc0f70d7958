// Small dense kernels of the path (plain fp32 ALU work): softmax cross-entropy with its
// gradient, and the activation backward with the bias gradient.
#include "gnn_internal.h"

namespace gnnmi {
namespace {

constexpr int kBlock = 256;
constexpr int kWave = 64;
constexpr int kRowsPerBlockAct = 256;
constexpr int kLossRowsPerWave = 16;

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
    float term = 0.f;
    // the wavefront's rows: their mask bytes in one read, then the zero rows (nothing to wait for,
    // the stores follow each other), then the train rows one by one
    const int64_t v0 = ((int64_t)blockIdx.x * (kBlock / kWave) + wave) * kLossRowsPerWave;
    const bool mine = lane < kLossRowsPerWave && v0 + lane < n;
    const unsigned long long in_range = __ballot(mine);
    const unsigned long long train = __ballot(mine && mask[v0 + lane] != 0);
    const bool vec = (c & 3) == 0 && (reinterpret_cast<uintptr_t>(grad) & 15) == 0;
    for (int it = 0; it < kLossRowsPerWave; ++it) {
        if (!((in_range >> it) & 1ull) || ((train >> it) & 1ull)) continue;
        float* g = grad + (v0 + it) * c;
        if (vec) {
            for (int j = lane; j < (c >> 2); j += kWave)
                reinterpret_cast<float4*>(g)[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        } else {
            for (int j = lane; j < c; j += kWave) g[j] = 0.f;
        }
    }
    // the labels of the wavefront's train rows in one read as well
    const int32_t my_label = (mine && ((train >> lane) & 1ull)) ? labels[v0 + lane] : 0;
    constexpr int NX = 4;                   // up to 256 classes: a row is read once, into registers
    for (int it = 0; c <= NX * kWave && it < kLossRowsPerWave; ++it) {
        if (!((train >> it) & 1ull)) continue;
        const int64_t v = v0 + it;
        const float* x = logits + v * c;
        float* g = grad + v * c;
        float xv[NX];
#pragma unroll
        for (int u = 0; u < NX; ++u) {
            const int j = lane + u * kWave;
            xv[u] = j < c ? x[j] : -INFINITY;
        }
        // (same order of operations per lane as the general loop below: the same bits)
        float mx = -INFINITY;
#pragma unroll
        for (int u = 0; u < NX; ++u) mx = fmaxf(mx, xv[u]);
        mx = wave_max(mx);
        float se = 0.f;
#pragma unroll
        for (int u = 0; u < NX; ++u)
            if (lane + u * kWave < c) se += expf(xv[u] - mx);
        se = wave_sum(se);
        const float lse = mx + logf(se);
        const int32_t y = __shfl(my_label, it, kWave);
        float xy = 0.f;
#pragma unroll
        for (int u = 0; u < NX; ++u) {
            const float cand = __shfl(xv[u], y & (kWave - 1), kWave);
            if ((y >> 6) == u) xy = cand;
        }
        term += lse - xy;
#pragma unroll
        for (int u = 0; u < NX; ++u) {
            const int j = lane + u * kWave;
            if (j < c) g[j] = (expf(xv[u] - lse) - (j == y ? 1.f : 0.f)) * inv_count;
        }
    }
    for (int it = 0; c > NX * kWave && it < kLossRowsPerWave; ++it) {
        if (!((train >> it) & 1ull)) continue;
        const int64_t v = v0 + it;
        const float* x = logits + v * c;
        float* g = grad + v * c;
        float mx = -INFINITY;
        for (int j = lane; j < c; j += kWave) mx = fmaxf(mx, x[j]);
        mx = wave_max(mx);
        float se = 0.f;
        for (int j = lane; j < c; j += kWave) se += expf(x[j] - mx);
        se = wave_sum(se);
        const float lse = mx + logf(se);
        const int32_t y = labels[v];
        term += lse - x[y];
        for (int j = lane; j < c; j += kWave)
            g[j] = (expf(x[j] - lse) - (j == y ? 1.f : 0.f)) * inv_count;
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

// dy = scale * g * [act > 0] (act == null: dy aliases g, nothing is written) and per-block column
// sums of dy into partial[block][d].  A block covers 256 rows.  Up to 256 columns are handled at
// a time: the block's threads form 256 / width row groups that walk the rows together (four
// rows in flight per thread), and the groups are combined through LDS in a fixed order.
__global__ __launch_bounds__(kBlock) void k_act_bwd(const float* __restrict__ g,
                                                    const float* __restrict__ act,
                                                    float* __restrict__ dy, int64_t rows,
                                                    int32_t d, float* __restrict__ partial,
                                                    float scale, const uint8_t* __restrict__ row_on)
{
    __shared__ float sm[kBlock];
    const int64_t r0 = (int64_t)blockIdx.x * kRowsPerBlockAct;
    const int64_t r1 = r0 + kRowsPerBlockAct < rows ? r0 + kRowsPerBlockAct : rows;
    for (int32_t cc = 0; cc < d; cc += kBlock) {
        const int cwe = d - cc < kBlock ? d - cc : kBlock;     // columns in this chunk
        const int rpp = kBlock / cwe;                          // rows per pass
        const int rsub = threadIdx.x / cwe;
        const int32_t c = cc + threadIdx.x % cwe;
        float s = 0.f;
        if (rsub < rpp) {
            constexpr int U = 4;
            for (int64_t r = r0 + rsub; r < r1; r += (int64_t)rpp * U) {
                float gv[U], av[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int64_t rr = r + (int64_t)u * rpp;
                    const bool ok = rr < r1 && (!row_on || row_on[rr]);   // other rows of g are zero
                    gv[u] = ok ? g[rr * d + c] : 0.f;
                    av[u] = (ok && act) ? act[rr * d + c] : 0.f;
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int64_t rr = r + (int64_t)u * rpp;
                    float v = gv[u];
                    if (act) {
                        v = av[u] > 0.f ? v * scale : 0.f;
                        if (rr < r1) dy[rr * d + c] = v;
                    }
                    s += v;
                }
            }
        }
        sm[threadIdx.x] = s;
        __syncthreads();
        if (threadIdx.x < cwe) {
            float total = 0.f;
            for (int q = 0; q < rpp; ++q) total += sm[q * cwe + threadIdx.x];
            partial[(int64_t)blockIdx.x * d + c] = total;
        }
        __syncthreads();
    }
}

// float4 variant for widths that are multiples of 4: cw = d / 4 threads cover one row, the
// block walks its 256 rows 256 / cw at a time with four row groups in flight, and the row
// groups are combined through LDS in a fixed order.
__global__ __launch_bounds__(kBlock) void k_act_bwd_vec(const float* __restrict__ g,
                                                        const float* __restrict__ act,
                                                        float* __restrict__ dy, int64_t rows,
                                                        int32_t d, float* __restrict__ partial,
                                                        float scale, const uint8_t* __restrict__ row_on)
{
    __shared__ float4 sm[kBlock];
    const int cw = d / 4;
    const int64_t r0 = (int64_t)blockIdx.x * kRowsPerBlockAct;
    const int64_t r1 = r0 + kRowsPerBlockAct < rows ? r0 + kRowsPerBlockAct : rows;
    for (int cc = 0; cc < cw; cc += kBlock) {
        const int cwe = cw - cc < kBlock ? cw - cc : kBlock;   // float4 columns in this chunk
        const int rpp = kBlock / cwe;                          // rows per pass
        const int rsub = threadIdx.x / cwe, cidx = cc + threadIdx.x % cwe;
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
        if (rsub < rpp) {
            constexpr int U = 4;
            for (int64_t r = r0 + rsub; r < r1; r += (int64_t)rpp * U) {
                float4 gv[U], av[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int64_t rr = r + (int64_t)u * rpp;
                    gv[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                    av[u] = make_float4(1.f, 1.f, 1.f, 1.f);
                    if (rr < r1 && (!row_on || row_on[rr])) {              // other rows of g are zero
                        gv[u] = reinterpret_cast<const float4*>(g + rr * d)[cidx];
                        if (act) av[u] = reinterpret_cast<const float4*>(act + rr * d)[cidx];
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int64_t rr = r + (int64_t)u * rpp;
                    float4 v = gv[u];
                    v.x = av[u].x > 0.f ? v.x * scale : 0.f;
                    v.y = av[u].y > 0.f ? v.y * scale : 0.f;
                    v.z = av[u].z > 0.f ? v.z * scale : 0.f;
                    v.w = av[u].w > 0.f ? v.w * scale : 0.f;
                    if (act && rr < r1) reinterpret_cast<float4*>(dy + rr * d)[cidx] = v;
                    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
                }
            }
        }
        sm[threadIdx.x] = s;
        __syncthreads();
        if (rsub == 0) {
            for (int q = 1; q < rpp; ++q) {
                const float4 o = sm[q * cwe + threadIdx.x];
                s.x += o.x; s.y += o.y; s.z += o.z; s.w += o.w;
            }
            reinterpret_cast<float4*>(partial + (int64_t)blockIdx.x * d)[cidx] = s;
        }
        __syncthreads();
    }
}

// bfloat16 variant: g fp32, act bfloat16 (may be null), dy bfloat16 (always written).  One
// thread per column walking the block's 256 rows; consecutive threads touch consecutive
// columns, so every access is coalesced.
__global__ __launch_bounds__(kBlock) void k_act_bwd_bf16(const float* __restrict__ g,
                                                         const uint16_t* __restrict__ act,
                                                         uint16_t* __restrict__ dy, int64_t rows,
                                                         int32_t d, float* __restrict__ partial,
                                                         float scale)
{
    const int64_t r0 = (int64_t)blockIdx.x * kRowsPerBlockAct;
    const int64_t r1 = r0 + kRowsPerBlockAct < rows ? r0 + kRowsPerBlockAct : rows;
    for (int32_t c = threadIdx.x; c < d; c += kBlock) {
        float s = 0.f;
        constexpr int U = 8;
        for (int64_t r = r0; r < r1; r += U) {
            float gv[U];
            uint32_t av[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const bool in = r + u < r1;
                gv[u] = in ? g[(r + u) * d + c] : 0.f;
                av[u] = (in && act) ? (uint32_t)act[(r + u) * d + c] : 0x3F80u;   // 1.0
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                // positive bfloat16: sign bit clear and not zero
                const bool pos = (av[u] & 0x8000u) == 0 && (av[u] & 0x7FFFu) != 0;
                const float v = pos ? gv[u] * scale : 0.f;
                if (r + u < r1) {
                    const uint32_t b = __float_as_uint(v);
                    dy[(r + u) * d + c] = (uint16_t)((b + 0x7FFFu + ((b >> 16) & 1u)) >> 16);
                }
                s += v;
            }
        }
        partial[(int64_t)blockIdx.x * d + c] = s;
    }
}

// The same for widths that are multiples of 4 (16-byte aligned rows): a block covers 256 rows x
// 256 columns, a thread four consecutive columns (16 bytes of g, 8 of act and dy) of every fourth
// row with four rows in flight; the four row groups are combined through LDS in a fixed order.
// The grid has one block per (row block, column chunk), so that a partition of 6*10^4 rows still
// gives every CU several workgroups.
__global__ __launch_bounds__(kBlock) void k_act_bwd_bf16_vec(const float* __restrict__ g,
                                                             const uint16_t* __restrict__ act,
                                                             uint16_t* __restrict__ dy, int64_t rows,
                                                             int32_t d, float* __restrict__ partial,
                                                             float scale)
{
    __shared__ float4 sm[kBlock];
    constexpr int CT = 64, RG = kBlock / CT;               // column threads, row groups
    const int64_t r0 = (int64_t)blockIdx.x * kRowsPerBlockAct;
    const int64_t r1 = r0 + kRowsPerBlockAct < rows ? r0 + kRowsPerBlockAct : rows;
    const int rsub = threadIdx.x / CT;
    const int32_t c = ((int32_t)blockIdx.y * CT + threadIdx.x % CT) * 4;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (c < d) {
        constexpr int U = 4;
        for (int64_t r = r0 + rsub; r < r1; r += (int64_t)RG * U) {
            float4 gv[U];
            uint2 av[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t rr = r + (int64_t)u * RG;
                gv[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                av[u] = make_uint2(0x3F803F80u, 0x3F803F80u);             // 1.0 four times
                if (rr < r1) {
                    gv[u] = *reinterpret_cast<const float4*>(g + rr * d + c);
                    if (act) av[u] = *reinterpret_cast<const uint2*>(act + rr * d + c);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t rr = r + (int64_t)u * RG;
                const uint32_t a4[4] = {av[u].x & 0xFFFFu, av[u].x >> 16, av[u].y & 0xFFFFu, av[u].y >> 16};
                const float g4[4] = {gv[u].x, gv[u].y, gv[u].z, gv[u].w};
                float v4[4];
                uint32_t b4[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    // positive bfloat16: sign bit clear and not zero
                    const bool pos = (a4[e] & 0x8000u) == 0 && (a4[e] & 0x7FFFu) != 0;
                    v4[e] = pos ? g4[e] * scale : 0.f;
                    const uint32_t b = __float_as_uint(v4[e]);
                    b4[e] = (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
                }
                if (rr < r1)
                    *reinterpret_cast<uint2*>(dy + rr * d + c) = make_uint2(b4[0] | (b4[1] << 16), b4[2] | (b4[3] << 16));
                s.x += v4[0]; s.y += v4[1]; s.z += v4[2]; s.w += v4[3];
            }
        }
    }
    sm[threadIdx.x] = s;
    __syncthreads();
    if (rsub == 0 && c < d) {
        for (int q = 1; q < RG; ++q) {
            const float4 o = sm[q * CT + threadIdx.x];
            s.x += o.x; s.y += o.y; s.z += o.z; s.w += o.w;
        }
        *reinterpret_cast<float4*>(partial + (int64_t)blockIdx.x * d + c) = s;
    }
}

// gb[c] += sum_b partial[b, c]: a block of 1024 threads owns 32 columns; its 32 row groups walk
// the partial rows 32 apart, eight loads in flight each, and are combined through LDS in a fixed
// order (a partition of 8*10^5 rows leaves 3*10^3 partial rows: with 8 row groups the walk took
// 48 us, bound by the latency of its ~100 dependent steps).
constexpr int kFinishGroups = 32;
__global__ __launch_bounds__(32 * kFinishGroups) void k_colsum_finish(const float* __restrict__ partial,
                                                                      int64_t nblocks, int32_t d,
                                                                      float* __restrict__ gb, int32_t ldp)
{
    __shared__ float sm[kFinishGroups][32];
    const int tx = threadIdx.x % 32, ty = threadIdx.x / 32;
    const int32_t c = blockIdx.x * 32 + tx;
    float s = 0.f;
    if (c < d) {
        constexpr int U = 8;
        for (int64_t b = ty; b < nblocks; b += kFinishGroups * U) {
            float x[U];
#pragma unroll
            for (int u = 0; u < U; ++u)
                x[u] = b + kFinishGroups * u < nblocks ? partial[(b + kFinishGroups * u) * ldp + c] : 0.f;
#pragma unroll
            for (int u = 0; u < U; ++u) s += x[u];
        }
    }
    sm[ty][tx] = s;
    __syncthreads();
    if (ty == 0 && c < d) {
        for (int q = 1; q < kFinishGroups; ++q) s += sm[q][tx];
        gb[c] += s;
    }
}

// Dropout after a hidden layer's activation (training): element (v, j), v an original vertex
// id, draws the upper 32 bits of splitmix64(key + v d + j) and is zeroed when the draw is below
// `threshold`, otherwise multiplied by `scale` = 1 / (1 - p).  Counter-based: the same element
// gets the same draw whatever partition its row is processed in.
__device__ inline unsigned long long splitmix64_dev(unsigned long long x)
{
    unsigned long long z = x + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

template <typename T>
__global__ __launch_bounds__(kBlock) void k_dropout(T* __restrict__ a, const int32_t* __restrict__ orig,
                                                    int64_t rows, int32_t d, unsigned long long key,
                                                    unsigned int threshold, float scale)
{
    const int64_t total = rows * d;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * kBlock) {
        const int64_t r = i / d;
        const int32_t j = (int32_t)(i - r * d);
        const unsigned long long idx = (unsigned long long)orig[r] * (unsigned long long)d + (unsigned long long)j;
        const unsigned int draw = (unsigned int)(splitmix64_dev(key + idx) >> 32);
        if constexpr (sizeof(T) == 4) {
            a[i] = draw < threshold ? 0.f : a[i] * scale;
        } else {
            const float v = draw < threshold ? 0.f : __uint_as_float((uint32_t)a[i] << 16) * scale;
            const uint32_t b = __float_as_uint(v);
            a[i] = (T)((b + 0x7FFFu + ((b >> 16) & 1u)) >> 16);
        }
    }
}

// Epilogue of a transform-first layer: out[r, j] = (accumulate ? out[r, j] : 0) + z[r, j]
// (+ bias[j]), then the activation.  z has row stride ldz >= d (padded to whole 16-byte
// vectors for the aggregation), out has row stride d.
__global__ __launch_bounds__(kBlock) void k_add_padded(float* __restrict__ out, const float* __restrict__ z,
                                                       int64_t rows, int32_t d, int32_t ldz,
                                                       const float* __restrict__ bias, int accumulate,
                                                       int relu, int32_t ldo)
{
    const int64_t total = rows * d;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * kBlock) {
        const int64_t r = i / d;
        const int32_t j = (int32_t)(i - r * d);
        float v = z[r * ldz + j];
        if (accumulate) v += out[r * ldo + j];
        if (bias) v += bias[j];
        if (relu) v = v > 0.f ? v : 0.f;
        out[r * ldo + j] = v;
    }
}

// out[i, j] = bf16(act(z[i, j] + bias[j])): z fp32 with row stride ldz, out bfloat16 with row stride d
__global__ __launch_bounds__(kBlock) void k_bias_act_bf16(uint16_t* __restrict__ out, const float* __restrict__ z,
                                                          int64_t rows, int32_t d, int32_t ldz,
                                                          const float* __restrict__ bias, int relu)
{
    const int64_t total = rows * d;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * kBlock) {
        const int64_t r = i / d;
        const int32_t j = (int32_t)(i - r * d);
        float v = z[r * ldz + j];
        if (bias) v += bias[j];
        if (relu) v = v > 0.f ? v : 0.f;
        const uint32_t u = __float_as_uint(v);
        out[i] = (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
    }
}

// the same, eight columns per thread (d a multiple of 8, z rows 16-byte aligned)
__global__ __launch_bounds__(kBlock) void k_bias_act_bf16_vec(uint4* __restrict__ out, const float* __restrict__ z,
                                                              int64_t rows, int32_t d, int32_t ldz,
                                                              const float* __restrict__ bias, int relu)
{
    const int32_t gpr = d / 8;                       // groups of eight columns per row
    const int64_t total = rows * gpr;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * kBlock) {
        const int64_t r = i / gpr;
        const int32_t j = (int32_t)(i - r * gpr) * 8;
        const float4 a = *reinterpret_cast<const float4*>(z + r * ldz + j);
        const float4 b = *reinterpret_cast<const float4*>(z + r * ldz + j + 4);
        float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        uint32_t h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float x = v[e] + (bias ? bias[j + e] : 0.f);
            if (relu) x = x > 0.f ? x : 0.f;
            const uint32_t u = __float_as_uint(x);
            h[e] = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
        }
        out[i] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
    }
}

// dst[r, 0..ld) = src[r, 0..d) followed by zeros (ld >= d)
__global__ __launch_bounds__(kBlock) void k_pad_rows(float* __restrict__ dst, const float* __restrict__ src,
                                                     int64_t rows, int32_t d, int32_t ld, int32_t lds)
{
    const int64_t total = rows * ld;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * kBlock) {
        const int64_t r = i / ld;
        const int32_t j = (int32_t)(i - r * ld);
        dst[i] = j < d ? src[r * lds + j] : 0.f;
    }
}

// One optimizer step over a parameter tensor of n floats.
// fp32 -> bfloat16, round to nearest even (the rounding of k_to_bf16)
__device__ inline uint16_t bf16_rne(float f)
{
    const uint32_t b = __float_as_uint(f);
    return (uint16_t)((b + 0x7FFFu + ((b >> 16) & 1u)) >> 16);
}

__global__ __launch_bounds__(kBlock) void k_adam(float* __restrict__ w, const float* __restrict__ g,
                                                 float* __restrict__ m, float* __restrict__ v, int64_t n,
                                                 float lr, float beta1, float beta2, float eps,
                                                 float weight_decay, float corr1, float corr2,
                                                 uint16_t* __restrict__ w16)
{
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n) return;
    const float wi = w[i];
    const float gi = g[i] + weight_decay * wi;
    const float mi = beta1 * m[i] + (1.f - beta1) * gi;
    const float vi = beta2 * v[i] + (1.f - beta2) * gi * gi;
    m[i] = mi;
    v[i] = vi;
    const float wn = wi - lr * (mi * corr1) / (sqrtf(vi * corr2) + eps);
    w[i] = wn;
    if (w16) w16[i] = bf16_rne(wn);
}

__global__ __launch_bounds__(kBlock) void k_sgd(float* __restrict__ w, const float* __restrict__ g,
                                                int64_t n, float lr, float weight_decay,
                                                uint16_t* __restrict__ w16)
{
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n) return;
    const float wi = w[i];
    const float wn = wi - lr * (g[i] + weight_decay * wi);
    w[i] = wn;
    if (w16) w16[i] = bf16_rne(wn);
}

}  // namespace

int64_t loss_partial_floats(int64_t n, int32_t k) { return n / (kLossRowsPerWave * (kBlock / kWave)) + k + 2; }

void launch_count_mask(const uint8_t* mask, int64_t n, unsigned long long* count_dev, hipStream_t s)
{
    launch_fill_zero(count_dev, sizeof(unsigned long long), s);
    int64_t cb = (n + kBlock * 64 - 1) / (kBlock * 64);
    hipLaunchKernelGGL(k_count_mask, dim3((unsigned)(cb < 1 ? 1 : cb)), dim3(kBlock), 0, s, mask, n,
                       count_dev);
}

int64_t launch_loss_rows(const float* logits, const int32_t* labels, const uint8_t* mask, float* grad,
                         int64_t rows, int32_t c, const unsigned long long* count_dev, float* partial,
                         hipStream_t s)
{
    if (rows <= 0) return 0;
    const int64_t rpb = kLossRowsPerWave * (kBlock / kWave);
    const int64_t blocks = (rows + rpb - 1) / rpb;
    hipLaunchKernelGGL(k_loss, dim3((unsigned)blocks), dim3(kBlock), 0, s, logits, labels, mask,
                       grad, rows, c, count_dev, partial);
    return blocks;
}

void launch_loss_finish(const float* partial, int64_t nparts, const unsigned long long* count_dev,
                        float* loss_dev, hipStream_t s)
{
    hipLaunchKernelGGL(k_loss_finish, dim3(1), dim3(kBlock), 0, s, partial, nparts, count_dev, loss_dev);
}

void launch_loss(const float* logits, const int32_t* labels, const uint8_t* mask, float* grad,
                 int64_t n, int32_t c, const int64_t* part_off, int32_t k, unsigned long long* count_dev,
                 float* partial, float* loss_dev, hipStream_t s)
{
    launch_count_mask(mask, n, count_dev, s);
    // partition by partition, so that the block partial sums group the rows exactly as the
    // streaming schedule does (which sees one partition block at a time): same bits in both
    int64_t blocks = 0;
    for (int32_t p = 0; p < k; ++p) {
        const int64_t r0 = part_off[p], np = part_off[p + 1] - r0;
        blocks += launch_loss_rows(logits + r0 * c, labels + r0, mask + r0, grad + r0 * c, np, c, count_dev,
                                   partial + blocks, s);
    }
    launch_loss_finish(partial, blocks, count_dev, loss_dev, s);
}

// ---- loss without a caller workspace --------------------------------------------------------
// The loss kernels need |M| (8 bytes) and one partial sum per block of 64 rows.  This array
// stands in for the caller's workspace when the caller cannot provide or allocate one.  Every
// device the library runs on holds its own copy for the life of the process; host code never
// uses the array's name as an address, only the per-device pointer looked up below.
constexpr int64_t kStaticScratchBytes = 4 << 20;
constexpr int64_t kStaticPartialOffset = 256;          // bytes; |M| sits at offset 0
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
void* g_static_ptr[kMaxDevices] = {};
}  // namespace

int64_t loss_static_max_partials() { return (kStaticScratchBytes - kStaticPartialOffset) / (int64_t)sizeof(float); }

hipError_t launch_loss_static(const float* logits, const int32_t* labels, const uint8_t* mask, float* grad,
                              int64_t n, int32_t c, const int64_t* part_off, int32_t k, float* loss_dev,
                              hipStream_t s)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (!g_static_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_static_ptr[dev] = ptr;
    }
    char* base = static_cast<char*>(g_static_ptr[dev]);
    unsigned long long* count_dev = reinterpret_cast<unsigned long long*>(base);
    float* partial = reinterpret_cast<float*>(base + kStaticPartialOffset);
    // the count is cleared by a fill kernel inside launch_loss; the partial sums of this call's
    // blocks are all overwritten before the last kernel reads exactly that many
    launch_loss(logits, labels, mask, grad, n, c, part_off, k, count_dev, partial, loss_dev, s);
    return hipGetLastError();
}

int64_t act_bwd_partial_floats(int64_t rows, int32_t d)
{
    return ((rows + kRowsPerBlockAct - 1) / kRowsPerBlockAct) * (int64_t)d;
}

void launch_act_bwd(const float* g, const float* act, float* dy, int64_t rows, int32_t d,
                    float* gb, float* partial, float scale, hipStream_t s, const uint8_t* row_on)
{
    if (!act) scale = 1.f;
    if (act) row_on = nullptr;                  // dy is written for every row
    if (rows <= 0) return;
    const int64_t blocks = (rows + kRowsPerBlockAct - 1) / kRowsPerBlockAct;
    if (!act && !gb) return;
    const bool vec = d % 4 == 0 && ((reinterpret_cast<uintptr_t>(g) | reinterpret_cast<uintptr_t>(act) |
                                     reinterpret_cast<uintptr_t>(dy) |
                                     reinterpret_cast<uintptr_t>(partial)) & 15) == 0;
    if (vec)
        hipLaunchKernelGGL(k_act_bwd_vec, dim3((unsigned)blocks), dim3(kBlock), 0, s, g, act, dy, rows,
                           d, partial, scale, row_on);
    else
        hipLaunchKernelGGL(k_act_bwd, dim3((unsigned)blocks), dim3(kBlock), 0, s, g, act, dy, rows, d,
                           partial, scale, row_on);
    if (gb)
        hipLaunchKernelGGL(k_colsum_finish, dim3((unsigned)((d + 31) / 32)), dim3(32 * kFinishGroups),
                           0, s, (const float*)partial, blocks, d, gb, d);
}

void launch_act_bwd_bf16(const float* g, const void* act, void* dy, int64_t rows, int32_t d,
                         float* gb, float* partial, float scale, hipStream_t s)
{
    if (rows <= 0) return;
    if (!act) scale = 1.f;
    const int64_t blocks = (rows + kRowsPerBlockAct - 1) / kRowsPerBlockAct;
    const bool vec = d % 4 == 0 && (reinterpret_cast<uintptr_t>(g) & 15) == 0 &&
                     (reinterpret_cast<uintptr_t>(partial) & 15) == 0 &&
                     ((reinterpret_cast<uintptr_t>(act) | reinterpret_cast<uintptr_t>(dy)) & 7) == 0;
    if (vec)
        hipLaunchKernelGGL(k_act_bwd_bf16_vec, dim3((unsigned)blocks, (unsigned)((d / 4 + 63) / 64)), dim3(kBlock),
                           0, s, g, (const uint16_t*)act, (uint16_t*)dy, rows, d, partial, scale);
    else
        hipLaunchKernelGGL(k_act_bwd_bf16, dim3((unsigned)blocks), dim3(kBlock), 0, s, g,
                           (const uint16_t*)act, (uint16_t*)dy, rows, d, partial, scale);
    if (gb)
        hipLaunchKernelGGL(k_colsum_finish, dim3((unsigned)((d + 31) / 32)), dim3(32 * kFinishGroups), 0, s,
                           (const float*)partial, blocks, d, gb, d);
}

void launch_dropout(void* a, int is_bf16, const int32_t* orig_of_row, int64_t rows, int32_t d,
                    uint64_t key, uint32_t threshold, float scale, hipStream_t s)
{
    if (rows <= 0 || d <= 0) return;
    int64_t blocks = (rows * d + kBlock - 1) / kBlock;
    if (blocks > 65536) blocks = 65536;
    if (is_bf16)
        hipLaunchKernelGGL(k_dropout<uint16_t>, dim3((unsigned)blocks), dim3(kBlock), 0, s, (uint16_t*)a,
                           orig_of_row, rows, d, (unsigned long long)key, threshold, scale);
    else
        hipLaunchKernelGGL(k_dropout<float>, dim3((unsigned)blocks), dim3(kBlock), 0, s, (float*)a,
                           orig_of_row, rows, d, (unsigned long long)key, threshold, scale);
}

void launch_colsum_finish(const float* partial, int64_t nblocks, int32_t d, float* out, hipStream_t s, int32_t ldp)
{
    if (nblocks <= 0 || d <= 0) return;
    hipLaunchKernelGGL(k_colsum_finish, dim3((unsigned)((d + 31) / 32)), dim3(32 * kFinishGroups), 0, s, partial, nblocks,
                       d, out, ldp > 0 ? ldp : d);
}

void launch_add_padded(float* out, const float* z, int64_t rows, int32_t d, int32_t ldz,
                       const float* bias, int accumulate, int relu, hipStream_t s, int32_t ldo)
{
    if (rows <= 0 || d <= 0) return;
    int64_t blocks = (rows * d + kBlock - 1) / kBlock;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(k_add_padded, dim3((unsigned)blocks), dim3(kBlock), 0, s, out, z, rows, d, ldz, bias,
                       accumulate, relu, ldo > 0 ? ldo : d);
}

void launch_bias_act_bf16(void* out, const float* z, int64_t rows, int32_t d, int32_t ldz, const float* bias,
                          int relu, hipStream_t s)
{
    if (rows <= 0 || d <= 0) return;
    if (d % 8 == 0 && ldz % 4 == 0 && (reinterpret_cast<uintptr_t>(out) & 15) == 0 &&
        (reinterpret_cast<uintptr_t>(z) & 15) == 0) {
        int64_t blocks = (rows * (d / 8) + kBlock - 1) / kBlock;
        if (blocks > 65536) blocks = 65536;
        hipLaunchKernelGGL(k_bias_act_bf16_vec, dim3((unsigned)blocks), dim3(kBlock), 0, s, (uint4*)out, z, rows, d,
                           ldz, bias, relu);
        return;
    }
    int64_t blocks = (rows * d + kBlock - 1) / kBlock;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(k_bias_act_bf16, dim3((unsigned)blocks), dim3(kBlock), 0, s, (uint16_t*)out, z, rows, d,
                       ldz, bias, relu);
}

void launch_pad_rows(float* dst, const float* src, int64_t rows, int32_t d, int32_t ld, hipStream_t s, int32_t lds)
{
    if (rows <= 0 || ld <= 0) return;
    int64_t blocks = (rows * ld + kBlock - 1) / kBlock;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(k_pad_rows, dim3((unsigned)blocks), dim3(kBlock), 0, s, dst, src, rows, d, ld, lds > 0 ? lds : d);
}

void launch_adam(float* w, const float* g, float* m, float* v, int64_t n, float lr, float beta1,
                 float beta2, float eps, float weight_decay, float corr1, float corr2, hipStream_t s,
                 void* w16)
{
    if (n <= 0) return;
    hipLaunchKernelGGL(k_adam, dim3((unsigned)((n + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, w, g, m, v,
                       n, lr, beta1, beta2, eps, weight_decay, corr1, corr2, (uint16_t*)w16);
}

void launch_sgd(float* w, const float* g, int64_t n, float lr, float weight_decay, hipStream_t s, void* w16)
{
    if (n <= 0) return;
    hipLaunchKernelGGL(k_sgd, dim3((unsigned)((n + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, w, g, n, lr,
                       weight_decay, (uint16_t*)w16);
}

}  // namespace gnnmi
