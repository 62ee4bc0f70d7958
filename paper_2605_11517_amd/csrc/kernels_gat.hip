// Kernels of the graph-attention layers (LeakyReLU slope 0.2; Velickovic et al.,
// the model family the paper evaluates next to GCN and GraphSAGE).  A layer transforms first:
// H = A^{l-1} W, s_src = H a_src, s_dst = H a_dst per vertex; a partition then gathers the rows
// of H and the scores s_src of its boundary vertices, computes the attention weight of every
// entry of T_p and aggregates with them (the aggregation kernel of the other models, with the
// attention weights as entry weights).  The backward pass regathers, recomputes the attention
// weights and needs one more edge-wise kernel: the dot product dY[v] . H[u] per entry.
//
// Several heads: the per-vertex scores of all heads of a vertex lie side by side (nh floats per
// vertex, so one fetch of a neighbour's scores serves every head), the per-entry arrays (attention
// weights, edge-wise products) are kept head after head, `hs` floats apart, and the row-wise
// passes take the heads of a row in blocks of up to four.
//
// Row-wise scalar passes: a wavefront takes a range item of short rows - rows of up to 128
// entries four at a time, a group of 16 lanes each, longer ones one after the other with the
// whole wavefront; long rows (more than 512 entries) are cut into the aggregation kernel's
// segments, one wavefront per segment, and combined per row in segment order.  All reductions
// are shuffles and fixed-order sums, so results are reproducible.
#include "gnn_internal.h"

namespace gnnmi {
namespace {

constexpr int kWave = 64;
constexpr int kBlock = 256;
constexpr float kSlope = 0.2f;

__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) v += __shfl_xor(v, m, kWave);
    return v;
}
__device__ inline float wave_max(float v)
{
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) v = fmaxf(v, __shfl_xor(v, m, kWave));
    return v;
}
// BLOCK: every thread of the workgroup calls these the same number of times
template <bool BLOCK> __device__ inline float red_sum(float v, float* sm)
{
    v = wave_sum(v);
    if (!BLOCK) return v;
    __syncthreads();
    if (threadIdx.x % kWave == 0) sm[threadIdx.x / kWave] = v;
    __syncthreads();
    return (sm[0] + sm[1]) + (sm[2] + sm[3]);
}
struct GatRows {
    const int64_t* rp;          // row pointers of the partition's rows (absolute positions)
    const int32_t* col;         // local columns (absolute positions)
    int64_t e0;                 // first absolute position of the partition
    int64_t n_own;
    const float* ssrc_own;      // s_src of the partition's own rows, nh floats per row
    const float* ssrc_bnd;      // s_src of its boundary rows (staged), nh floats per row
    const float* sdst_own;      // nh floats per row
    int32_t nh;                 // heads
    int64_t hs;                 // floats between two heads' per-entry arrays
    // work decomposition
    const int32_t* range_rows;
    int64_t nranges;
    const int32_t* long_row;
    int64_t nlong;
    __device__ float ssrc(int32_t c, int32_t h) const
    {
        return c < n_own ? ssrc_own[(int64_t)c * nh + h] : ssrc_bnd[(int64_t)(c - n_own) * nh + h];
    }
};

__device__ inline float lrelu(float x) { return x > 0.f ? x : kSlope * x; }

// head h = blockIdx.y: s_src[r nh + h] = H_h[r,:] . a_src_h, s_dst[r nh + h] = H_h[r,:] . a_dst_h with
// H_h = H + h head_off (rows ld floats apart) and the head's f entries of the attention vectors;
// one wavefront per row and head
__global__ __launch_bounds__(kBlock) void k_gat_scores(const float* __restrict__ H, int32_t ld, int32_t f,
                                                       int64_t rows, const float* __restrict__ a_src,
                                                       const float* __restrict__ a_dst,
                                                       float* __restrict__ ssrc, float* __restrict__ sdst,
                                                       int32_t nh, int64_t head_off)
{
    const int lane = threadIdx.x % kWave;
    const int64_t r = (int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
    if (r >= rows) return;
    const int32_t hd = blockIdx.y;
    H += hd * head_off;
    a_src += hd * f;
    a_dst += hd * f;
    ssrc += hd;
    sdst += hd;
    float s1 = 0.f, s2 = 0.f;
    for (int j = lane; j < f; j += kWave) {
        const float h = H[r * ld + j];
        s1 += h * a_src[j];
        s2 += h * a_dst[j];
    }
    s1 = wave_sum(s1);
    s2 = wave_sum(s2);
    if (lane == 0) {
        ssrc[r * nh] = s1;
        sdst[r * nh] = s2;
    }
}

// attention weights of one short row (at most kSpmmSegment = 8 x 64 entries):
// att[e - e0] = softmax over the row's entries of LeakyReLU(s_src(col) + s_dst(row)).  Every
// lane keeps its up to eight scores in registers, so the scores are gathered once.
constexpr int kPerLane = kSpmmSegment / kWave;

// The row-wise passes take HB heads of a row at a time (h0 .. h0 + HB - 1, those below nh):
// the scores of the HB heads of a neighbour lie side by side and are fetched together (VEC: as
// one 16-byte vector; needs HB = 4 and nh a multiple of 4), and the HB reductions run beside
// each other instead of one after the other.
// The same for heads lying side by side in rows of nh f floats, f a power of two between 4 and
// 256: one wavefront per row reads the whole row (a 16-byte vector per lane and 256-column block)
// and the f / 4 lanes of a head add up their products.
__global__ __launch_bounds__(kBlock) void k_gat_scores_side(const float* __restrict__ H, int32_t ld, int32_t f,
                                                            int64_t rows, const float* __restrict__ a_src,
                                                            const float* __restrict__ a_dst,
                                                            float* __restrict__ ssrc, float* __restrict__ sdst,
                                                            int32_t nh)
{
    const int lane = threadIdx.x % kWave;
    const int64_t r = (int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
    if (r >= rows) return;
    const int32_t d = nh * f;
    const int gl = f / 4;                       // lanes per head
    for (int32_t c0 = 0; c0 < d; c0 += 4 * kWave) {
        const int32_t c = c0 + 4 * lane;
        float s1 = 0.f, s2 = 0.f;
        if (c < d) {
            const float4 h = *reinterpret_cast<const float4*>(H + r * ld + c);
            const float4 as = *reinterpret_cast<const float4*>(a_src + c);
            const float4 ad = *reinterpret_cast<const float4*>(a_dst + c);
            s1 = (h.x * as.x + h.y * as.y) + (h.z * as.z + h.w * as.w);
            s2 = (h.x * ad.x + h.y * ad.y) + (h.z * ad.z + h.w * ad.w);
        }
        for (int m = 1; m < gl; m <<= 1) {
            s1 += __shfl_xor(s1, m, kWave);
            s2 += __shfl_xor(s2, m, kWave);
        }
        if (c < d && lane % gl == 0) {
            ssrc[r * nh + c / f] = s1;
            sdst[r * nh + c / f] = s2;
        }
    }
}

template <int HB, bool VEC>
__device__ inline void load_scores(const GatRows& g, int32_t c, int32_t h0, int nhb, float (&out)[HB])
{
    const float* p = c < g.n_own ? g.ssrc_own + (int64_t)c * g.nh + h0
                                 : g.ssrc_bnd + (int64_t)(c - g.n_own) * g.nh + h0;
    if (VEC) {
        static_assert(!VEC || HB == 4, "vector loads take four heads");
        const float4 v = *reinterpret_cast<const float4*>(p);
        out[0] = v.x; out[1 % HB] = v.y; out[2 % HB] = v.z; out[3 % HB] = v.w;
    } else {
#pragma unroll
        for (int b = 0; b < HB; ++b) out[b] = b < nhb ? p[b] : 0.f;
    }
}

template <int HB, bool VEC>
__device__ inline void att_row_wave(const GatRows& g, int32_t row, int32_t h0, float* __restrict__ att_all)
{
    const int t = threadIdx.x % kWave;
    const int nhb = g.nh - h0 < HB ? g.nh - h0 : HB;
    const int64_t eb = g.rp[row], ee = g.rp[row + 1];
    const int niter = (int)((ee - eb + kWave - 1) / kWave);
    float sd[HB], m[HB];
#pragma unroll
    for (int b = 0; b < HB; ++b) {
        sd[b] = b < nhb ? g.sdst_own[(int64_t)row * g.nh + h0 + b] : 0.f;
        m[b] = -INFINITY;
    }
    float x[HB][kPerLane];
#pragma unroll
    for (int i = 0; i < kPerLane; ++i) {
#pragma unroll
        for (int b = 0; b < HB; ++b) x[b][i] = -INFINITY;
        if (i < niter) {
            const int64_t e = eb + t + (int64_t)i * kWave;
            if (e < ee) {
                float sc[HB];
                load_scores<HB, VEC>(g, g.col[e], h0, nhb, sc);
#pragma unroll
                for (int b = 0; b < HB; ++b) x[b][i] = lrelu(sc[b] + sd[b]);
            }
#pragma unroll
            for (int b = 0; b < HB; ++b) m[b] = fmaxf(m[b], x[b][i]);
        }
    }
    float s[HB];
#pragma unroll
    for (int b = 0; b < HB; ++b) {
        m[b] = wave_max(m[b]);
        s[b] = 0.f;
    }
#pragma unroll
    for (int i = 0; i < kPerLane; ++i)
        if (i < niter) {
#pragma unroll
            for (int b = 0; b < HB; ++b) {
                x[b][i] = expf(x[b][i] - m[b]);          // exp(-inf) = 0 for the lanes past the row end
                s[b] += x[b][i];
            }
        }
#pragma unroll
    for (int b = 0; b < HB; ++b) s[b] = 1.f / wave_sum(s[b]);
#pragma unroll
    for (int i = 0; i < kPerLane; ++i)
        if (i < niter) {
            const int64_t e = eb + t + (int64_t)i * kWave;
            if (e < ee) {
#pragma unroll
                for (int b = 0; b < HB; ++b)
                    if (b < nhb) att_all[(h0 + b) * g.hs + (e - g.e0)] = x[b][i] * s[b];
            }
        }
}

// after the edge-wise dot products dal[e] = dY[row] . H[col]: t = sum att dal;
// dpre[e] = att (dal - t) LeakyReLU'(x)  (gradient of the pre-activation score);
// gs_dst[row] = sum of those.  The pairs (att, dpre) of an entry are written side by side for
// all heads, pair[((e - e0) nh + h) 2 + {0, 1}]: the transposed pass fetches an entry's values by
// position, and finds those of every head in one place.
template <int HB, bool VEC>
__device__ inline void bwd_row_wave(const GatRows& g, int32_t row, int32_t h0, const float* __restrict__ att_all,
                                    const float* __restrict__ dal_all, float* __restrict__ pair,
                                    float* __restrict__ gs_dst_own)
{
    static_assert(HB == 1 || HB == 2 || HB == 4, "blocks of one, two or four heads");
    const int t = threadIdx.x % kWave;
    const int nhb = g.nh - h0 < HB ? g.nh - h0 : HB;
    const int64_t eb = g.rp[row], ee = g.rp[row + 1];
    const int niter = (int)((ee - eb + kWave - 1) / kWave);
    float sd[HB], tv[HB];
    unsigned pos[HB];           // bit i: the score of the lane's i-th entry is positive
#pragma unroll
    for (int b = 0; b < HB; ++b) {
        sd[b] = b < nhb ? g.sdst_own[(int64_t)row * g.nh + h0 + b] : 0.f;
        tv[b] = 0.f;
        pos[b] = 0u;
    }
    float a[HB][kPerLane], d[HB][kPerLane];
#pragma unroll
    for (int i = 0; i < kPerLane; ++i) {
#pragma unroll
        for (int b = 0; b < HB; ++b) { a[b][i] = 0.f; d[b][i] = 0.f; }
        if (i < niter) {
            const int64_t e = eb + t + (int64_t)i * kWave;
            if (e < ee) {
                float sc[HB];
                load_scores<HB, VEC && HB == 4>(g, g.col[e], h0, nhb, sc);
#pragma unroll
                for (int b = 0; b < HB; ++b)
                    if (b < nhb) {
                        a[b][i] = att_all[(h0 + b) * g.hs + (e - g.e0)];
                        d[b][i] = dal_all[(h0 + b) * g.hs + (e - g.e0)];
                        if (sc[b] + sd[b] > 0.f) pos[b] |= 1u << i;
                    }
            }
#pragma unroll
            for (int b = 0; b < HB; ++b) tv[b] += a[b][i] * d[b][i];
        }
    }
    float ds[HB];
#pragma unroll
    for (int b = 0; b < HB; ++b) {
        tv[b] = wave_sum(tv[b]);
        ds[b] = 0.f;
    }
#pragma unroll
    for (int i = 0; i < kPerLane; ++i)
        if (i < niter) {
            const int64_t e = eb + t + (int64_t)i * kWave;
            float dp[HB];
#pragma unroll
            for (int b = 0; b < HB; ++b) {
                dp[b] = a[b][i] * (d[b][i] - tv[b]) * ((pos[b] >> i) & 1u ? 1.f : kSlope);
                ds[b] += dp[b];
            }
            if (e < ee) {
                float* q = pair + ((e - g.e0) * g.nh + h0) * 2;
                if (VEC) {          // whole blocks of an even number of heads: 16-byte stores
#pragma unroll
                    for (int b = 0; b + 1 < HB; b += 2)
                        *reinterpret_cast<float4*>(q + 2 * b) = make_float4(a[b][i], dp[b], a[b + 1][i], dp[b + 1]);
                } else {
#pragma unroll
                    for (int b = 0; b < HB; ++b)
                        if (b < nhb) *reinterpret_cast<float2*>(q + 2 * b) = make_float2(a[b][i], dp[b]);
                }
            }
        }
#pragma unroll
    for (int b = 0; b < HB; ++b) {
        ds[b] = wave_sum(ds[b]);
        if (t == 0 && b < nhb) gs_dst_own[(int64_t)row * g.nh + h0 + b] = ds[b];
    }
}

// Rows of at most kGroupRow entries: a group of 16 lanes per row, four rows of the range item
// at a time (a wavefront that walks its rows one after the other waits three dependent memory
// round trips per row - row pointer, columns, scores - with nothing else in flight).  Every lane
// of the wavefront runs the same number of row steps; lanes without a row take an empty one.
constexpr int kGroup = 16;
constexpr int kGroupRow = kGroup * kPerLane;      // 128 entries

template <int HB, bool VEC>
__device__ inline void att_rows_groups(const GatRows& g, int32_t r0, int32_t r1, float* __restrict__ att_all)
{
    const int lane = threadIdx.x % kWave, gl = lane % kGroup, grp = lane / kGroup;
    for (int32_t i0 = r0; i0 < r1; i0 += kWave / kGroup) {
        const int32_t row = i0 + grp;
        int64_t eb = 0, ee = 0;
        if (row < r1) {
            eb = g.rp[row];
            ee = g.rp[row + 1];
            if (ee - eb > kGroupRow) ee = eb;           // longer rows: a whole wavefront each, afterwards
        }
        const int niter = (int)((ee - eb + kGroup - 1) / kGroup);
        int32_t cols[kPerLane];
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            const int64_t e = eb + gl + (int64_t)i * kGroup;
            cols[i] = e < ee ? g.col[e] : -1;
        }
        for (int32_t h0 = 0; h0 < g.nh; h0 += HB) {
            const int nhb = g.nh - h0 < HB ? g.nh - h0 : HB;
            float sd[HB], m[HB], sum[HB];
#pragma unroll
            for (int b = 0; b < HB; ++b) {
                sd[b] = (b < nhb && row < r1) ? g.sdst_own[(int64_t)row * g.nh + h0 + b] : 0.f;
                m[b] = -INFINITY;
                sum[b] = 0.f;
            }
            float x[HB][kPerLane];
#pragma unroll
            for (int i = 0; i < kPerLane; ++i) {
#pragma unroll
                for (int b = 0; b < HB; ++b) x[b][i] = -INFINITY;
                if (i < niter && cols[i] >= 0) {
                    float sc[HB];
                    load_scores<HB, VEC>(g, cols[i], h0, nhb, sc);
#pragma unroll
                    for (int b = 0; b < HB; ++b) x[b][i] = lrelu(sc[b] + sd[b]);
                }
#pragma unroll
                for (int b = 0; b < HB; ++b) m[b] = fmaxf(m[b], x[b][i]);
            }
#pragma unroll
            for (int b = 0; b < HB; ++b) {
#pragma unroll
                for (int k = 1; k < kGroup; k <<= 1) m[b] = fmaxf(m[b], __shfl_xor(m[b], k, kWave));
            }
#pragma unroll
            for (int i = 0; i < kPerLane; ++i)
                if (i < niter) {
#pragma unroll
                    for (int b = 0; b < HB; ++b) {
                        x[b][i] = expf(x[b][i] - m[b]);      // exp(-inf) = 0 past the row end
                        sum[b] += x[b][i];
                    }
                }
#pragma unroll
            for (int b = 0; b < HB; ++b) {
#pragma unroll
                for (int k = 1; k < kGroup; k <<= 1) sum[b] += __shfl_xor(sum[b], k, kWave);
                sum[b] = 1.f / sum[b];
            }
#pragma unroll
            for (int i = 0; i < kPerLane; ++i)
                if (i < niter && cols[i] >= 0) {
                    const int64_t e = eb + gl + (int64_t)i * kGroup;
#pragma unroll
                    for (int b = 0; b < HB; ++b)
                        if (b < nhb) att_all[(h0 + b) * g.hs + (e - g.e0)] = x[b][i] * sum[b];
                }
        }
    }
}

// The backward scalars of such rows, the same way (see bwd_row_wave for what is computed).
template <int HB, bool VEC>
__device__ inline void bwd_rows_groups(const GatRows& g, int32_t r0, int32_t r1, const float* __restrict__ att_all,
                                       const float* __restrict__ dal_all, float* __restrict__ pair,
                                       float* __restrict__ gs_dst_own)
{
    const int lane = threadIdx.x % kWave, gl = lane % kGroup, grp = lane / kGroup;
    for (int32_t i0 = r0; i0 < r1; i0 += kWave / kGroup) {
        const int32_t row = i0 + grp;
        int64_t eb = 0, ee = 0;
        if (row < r1) {
            eb = g.rp[row];
            ee = g.rp[row + 1];
            if (ee - eb > kGroupRow) ee = eb;           // longer rows: a whole wavefront each, afterwards
        }
        const int niter = (int)((ee - eb + kGroup - 1) / kGroup);
        int32_t cols[kPerLane];
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            const int64_t e = eb + gl + (int64_t)i * kGroup;
            cols[i] = e < ee ? g.col[e] : -1;
        }
        for (int32_t h0 = 0; h0 < g.nh; h0 += HB) {
            const int nhb = g.nh - h0 < HB ? g.nh - h0 : HB;
            float sd[HB], tv[HB], ds[HB];
            unsigned pos[HB];
#pragma unroll
            for (int b = 0; b < HB; ++b) {
                sd[b] = (b < nhb && row < r1) ? g.sdst_own[(int64_t)row * g.nh + h0 + b] : 0.f;
                tv[b] = 0.f;
                ds[b] = 0.f;
                pos[b] = 0u;
            }
            float a[HB][kPerLane], d[HB][kPerLane];
#pragma unroll
            for (int i = 0; i < kPerLane; ++i) {
#pragma unroll
                for (int b = 0; b < HB; ++b) { a[b][i] = 0.f; d[b][i] = 0.f; }
                if (i < niter && cols[i] >= 0) {
                    const int64_t e = eb + gl + (int64_t)i * kGroup;
                    float sc[HB];
                    load_scores<HB, VEC && HB == 4>(g, cols[i], h0, nhb, sc);
#pragma unroll
                    for (int b = 0; b < HB; ++b)
                        if (b < nhb) {
                            a[b][i] = att_all[(h0 + b) * g.hs + (e - g.e0)];
                            d[b][i] = dal_all[(h0 + b) * g.hs + (e - g.e0)];
                            if (sc[b] + sd[b] > 0.f) pos[b] |= 1u << i;
                        }
                }
#pragma unroll
                for (int b = 0; b < HB; ++b) tv[b] += a[b][i] * d[b][i];
            }
#pragma unroll
            for (int b = 0; b < HB; ++b) {
#pragma unroll
                for (int k = 1; k < kGroup; k <<= 1) tv[b] += __shfl_xor(tv[b], k, kWave);
            }
#pragma unroll
            for (int i = 0; i < kPerLane; ++i)
                if (i < niter) {
                    float dp[HB];
#pragma unroll
                    for (int b = 0; b < HB; ++b) {
                        dp[b] = a[b][i] * (d[b][i] - tv[b]) * ((pos[b] >> i) & 1u ? 1.f : kSlope);
                        ds[b] += dp[b];
                    }
                    if (cols[i] >= 0) {
                        const int64_t e = eb + gl + (int64_t)i * kGroup;
                        float* q = pair + ((e - g.e0) * g.nh + h0) * 2;
                        if (VEC) {
#pragma unroll
                            for (int b = 0; b + 1 < HB; b += 2)
                                *reinterpret_cast<float4*>(q + 2 * b) =
                                    make_float4(a[b][i], dp[b], a[b + 1][i], dp[b + 1]);
                        } else {
#pragma unroll
                            for (int b = 0; b < HB; ++b)
                                if (b < nhb) *reinterpret_cast<float2*>(q + 2 * b) = make_float2(a[b][i], dp[b]);
                        }
                    }
                }
#pragma unroll
            for (int b = 0; b < HB; ++b) {
#pragma unroll
                for (int k = 1; k < kGroup; k <<= 1) ds[b] += __shfl_xor(ds[b], k, kWave);
                if (gl == 0 && b < nhb && ee > eb) gs_dst_own[(int64_t)row * g.nh + h0 + b] = ds[b];
            }
        }
    }
}

// MODE 0: attention weights; MODE 1: backward scalars.  One range item of short rows per
// wavefront; long rows are skipped here and handled segment by segment below.
template <int MODE, int HB, bool VEC>
__global__ __launch_bounds__(kBlock) void k_gat_rows(const GatRows g, float* __restrict__ att,
                                                     float* __restrict__ dal, float* __restrict__ pair,
                                                     float* __restrict__ gs_dst_own)
{
    const int64_t item = (int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
    if (item >= g.nranges) return;
    const int32_t r1 = g.range_rows[item + 1];
    if constexpr (MODE == 0) att_rows_groups<HB, VEC>(g, g.range_rows[item], r1, att);
    else bwd_rows_groups<HB, VEC>(g, g.range_rows[item], r1, att, dal, pair, gs_dst_own);
    for (int32_t row = g.range_rows[item]; row < r1; ++row) {
        const int64_t len = g.rp[row + 1] - g.rp[row];
        if (len > kSpmmSegment || len <= kGroupRow) continue;
        for (int32_t h0 = 0; h0 < g.nh; h0 += HB) {
            if constexpr (MODE == 0) att_row_wave<HB, VEC>(g, row, h0, att);
            else bwd_row_wave<HB, VEC>(g, row, h0, att, dal, pair, gs_dst_own);
        }
    }
}

// ---- long rows, segment-parallel --------------------------------------------------------------
// A long row is cut into segments of at most kSpmmSegment entries (the aggregation kernel's work
// items); one wavefront handles one segment with its entries in registers, a second small
// kernel combines the segments of each row in segment order, a third applies the result.
struct GatSegs {
    const int32_t* seg_row;
    const int64_t* seg_begin;
    const int32_t* seg_len;
    int64_t nsegs;
    const int32_t* long_row;
    const int32_t* long_first;
    const int32_t* long_nseg;
    int64_t nlong;
};

// STEP 0: per segment local max m and sum of exp(x - m); att <- exp(x - m)
// STEP 1: att *= factor[segment]
// STEP 2: per segment sum of att * dal
// STEP 3: dpre = att (dal - t[segment]) LeakyReLU'(x) written beside att into `pair` (see
//         bwd_row_wave); per segment sum of those
// Per-entry arrays of head h lie hs floats on, per-segment arrays 2 nsegs (stat) / nsegs (factor)
// floats on.  Steps 0 and 3 take the heads in blocks of HB as the row-wise passes do.
template <int STEP, int HB, bool VEC>
__global__ __launch_bounds__(kBlock) void k_gat_segments(const GatRows g, const GatSegs q,
                                                         float* __restrict__ att_all, float* __restrict__ dal_all,
                                                         float* __restrict__ stat_all,
                                                         const float* __restrict__ factor_all,
                                                         float* __restrict__ pair)
{
    const int t = threadIdx.x % kWave;
    const int64_t sgi = (int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
    if (sgi >= q.nsegs) return;
    const int32_t row = q.seg_row[sgi];
    const int64_t eb = q.seg_begin[sgi], ee = eb + q.seg_len[sgi];
    if constexpr (STEP == 0) {
        for (int32_t h0 = 0; h0 < g.nh; h0 += HB) {
            const int nhb = g.nh - h0 < HB ? g.nh - h0 : HB;
            float sd[HB], m[HB], sum[HB];
#pragma unroll
            for (int b = 0; b < HB; ++b) {
                sd[b] = b < nhb ? g.sdst_own[(int64_t)row * g.nh + h0 + b] : 0.f;
                m[b] = -INFINITY;
                sum[b] = 0.f;
            }
            float x[HB][kPerLane];
#pragma unroll
            for (int i = 0; i < kPerLane; ++i) {
                const int64_t e = eb + t + (int64_t)i * kWave;
#pragma unroll
                for (int b = 0; b < HB; ++b) x[b][i] = -INFINITY;
                if (e < ee) {
                    float sc[HB];
                    load_scores<HB, VEC>(g, g.col[e], h0, nhb, sc);
#pragma unroll
                    for (int b = 0; b < HB; ++b) x[b][i] = lrelu(sc[b] + sd[b]);
                }
#pragma unroll
                for (int b = 0; b < HB; ++b) m[b] = fmaxf(m[b], x[b][i]);
            }
#pragma unroll
            for (int b = 0; b < HB; ++b) m[b] = wave_max(m[b]);
#pragma unroll
            for (int i = 0; i < kPerLane; ++i) {
                const int64_t e = eb + t + (int64_t)i * kWave;
#pragma unroll
                for (int b = 0; b < HB; ++b) {
                    const float ex = expf(x[b][i] - m[b]);
                    if (e < ee && b < nhb) att_all[(h0 + b) * g.hs + (e - g.e0)] = ex;
                    sum[b] += ex;
                }
            }
#pragma unroll
            for (int b = 0; b < HB; ++b) {
                sum[b] = wave_sum(sum[b]);
                if (t == 0 && b < nhb) {
                    float* stat = stat_all + (int64_t)(h0 + b) * 2 * q.nsegs;
                    stat[2 * sgi] = m[b];
                    stat[2 * sgi + 1] = sum[b];
                }
            }
        }
    } else if constexpr (STEP == 3) {
        static_assert(STEP != 3 || HB == 1 || HB == 2 || HB == 4, "blocks of one, two or four heads");
        for (int32_t h0 = 0; h0 < g.nh; h0 += HB) {
            const int nhb = g.nh - h0 < HB ? g.nh - h0 : HB;
            float sd[HB], tv[HB], ds[HB];
#pragma unroll
            for (int b = 0; b < HB; ++b) {
                sd[b] = b < nhb ? g.sdst_own[(int64_t)row * g.nh + h0 + b] : 0.f;
                tv[b] = b < nhb ? factor_all[(int64_t)(h0 + b) * q.nsegs + sgi] : 0.f;
                ds[b] = 0.f;
            }
#pragma unroll
            for (int i = 0; i < kPerLane; ++i) {
                const int64_t e = eb + t + (int64_t)i * kWave;
                if (e < ee) {
                    float sc[HB], av[HB], dp[HB];
                    load_scores<HB, VEC && HB == 4>(g, g.col[e], h0, nhb, sc);
#pragma unroll
                    for (int b = 0; b < HB; ++b) {
                        av[b] = 0.f; dp[b] = 0.f;
                        if (b < nhb) {
                            av[b] = att_all[(h0 + b) * g.hs + (e - g.e0)];
                            dp[b] = av[b] * (dal_all[(h0 + b) * g.hs + (e - g.e0)] - tv[b]) *
                                    (sc[b] + sd[b] > 0.f ? 1.f : kSlope);
                            ds[b] += dp[b];
                        }
                    }
                    float* qp = pair + ((e - g.e0) * g.nh + h0) * 2;
                    if (VEC) {          // whole blocks of an even number of heads: 16-byte stores
#pragma unroll
                        for (int b = 0; b + 1 < HB; b += 2)
                            *reinterpret_cast<float4*>(qp + 2 * b) = make_float4(av[b], dp[b], av[b + 1], dp[b + 1]);
                    } else {
#pragma unroll
                        for (int b = 0; b < HB; ++b)
                            if (b < nhb) *reinterpret_cast<float2*>(qp + 2 * b) = make_float2(av[b], dp[b]);
                    }
                }
            }
#pragma unroll
            for (int b = 0; b < HB; ++b) {
                ds[b] = wave_sum(ds[b]);
                if (t == 0 && b < nhb) stat_all[(int64_t)(h0 + b) * 2 * q.nsegs + sgi] = ds[b];
            }
        }
    } else {
        for (int32_t h = 0; h < g.nh; ++h) {
            float* __restrict__ att = att_all + h * g.hs;
            if (STEP == 1) {
                const float f = factor_all[(int64_t)h * q.nsegs + sgi];
                for (int64_t e = eb + t; e < ee; e += kWave) att[e - g.e0] *= f;
            } else {
                const float* __restrict__ dal = dal_all + h * g.hs;
                float tv = 0.f;
                for (int64_t e = eb + t; e < ee; e += kWave) tv += att[e - g.e0] * dal[e - g.e0];
                tv = wave_sum(tv);
                if (t == 0) stat_all[(int64_t)h * 2 * q.nsegs + sgi] = tv;
            }
        }
    }
}

// One wavefront per long row, its segments in ascending order, head after head.
// STEP 0: from (m, sum) per segment: factor[segment] = exp(m_seg - M) / S
// STEP 2: factor[segment] = sum of the row's stat (the row's t)
// STEP 3: gs_dst_own[row] = sum of the row's stat
template <int STEP>
__global__ __launch_bounds__(kBlock) void k_gat_combine(const GatSegs q, int32_t nh,
                                                        const float* __restrict__ stat_all,
                                                        float* __restrict__ factor_all,
                                                        float* __restrict__ gs_dst_own)
{
    const int t = threadIdx.x % kWave;
    const int64_t i = (int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
    if (i >= q.nlong) return;
    const int32_t first = q.long_first[i], ns = q.long_nseg[i];
    for (int32_t h = 0; h < nh; ++h) {
        const float* __restrict__ stat = stat_all + (int64_t)h * 2 * q.nsegs;
        float* __restrict__ factor = factor_all ? factor_all + (int64_t)h * q.nsegs : nullptr;
        if (STEP == 0) {
            float M = -INFINITY;
            for (int32_t j = t; j < ns; j += kWave) M = fmaxf(M, stat[2 * (int64_t)(first + j)]);
            M = wave_max(M);
            float S = 0.f;
            for (int32_t j = t; j < ns; j += kWave)
                S += stat[2 * (int64_t)(first + j) + 1] * expf(stat[2 * (int64_t)(first + j)] - M);
            S = wave_sum(S);
            const float inv = 1.f / S;
            for (int32_t j = t; j < ns; j += kWave) factor[first + j] = expf(stat[2 * (int64_t)(first + j)] - M) * inv;
        } else {
            float v = 0.f;
            for (int32_t j = t; j < ns; j += kWave) v += stat[first + j];
            v = wave_sum(v);
            if (STEP == 2) {
                for (int32_t j = t; j < ns; j += kWave) factor[first + j] = v;
            } else if (t == 0) {
                gs_dst_own[(int64_t)q.long_row[i] * nh + h] = v;
            }
        }
    }
}

// Rows of the transposed operator (the entries of R_p = [own ; boundary] as sources), every head:
// tw_att[h hs + pos - e0] = att of entry tperm[pos] (entry weights of the transposed aggregation)
// and gs_src[(owner row of i) nh + h] += sum over the row of dpre of entry tperm[pos], both read
// from the pairs the backward scalar pass wrote (pair[(entry nh + h) 2 + {0, 1}] = att, dpre: the
// values of all heads of an entry lie in one place, a fetch by position finds them together).
struct GatTRows {
    const int64_t* trp;
    const int32_t* tperm;
    int64_t e0;
    int64_t n_own, base_row;
    const int32_t* bnd;         // library rows of the boundary vertices
    int32_t nh;                 // heads: gs_src holds nh floats per vertex,
    int64_t hs;                 // tw_att one array per head, hs floats apart
    const int32_t* range_rows;
    int64_t nranges;
};
// Long transposed rows (a hub as a source: up to 10^5 destinations in one partition) are cut
// into the aggregation's segments like the long forward rows: one wavefront per segment and all
// heads, then one wavefront per row adds the segments' sums in segment order.  (A workgroup per
// row walked a hub's entries in a hundred dependent steps: 245 us per launch, whatever the heads.)
__global__ __launch_bounds__(kBlock) void k_gat_tsegs(const GatTRows g, const GatSegs q,
                                                      const float* __restrict__ pair, float* __restrict__ tw_att,
                                                      float* __restrict__ stat)
{
    const int t = threadIdx.x % kWave;
    const int64_t sgi = (int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
    if (sgi >= q.nsegs) return;
    const int64_t eb = q.seg_begin[sgi], ee = eb + q.seg_len[sgi];
    int32_t fe[kPerLane];
#pragma unroll
    for (int i = 0; i < kPerLane; ++i) {
        const int64_t e = eb + t + (int64_t)i * kWave;
        fe[i] = e < ee ? g.tperm[e] : -1;
    }
    for (int32_t h = 0; h < g.nh; ++h) {
        float2 v[kPerLane];
#pragma unroll
        for (int i = 0; i < kPerLane; ++i)
            v[i] = fe[i] >= 0 ? *reinterpret_cast<const float2*>(pair + ((int64_t)fe[i] * g.nh + h) * 2)
                              : make_float2(0.f, 0.f);
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            const int64_t e = eb + t + (int64_t)i * kWave;
            if (e < ee) tw_att[h * g.hs + e - g.e0] = v[i].x;
            sum += v[i].y;
        }
        sum = wave_sum(sum);
        if (t == 0) stat[(int64_t)h * q.nsegs + sgi] = sum;
    }
}
__global__ __launch_bounds__(kBlock) void k_gat_tcombine(const GatTRows g, const GatSegs q,
                                                         const float* __restrict__ stat, float* __restrict__ gs_src)
{
    const int t = threadIdx.x % kWave;
    const int64_t i = (int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
    if (i >= q.nlong) return;
    const int32_t first = q.long_first[i], ns = q.long_nseg[i], row = q.long_row[i];
    const int64_t r = row < g.n_own ? g.base_row + row : (int64_t)g.bnd[row - g.n_own];
    for (int32_t h = 0; h < g.nh; ++h) {
        float v = 0.f;
        for (int32_t j = t; j < ns; j += kWave) v += stat[(int64_t)h * q.nsegs + first + j];
        v = wave_sum(v);
        if (t == 0) gs_src[r * g.nh + h] += v;
    }
}
// EVEN: nh is even, two heads' pairs are read as one 16-byte vector
template <bool EVEN>
__global__ __launch_bounds__(kBlock) void k_gat_trows(const GatTRows g, const float* __restrict__ pair,
                                                      float* __restrict__ tw_att, float* __restrict__ gs_src)
{
    {
        // transposed rows are short (a source feeds about ten destinations of a partition): a
        // group of 16 lanes takes a row, four rows of the item at a time, four heads at a time
        constexpr int GW = 16, HB = 4;
        const int lane = threadIdx.x % kWave, gl = lane % GW, grp = lane / GW;
        const int64_t item = (int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
        if (item >= g.nranges) return;
        const int32_t r1 = g.range_rows[item + 1];
        // (every lane of the wavefront runs the same number of row steps: the shuffles below
        // need all 64 lanes; lanes without a row take an empty one)
        for (int32_t i0 = g.range_rows[item]; i0 < r1; i0 += kWave / GW) {
            const int32_t i = i0 + grp;
            int64_t eb = 0, ee = 0;
            if (i < r1) {
                eb = g.trp[i];
                ee = g.trp[i + 1];
                if (ee - eb > kSpmmSegment) ee = eb;      // long rows: the other kernel
            }
            for (int32_t h0 = 0; h0 < g.nh; h0 += HB) {
                const int nhb = g.nh - h0 < HB ? g.nh - h0 : HB;
                float sum[HB] = {0.f, 0.f, 0.f, 0.f};
                for (int64_t e = eb + gl; e < ee; e += GW) {
                    const float* q = pair + ((int64_t)g.tperm[e] * g.nh + h0) * 2;
                    float av[HB], dv[HB];
                    if (EVEN) {
#pragma unroll
                        for (int b = 0; b < HB; b += 2) {
                            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                            if (b < nhb) v = *reinterpret_cast<const float4*>(q + 2 * b);
                            av[b] = v.x; dv[b] = v.y; av[b + 1] = v.z; dv[b + 1] = v.w;
                        }
                    } else {
#pragma unroll
                        for (int b = 0; b < HB; ++b) {
                            float2 v = make_float2(0.f, 0.f);
                            if (b < nhb) v = *reinterpret_cast<const float2*>(q + 2 * b);
                            av[b] = v.x; dv[b] = v.y;
                        }
                    }
#pragma unroll
                    for (int b = 0; b < HB; ++b)
                        if (b < nhb) {
                            tw_att[(h0 + b) * g.hs + e - g.e0] = av[b];
                            sum[b] += dv[b];
                        }
                }
#pragma unroll
                for (int b = 0; b < HB; ++b) {
#pragma unroll
                    for (int m = 1; m < GW; m <<= 1) sum[b] += __shfl_xor(sum[b], m, kWave);
                    if (gl == 0 && b < nhb && ee > eb) {
                        const int64_t r = i < g.n_own ? g.base_row + i : (int64_t)g.bnd[i - g.n_own];
                        gs_src[r * g.nh + h0 + b] += sum[b];
                    }
                }
            }
        }
    }
}

// Edge-wise dot products: dal[e - e0] = dY[row,:] . src(col[e])[:] with src the partition's own
// rows of H or the staged boundary rows.  One wavefront per work item (a segment of a long row
// or a range of short rows); the 64 lanes form 64 / G slots of G lanes, a slot handles one entry
// at a time with NV 16-byte vectors per lane and sums its G partial products with shuffles.
struct GatDotArgs {
    const int64_t* rp;
    const int32_t* col;
    int64_t e0, n_own;
    const float* a_rows;
    const float* b_rows;
    const float* dy;            // [n_own, ld]
    int32_t ld;                 // row stride of H, staging and dy (multiple of 4)
    int32_t d;                  // columns of those rows the products run over (multiple of 4)
    float* dal;
    // nslice > 1: one launch for the heads of a layer whose heads lie side by side: workgroup b
    // takes head b % nslice, i.e. columns [head d, (head + 1) d) of every row and the head's array
    // of products, dal_stride floats on (consecutive workgroups, on different XCDs, read different
    // columns of the same source rows)
    int32_t nslice;
    int64_t dal_stride;
    SpmmItems it;
};
template <int G, int NV>
__device__ inline void dot_entries(const GatDotArgs& g, int32_t row, int64_t eb, int64_t ee, int lane)
{
    constexpr int S = kWave / G;
    constexpr int U = 4;
    const int slot = lane / G, gl = lane % G;
    float4 y[NV];
    int cv[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int c = (v * G + gl) * 4;
        cv[v] = c < g.d ? c : -1;
        y[v] = cv[v] >= 0 ? *reinterpret_cast<const float4*>(g.dy + (int64_t)row * g.ld + c)
                          : make_float4(0.f, 0.f, 0.f, 0.f);
        if (cv[v] < 0) cv[v] = 0;
    }
    if (eb >= ee) return;
    // the column indices of a batch are fetched one batch ahead, so that the row loads of a batch
    // do not wait for an index load first
    int32_t cnext[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t ee_u = eb + u * S + slot;
        cnext[u] = g.col[ee_u < ee ? ee_u : ee - 1];
    }
    for (int64_t e = eb; e < ee; e += S * U) {
        float acc[U];
        const float* src[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int32_t c = cnext[u];
            src[u] = c < g.n_own ? g.a_rows + (int64_t)c * g.ld : g.b_rows + ((int64_t)c - g.n_own) * g.ld;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t ee_u = e + S * U + u * S + slot;
            cnext[u] = g.col[ee_u < ee ? ee_u : ee - 1];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            acc[u] = 0.f;
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const float4 h = *reinterpret_cast<const float4*>(src[u] + cv[v]);
                acc[u] += (h.x * y[v].x + h.y * y[v].y) + (h.z * y[v].z + h.w * y[v].w);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float a = acc[u];
#pragma unroll
            for (int m = 1; m < G; m <<= 1) a += __shfl_xor(a, m, kWave);
            const int64_t ee_u = e + u * S + slot;
            if (gl == 0 && ee_u < ee) g.dal[ee_u - g.e0] = a;
        }
    }
}
template <int G, int NV>
__global__ __launch_bounds__(kBlock) void k_gat_dots(GatDotArgs g)
{
    const int lane = threadIdx.x % kWave;
    unsigned blk = blockIdx.x;
    if (g.nslice > 1) {
        const int64_t hd = blk % (unsigned)g.nslice;
        blk /= (unsigned)g.nslice;
        g.a_rows += hd * g.d;
        g.b_rows += hd * g.d;
        g.dy += hd * g.d;
        g.dal += hd * g.dal_stride;
    }
    const int64_t item = (int64_t)blk * (kBlock / kWave) + threadIdx.x / kWave;
    if (item < g.it.nsegs) {
        const int64_t eb = g.it.seg_begin[item];
        dot_entries<G, NV>(g, g.it.seg_row[item], eb, eb + g.it.seg_len[item], lane);
        return;
    }
    const int64_t ri = item - g.it.nsegs;
    if (ri >= g.it.nranges) return;
    const int32_t r1 = g.it.range_rows[ri + 1];
    for (int32_t row = g.it.range_rows[ri]; row < r1; ++row) {
        const int64_t eb = g.rp[row], ee = g.rp[row + 1];
        if (ee - eb > kSpmmSegment) continue;
        dot_entries<G, NV>(g, row, eb, ee, lane);
    }
}

// gH[r, j] += gs_src[r nh] a_src[j] + gs_dst[r nh] a_dst[j] for the rows of one partition (one
// head: its scores are nh floats apart), and the
// per-block partial column sums  sum_r gs_src[r] H[r, j]  (first f columns of `partial` rows) and
// sum_r gs_dst[r] H[r, j]  (next f columns), 256 rows per block.
__global__ __launch_bounds__(kBlock) void k_gat_rank1(float* __restrict__ gH, const float* __restrict__ H,
                                                      int32_t ld, int32_t f, int64_t rows,
                                                      const float* __restrict__ gs_src,
                                                      const float* __restrict__ gs_dst,
                                                      const float* __restrict__ a_src,
                                                      const float* __restrict__ a_dst,
                                                      float* __restrict__ partial, int32_t nh, int32_t fh)
{
    const int64_t r0 = (int64_t)blockIdx.x * 256;
    const int64_t r1 = r0 + 256 < rows ? r0 + 256 : rows;
    for (int32_t j = threadIdx.x; j < f; j += kBlock) {
        const float as = a_src[j], ad = a_dst[j];
        float p1 = 0.f, p2 = 0.f;
        for (int64_t r = r0; r < r1; ++r) {
            const float gs = gs_src[r * nh + j / fh], gd = gs_dst[r * nh + j / fh];
            const float h = H[r * ld + j];
            gH[r * ld + j] += gs * as + gd * ad;
            p1 += gs * h;
            p2 += gd * h;
        }
        partial[(int64_t)blockIdx.x * 2 * f + j] = p1;
        partial[(int64_t)blockIdx.x * 2 * f + f + j] = p2;
    }
}

// The same for rows of at most CW <= 128 columns: the 256 threads form kBlock / CW row groups of
// CW columns, each group takes every (kBlock / CW)-th row of the block's 256, and the groups'
// partial column sums are combined in group order.
template <int CW>
__global__ __launch_bounds__(kBlock) void k_gat_rank1_narrow(float* __restrict__ gH, const float* __restrict__ H,
                                                             int32_t ld, int32_t f, int64_t rows,
                                                             const float* __restrict__ gs_src,
                                                             const float* __restrict__ gs_dst,
                                                             const float* __restrict__ a_src,
                                                             const float* __restrict__ a_dst,
                                                             float* __restrict__ partial, int32_t nh, int32_t fh)
{
    constexpr int RG = kBlock / CW;
    __shared__ float sm[RG][CW][2];
    const int j = threadIdx.x % CW, rgp = threadIdx.x / CW;
    const int64_t r0 = (int64_t)blockIdx.x * 256;
    const int64_t r1 = r0 + 256 < rows ? r0 + 256 : rows;
    float p1 = 0.f, p2 = 0.f;
    if (j < f) {
        const float as = a_src[j], ad = a_dst[j];
        for (int64_t r = r0 + rgp; r < r1; r += RG) {
            const float gs = gs_src[r * nh + j / fh], gd = gs_dst[r * nh + j / fh];
            const float h = H[r * ld + j];
            gH[r * ld + j] += gs * as + gd * ad;
            p1 += gs * h;
            p2 += gd * h;
        }
    }
    sm[rgp][j][0] = p1;
    sm[rgp][j][1] = p2;
    __syncthreads();
    if (rgp == 0 && j < f) {
        for (int q = 1; q < RG; ++q) {
            p1 += sm[q][j][0];
            p2 += sm[q][j][1];
        }
        partial[(int64_t)blockIdx.x * 2 * f + j] = p1;
        partial[(int64_t)blockIdx.x * 2 * f + f + j] = p2;
    }
}

}  // namespace

void launch_gat_scores(const float* H, int32_t ld, int32_t f, int64_t rows, const float* a_src,
                       const float* a_dst, float* ssrc, float* sdst, int32_t nh, int64_t head_off, hipStream_t s)
{
    if (rows <= 0) return;
    const int64_t blocks = (rows + kBlock / kWave - 1) / (kBlock / kWave);
    const bool aligned = ((reinterpret_cast<uintptr_t>(H) | reinterpret_cast<uintptr_t>(a_src) |
                           reinterpret_cast<uintptr_t>(a_dst)) & 15) == 0 && ld % 4 == 0;
    if (nh > 1 && head_off == f && f >= 4 && f <= 256 && (f & (f - 1)) == 0 && aligned) {
        hipLaunchKernelGGL(k_gat_scores_side, dim3((unsigned)blocks), dim3(kBlock), 0, s, H, ld, f, rows, a_src, a_dst,
                           ssrc, sdst, nh);
        return;
    }
    hipLaunchKernelGGL(k_gat_scores, dim3((unsigned)blocks, (unsigned)nh), dim3(kBlock), 0, s, H, ld, f, rows, a_src,
                       a_dst, ssrc, sdst, nh, head_off);
}

static GatRows make_rows(const GatRowsHost& h)
{
    GatRows g;
    g.rp = h.rp; g.col = h.col; g.e0 = h.e0; g.n_own = h.n_own;
    g.ssrc_own = h.ssrc_own; g.ssrc_bnd = h.ssrc_bnd; g.sdst_own = h.sdst_own;
    g.nh = h.nh; g.hs = h.hs;
    g.range_rows = h.items.range_rows; g.nranges = h.items.nranges;
    g.long_row = h.items.long_row; g.nlong = h.items.nlong;
    return g;
}

static GatSegs make_segs(const GatRowsHost& h)
{
    GatSegs q;
    q.seg_row = h.items.seg_row; q.seg_begin = h.items.seg_begin; q.seg_len = h.items.seg_len;
    q.nsegs = h.items.nsegs;
    q.long_row = h.items.long_row; q.long_first = h.items.long_first; q.long_nseg = h.items.long_nseg;
    q.nlong = h.items.nlong;
    return q;
}

// `segwork`: 3 floats per head and segment of the partition's long rows
void launch_gat_attention(const GatRowsHost& h, float* att, float* segwork, hipStream_t s)
{
    const GatRows g = make_rows(h);
    if (g.nranges > 0) {
        const dim3 grid((unsigned)((g.nranges + 3) / 4)), b(kBlock);
        float* none = nullptr;
        if (g.nh == 1) hipLaunchKernelGGL((k_gat_rows<0, 1, false>), grid, b, 0, s, g, att, none, none, none);
        else if (g.nh % 4 == 0) hipLaunchKernelGGL((k_gat_rows<0, 4, true>), grid, b, 0, s, g, att, none, none, none);
        else hipLaunchKernelGGL((k_gat_rows<0, 4, false>), grid, b, 0, s, g, att, none, none, none);
    }
    const GatSegs q = make_segs(h);
    if (q.nsegs > 0 && q.nlong > 0) {
        float* stat = segwork;
        float* factor = segwork + 2 * q.nsegs * g.nh;
        float* none = nullptr;
        const dim3 gs((unsigned)((q.nsegs + 3) / 4)), gl((unsigned)((q.nlong + 3) / 4)), b(kBlock);
        const float* nof = nullptr;
        if (g.nh == 1) hipLaunchKernelGGL((k_gat_segments<0, 1, false>), gs, b, 0, s, g, q, att, none, stat, nof, none);
        else if (g.nh % 4 == 0) hipLaunchKernelGGL((k_gat_segments<0, 4, true>), gs, b, 0, s, g, q, att, none, stat, nof, none);
        else hipLaunchKernelGGL((k_gat_segments<0, 4, false>), gs, b, 0, s, g, q, att, none, stat, nof, none);
        hipLaunchKernelGGL((k_gat_combine<0>), gl, b, 0, s, q, g.nh, (const float*)stat, factor, none);
        hipLaunchKernelGGL((k_gat_segments<1, 1, false>), gs, b, 0, s, g, q, att, none, none, (const float*)factor, none);
    }
}

void launch_gat_bwd_scalars(const GatRowsHost& h, const float* att, const float* dal, float* pair,
                            float* gs_dst_own, float* segwork, hipStream_t s)
{
    const GatRows g = make_rows(h);
    float* a = const_cast<float*>(att);
    float* d = const_cast<float*>(dal);
    if (g.nranges > 0) {
        const dim3 grid((unsigned)((g.nranges + 3) / 4)), b(kBlock);
        if (g.nh == 1) hipLaunchKernelGGL((k_gat_rows<1, 1, false>), grid, b, 0, s, g, a, d, pair, gs_dst_own);
        else if (g.nh % 4 == 0) hipLaunchKernelGGL((k_gat_rows<1, 4, true>), grid, b, 0, s, g, a, d, pair, gs_dst_own);
        else if (g.nh % 2 == 0) hipLaunchKernelGGL((k_gat_rows<1, 2, true>), grid, b, 0, s, g, a, d, pair, gs_dst_own);
        else hipLaunchKernelGGL((k_gat_rows<1, 2, false>), grid, b, 0, s, g, a, d, pair, gs_dst_own);
    }
    const GatSegs q = make_segs(h);
    if (q.nsegs > 0 && q.nlong > 0) {
        float* stat = segwork;
        float* factor = segwork + 2 * q.nsegs * g.nh;
        float* none = nullptr;
        const dim3 gs((unsigned)((q.nsegs + 3) / 4)), gl((unsigned)((q.nlong + 3) / 4)), b(kBlock);
        hipLaunchKernelGGL((k_gat_segments<2, 1, false>), gs, b, 0, s, g, q, a, d, stat, (const float*)nullptr, none);
        hipLaunchKernelGGL((k_gat_combine<2>), gl, b, 0, s, q, g.nh, (const float*)stat, factor, none);
        if (g.nh == 1)
            hipLaunchKernelGGL((k_gat_segments<3, 1, false>), gs, b, 0, s, g, q, a, d, stat, (const float*)factor, pair);
        else if (g.nh % 4 == 0)
            hipLaunchKernelGGL((k_gat_segments<3, 4, true>), gs, b, 0, s, g, q, a, d, stat, (const float*)factor, pair);
        else if (g.nh % 2 == 0)
            hipLaunchKernelGGL((k_gat_segments<3, 2, true>), gs, b, 0, s, g, q, a, d, stat, (const float*)factor, pair);
        else
            hipLaunchKernelGGL((k_gat_segments<3, 2, false>), gs, b, 0, s, g, q, a, d, stat, (const float*)factor, pair);
        hipLaunchKernelGGL((k_gat_combine<3>), gl, b, 0, s, q, g.nh, (const float*)stat, none, gs_dst_own);
    }
}

void launch_gat_transposed(const int64_t* trp, const int32_t* tperm, int64_t e0, int64_t n_own,
                           int64_t base_row, const int32_t* bnd, const SpmmItems& items, const float* pair,
                           float* tw_att, float* gs_src, int32_t nh, int64_t hs, float* segwork, hipStream_t s)
{
    GatTRows g;
    g.trp = trp; g.tperm = tperm; g.e0 = e0; g.n_own = n_own; g.base_row = base_row; g.bnd = bnd;
    g.nh = nh; g.hs = hs;
    g.range_rows = items.range_rows; g.nranges = items.nranges;
    if (g.nranges > 0) {
        const dim3 grid((unsigned)((g.nranges + 3) / 4)), b(kBlock);
        if (nh % 2 == 0) hipLaunchKernelGGL((k_gat_trows<true>), grid, b, 0, s, g, pair, tw_att, gs_src);
        else hipLaunchKernelGGL((k_gat_trows<false>), grid, b, 0, s, g, pair, tw_att, gs_src);
    }
    if (items.nlong > 0 && items.nsegs > 0) {
        GatSegs q;
        q.seg_row = items.seg_row; q.seg_begin = items.seg_begin; q.seg_len = items.seg_len; q.nsegs = items.nsegs;
        q.long_row = items.long_row; q.long_first = items.long_first; q.long_nseg = items.long_nseg;
        q.nlong = items.nlong;
        hipLaunchKernelGGL(k_gat_tsegs, dim3((unsigned)((q.nsegs + 3) / 4)), dim3(kBlock), 0, s, g, q, pair, tw_att,
                           segwork);
        hipLaunchKernelGGL(k_gat_tcombine, dim3((unsigned)((q.nlong + 3) / 4)), dim3(kBlock), 0, s, g, q,
                           (const float*)segwork, gs_src);
    }
}

void launch_gat_dots(const int64_t* rp, const int32_t* col, int64_t e0, int64_t n_own, const float* a_rows,
                     const float* b_rows, const float* dy, int32_t d, int32_t ld, float* dal, const SpmmItems& items,
                     hipStream_t s, int32_t nslice, int64_t dal_stride)
{
    const int64_t nitems = items.nsegs + items.nranges;
    if (nitems <= 0) return;
    if (nslice < 1) nslice = 1;
    GatDotArgs g;
    g.rp = rp; g.col = col; g.e0 = e0; g.n_own = n_own; g.a_rows = a_rows; g.b_rows = b_rows; g.dy = dy;
    g.ld = ld; g.d = d; g.dal = dal; g.it = items;
    g.nslice = nslice; g.dal_stride = dal_stride;
    const dim3 grid((unsigned)((nitems + 3) / 4 * nslice)), block(kBlock);
    const int vecs = d / 4;
    if (vecs <= 4) hipLaunchKernelGGL((k_gat_dots<4, 1>), grid, block, 0, s, g);
    else if (vecs <= 8) hipLaunchKernelGGL((k_gat_dots<8, 1>), grid, block, 0, s, g);
    else if (vecs <= 16) hipLaunchKernelGGL((k_gat_dots<16, 1>), grid, block, 0, s, g);
    else if (vecs <= 32) hipLaunchKernelGGL((k_gat_dots<32, 1>), grid, block, 0, s, g);
    // 1 KB rows: four 16-lane slots with four vectors per lane keep 16 source rows in flight per
    // wavefront and need four shuffle steps per entry (one 64-lane slot: 4 rows, six steps)
    else if (vecs <= 64) hipLaunchKernelGGL((k_gat_dots<16, 4>), grid, block, 0, s, g);
    else if (vecs <= 128) hipLaunchKernelGGL((k_gat_dots<64, 2>), grid, block, 0, s, g);
    else hipLaunchKernelGGL((k_gat_dots<64, 4>), grid, block, 0, s, g);
}

int64_t gat_rank1_partial_floats(int64_t rows, int32_t f) { return ((rows + 255) / 256) * 2 * (int64_t)f; }

void launch_gat_rank1(float* gH, const float* H, int32_t ld, int32_t f, int64_t rows, const float* gs_src,
                      const float* gs_dst, int32_t nh, int32_t fh, const float* a_src, const float* a_dst,
                      float* partial, hipStream_t s)
{
    if (rows <= 0) return;
    const dim3 grid((unsigned)((rows + 255) / 256)), b(kBlock);
    if (f <= 32)
        hipLaunchKernelGGL((k_gat_rank1_narrow<32>), grid, b, 0, s, gH, H, ld, f, rows, gs_src, gs_dst, a_src, a_dst,
                           partial, nh, fh);
    else if (f <= 64)
        hipLaunchKernelGGL((k_gat_rank1_narrow<64>), grid, b, 0, s, gH, H, ld, f, rows, gs_src, gs_dst, a_src, a_dst,
                           partial, nh, fh);
    else if (f <= 128)
        hipLaunchKernelGGL((k_gat_rank1_narrow<128>), grid, b, 0, s, gH, H, ld, f, rows, gs_src, gs_dst, a_src, a_dst,
                           partial, nh, fh);
    else
        hipLaunchKernelGGL(k_gat_rank1, grid, b, 0, s, gH, H, ld, f, rows, gs_src, gs_dst, a_src, a_dst, partial, nh, fh);
}

}  // namespace gnnmi
