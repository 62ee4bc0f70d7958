// Dense contractions with bfloat16 operands and fp32 accumulation on the matrix cores
// (v_mfma_f32_32x32x16_bf16), gfx950.  Same three products as the fp32 file:
//
//   forward   A_p^l  = act( Z_p W^l (+ X_p W_s^l) + b^l )     bf16 x bf16 -> bf16 (fp32 logits)
//   backward  dZ_p   = dY_p (W^l)^T                           bf16 x bf16 -> bf16 / += fp32
//             grad W^l += Z_p^T dY_p                          bf16 x bf16 -> fp32, split-K
//
// A workgroup of 4 wavefronts (2 x 2) owns a BM x BN tile of C and walks K in steps of 32.
// Both operands sit in LDS as [row][k] with k contiguous, because an MFMA lane consumes eight
// consecutive k of its row as one 16-byte register group.  Operands that are k-contiguous in
// memory are copied with 16-byte loads and stores; operands that are row-contiguous in memory
// (W in the forward product, both operands of Z^T dY) are transposed on the way into LDS.
#include "gnn_internal.h"

namespace gnnmi {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint16_t bf16_t;

constexpr int kThreads = 256;
constexpr int BK = 32;
constexpr int LDK = BK + 8;   // LDS row stride in elements (80 bytes: conflict-free 16-byte reads)

__device__ inline float bf16_to_float(uint32_t h) { return __uint_as_float(h << 16); }
__device__ inline uint32_t float_to_bf16(float f)
{
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// (slow = m or n, fast = k): thread t covers slow = t / 4 + 64 i, k = 8 (t % 4) .. + 7.
template <int BT, bool VEC>
__device__ inline void load_kfast(const bf16_t* __restrict__ p, int64_t ld, int64_t slow0,
                                  int64_t nslow, int64_t k0, int64_t kend, uint4 (&r)[BT / 64])
{
    const int t = threadIdx.x;
    const int kq = (t & 3) * 8;
#pragma unroll
    for (int i = 0; i < BT / 64; ++i) {
        const int64_t sidx = slow0 + (t >> 2) + 64 * i;
        const int64_t k = k0 + kq;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (sidx < nslow) {
            const bf16_t* q = p + sidx * ld + k;
            if (VEC) {
                if (k < kend) v = *reinterpret_cast<const uint4*>(q);
            } else {
                uint32_t e[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) e[j] = (k + j < kend) ? q[j] : 0u;
                v = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16),
                               e[6] | (e[7] << 16));
            }
        }
        r[i] = v;
    }
}
template <int BT>
__device__ inline void store_kfast(bf16_t* S, const uint4 (&r)[BT / 64])
{
    const int t = threadIdx.x;
    const int kq = (t & 3) * 8;
#pragma unroll
    for (int i = 0; i < BT / 64; ++i)
        *reinterpret_cast<uint4*>(S + ((t >> 2) + 64 * i) * LDK + kq) = r[i];
}

// (slow = k, fast = m or n): thread t covers k = t / (BT/8) + (2048/BT) i, fast = 8 (t % (BT/8)) .. + 7.
template <int BT, bool VEC>
__device__ inline void load_kslow(const bf16_t* __restrict__ p, int64_t ld, int64_t k0, int64_t kend,
                                  int64_t fast0, int64_t nfast, uint4 (&r)[BT / 64])
{
    constexpr int TPR = BT / 8;
    constexpr int KPP = kThreads / TPR;
    const int t = threadIdx.x;
    const int fq = (t % TPR) * 8;
#pragma unroll
    for (int i = 0; i < BT / 64; ++i) {
        const int64_t k = k0 + t / TPR + KPP * i;
        const int64_t f = fast0 + fq;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (k < kend) {
            const bf16_t* q = p + k * ld + f;
            if (VEC) {
                if (f < nfast) v = *reinterpret_cast<const uint4*>(q);
            } else {
                uint32_t e[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) e[j] = (f + j < nfast) ? q[j] : 0u;
                v = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16),
                               e[6] | (e[7] << 16));
            }
        }
        r[i] = v;
    }
}
// transposing store: element j of the vector belongs to LDS row fq + j, column k
template <int BT>
__device__ inline void store_kslow(bf16_t* S, const uint4 (&r)[BT / 64])
{
    constexpr int TPR = BT / 8;
    constexpr int KPP = kThreads / TPR;
    const int t = threadIdx.x;
    const int fq = (t % TPR) * 8;
#pragma unroll
    for (int i = 0; i < BT / 64; ++i) {
        const int k = t / TPR + KPP * i;
        const uint32_t w[4] = {r[i].x, r[i].y, r[i].z, r[i].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            S[(fq + 2 * j) * LDK + k] = (bf16_t)(w[j] & 0xFFFFu);
            S[(fq + 2 * j + 1) * LDK + k] = (bf16_t)(w[j] >> 16);
        }
    }
}

struct Args {
    const bf16_t* a[2];
    const bf16_t* b[2];
    int64_t lda[2], ldb[2];
    int32_t kseg[2];
    void* c;                 // fp32 or bf16
    int64_t ldc;
    int64_t m;
    int32_t n;
    const float* bias;
    int32_t relu, accumulate, out_bf16;
    int64_t split_chunk, split_stride;
};

template <int BM, int BN, bool A_KFAST, bool B_KFAST, bool VEC_A, bool VEC_B>
__global__ __launch_bounds__(kThreads) void k_gemm_bf16(const Args g)
{
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int TM = WM / 32, TN = WN / 32;
    __shared__ __attribute__((aligned(16))) bf16_t As[2][BM * LDK];
    __shared__ __attribute__((aligned(16))) bf16_t Bs[2][BN * LDK];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wm0 = (wave >> 1) * WM, wn0 = (wave & 1) * WN;
    const int64_t m0 = (int64_t)blockIdx.x * BM;
    const int32_t n0 = blockIdx.y * BN;

    int64_t kbeg = 0, kend0 = g.kseg[0];
    int64_t coff = 0;
    if (g.split_chunk > 0) {
        kbeg = (int64_t)blockIdx.z * g.split_chunk;
        kend0 = kbeg + g.split_chunk < kend0 ? kbeg + g.split_chunk : kend0;
        coff = (int64_t)blockIdx.z * g.split_stride;
    }
    const int64_t tiles0 = kend0 > kbeg ? (kend0 - kbeg + BK - 1) / BK : 0;
    const int64_t tiles1 = (g.kseg[1] + BK - 1) / BK;
    const int64_t ntiles = tiles0 + tiles1;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    uint4 ra[BM / 64], rb[BN / 64];
    auto load_tile = [&](int64_t t) {
        const int seg = t < tiles0 ? 0 : 1;
        const int64_t k0 = seg == 0 ? kbeg + t * BK : (t - tiles0) * BK;
        const int64_t kend = seg == 0 ? kend0 : (int64_t)g.kseg[1];
        if (A_KFAST) load_kfast<BM, VEC_A>(g.a[seg], g.lda[seg], m0, g.m, k0, kend, ra);
        else load_kslow<BM, VEC_A>(g.a[seg], g.lda[seg], k0, kend, m0, g.m, ra);
        if (B_KFAST) load_kfast<BN, VEC_B>(g.b[seg], g.ldb[seg], n0, g.n, k0, kend, rb);
        else load_kslow<BN, VEC_B>(g.b[seg], g.ldb[seg], k0, kend, n0, g.n, rb);
    };
    auto store_tile = [&](int buf) {
        if (A_KFAST) store_kfast<BM>(As[buf], ra); else store_kslow<BM>(As[buf], ra);
        if (B_KFAST) store_kfast<BN>(Bs[buf], rb); else store_kslow<BN>(Bs[buf], rb);
    };

    if (ntiles > 0) {
        load_tile(0);
        store_tile(0);
    }
    __syncthreads();
    for (int64_t t = 0; t < ntiles; ++t) {
        const int buf = (int)(t & 1);
        if (t + 1 < ntiles) load_tile(t + 1);
        const int half = lane >> 5, xl = lane & 31;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 av[TM], bv[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                av[i] = *reinterpret_cast<const bf16x8*>(&As[buf][(wm0 + 32 * i + xl) * LDK + 16 * ks + 8 * half]);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bv[j] = *reinterpret_cast<const bf16x8*>(&Bs[buf][(wn0 + 32 * j + xl) * LDK + 16 * ks + 8 * half]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[j], acc[i][j], 0, 0, 0);
        }
        if (t + 1 < ntiles) store_tile(buf ^ 1);
        __syncthreads();
    }

    // lane holds C[8 (r/4) + 4 (lane/32) + r%4][lane%32] of each 32x32 tile
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int32_t col = n0 + wn0 + 32 * j + (lane & 31);
            if (col >= g.n) continue;
            const float bvl = g.bias ? g.bias[col] : 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = m0 + wm0 + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (row >= g.m) continue;
                float v = acc[i][j][r] + bvl;
                if (g.relu) v = v > 0.f ? v : 0.f;
                const int64_t at = coff + row * g.ldc + col;
                if (g.out_bf16) {
                    static_cast<bf16_t*>(g.c)[at] = (bf16_t)float_to_bf16(v);
                } else {
                    float* dst = static_cast<float*>(g.c) + at;
                    if (g.accumulate) v += *dst;
                    *dst = v;
                }
            }
        }
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

template <bool A_KFAST, bool B_KFAST>
void launch(const Args& g, int splits, hipStream_t s)
{
    if (g.m <= 0 || g.n <= 0) return;
    bool va = true, vb = true;
    for (int i = 0; i < 2; ++i) {
        if (g.kseg[i] == 0) continue;
        va = va && aligned16(g.a[i]) && g.lda[i] % 8 == 0 && (!A_KFAST || g.kseg[i] % 8 == 0);
        vb = vb && aligned16(g.b[i]) && g.ldb[i] % 8 == 0 && (!B_KFAST || g.kseg[i] % 8 == 0);
    }
    if (!A_KFAST) va = va && g.m % 8 == 0;
    if (!B_KFAST) vb = vb && g.n % 8 == 0;
    const bool big_m = g.m > 64, big_n = g.n > 64;
#define GNN_GEMM(BM, BN, VA, VB)                                                                \
    hipLaunchKernelGGL((k_gemm_bf16<BM, BN, A_KFAST, B_KFAST, VA, VB>),                         \
                       dim3((unsigned)((g.m + BM - 1) / BM), (unsigned)((g.n + BN - 1) / BN),   \
                            (unsigned)splits),                                                  \
                       dim3(kThreads), 0, s, g)
#define GNN_GEMM_TILE(VA, VB)                                     \
    do {                                                          \
        if (big_m && big_n) GNN_GEMM(128, 128, VA, VB);           \
        else if (big_m) GNN_GEMM(128, 64, VA, VB);                \
        else if (big_n) GNN_GEMM(64, 128, VA, VB);                \
        else GNN_GEMM(64, 64, VA, VB);                            \
    } while (0)
    if (va && vb) GNN_GEMM_TILE(true, true);
    else if (va) GNN_GEMM_TILE(true, false);
    else if (vb) GNN_GEMM_TILE(false, true);
    else GNN_GEMM_TILE(false, false);
#undef GNN_GEMM_TILE
#undef GNN_GEMM
}

// dst[i] = bf16(src[i])
__global__ __launch_bounds__(256) void k_to_bf16(const float* __restrict__ src, bf16_t* __restrict__ dst,
                                                 int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
        dst[i] = (bf16_t)float_to_bf16(src[i]);
}

}  // namespace

void launch_gemm_bf16_nn(const GemmSegBf16* segs, int nseg, void* c, int out_bf16, int64_t ldc,
                         int64_t m, int32_t n, const GemmEpilogue& ep, hipStream_t s)
{
    Args g{};
    for (int i = 0; i < 2; ++i) {
        const GemmSegBf16& sg = segs[i < nseg ? i : 0];
        g.a[i] = (const bf16_t*)sg.a; g.lda[i] = sg.lda;
        g.b[i] = (const bf16_t*)sg.b; g.ldb[i] = sg.ldb;
        g.kseg[i] = i < nseg ? sg.k : 0;
    }
    g.c = c; g.ldc = ldc; g.m = m; g.n = n; g.out_bf16 = out_bf16;
    g.bias = ep.bias; g.relu = ep.relu; g.accumulate = ep.accumulate;
    launch<true, false>(g, 1, s);
}

void launch_gemm_bf16_nt(const void* a, int64_t lda, const void* b, int64_t ldb, void* c,
                         int out_bf16, int64_t ldc, int64_t m, int32_t n, int32_t k,
                         const GemmEpilogue& ep, hipStream_t s)
{
    Args g{};
    g.a[0] = g.a[1] = (const bf16_t*)a; g.lda[0] = g.lda[1] = lda;
    g.b[0] = g.b[1] = (const bf16_t*)b; g.ldb[0] = g.ldb[1] = ldb;
    g.kseg[0] = k; g.kseg[1] = 0;
    g.c = c; g.ldc = ldc; g.m = m; g.n = n; g.out_bf16 = out_bf16;
    g.bias = ep.bias; g.relu = ep.relu; g.accumulate = ep.accumulate;
    launch<true, true>(g, 1, s);
}

void launch_gemm_bf16_tn(const void* a, int64_t lda, const void* b, int64_t ldb, float* c,
                         int64_t ldc, int32_t m, int32_t n, int64_t kdim, float* partial,
                         hipStream_t s)
{
    if (kdim <= 0 || m <= 0 || n <= 0) return;
    const int splits = gemm_tn_splits(kdim, m, n);
    int64_t chunk = (kdim + splits - 1) / splits;
    chunk = (chunk + BK - 1) / BK * BK;
    Args g{};
    g.a[0] = g.a[1] = (const bf16_t*)a; g.lda[0] = g.lda[1] = lda;
    g.b[0] = g.b[1] = (const bf16_t*)b; g.ldb[0] = g.ldb[1] = ldb;
    g.kseg[0] = (int32_t)kdim; g.kseg[1] = 0;
    g.c = partial; g.ldc = n; g.m = m; g.n = n; g.out_bf16 = 0;
    g.split_chunk = chunk;
    g.split_stride = (int64_t)m * n;
    launch<false, false>(g, splits, s);
    launch_reduce_partials(partial, splits, (int64_t)m * n, c, ldc, m, n, s);
}

void launch_to_bf16(const float* src, void* dst, int64_t n, hipStream_t s)
{
    if (n <= 0) return;
    int64_t blocks = (n + 255) / 256;
    blocks = blocks > 16384 ? 16384 : blocks;
    hipLaunchKernelGGL(k_to_bf16, dim3((unsigned)blocks), dim3(256), 0, s, src, (bf16_t*)dst, n);
}

}  // namespace gnnmi
