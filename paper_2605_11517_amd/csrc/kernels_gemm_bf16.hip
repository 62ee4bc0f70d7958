// Dense contractions with bfloat16 operands and fp32 accumulation on the matrix cores
// (v_mfma_f32_32x32x16_bf16), gfx950.  Same three products as the fp32 file:
//
//   forward   A_p^l  = act( Z_p W^l (+ X_p W_s^l) + b^l )     bf16 x bf16 -> bf16 (fp32 logits)
//   backward  dZ_p   = dY_p (W^l)^T                           bf16 x bf16 -> bf16 / += fp32
//             grad W^l += Z_p^T dY_p                          bf16 x bf16 -> fp32, split-K
//
// Two families.  The large products (at least 512 rows and 256 columns, K a multiple of 64, one
// K segment) run on the 256 x 256 tile kernels further down (k_gemm_bf16_wide for k-contiguous
// operands, k_gemm_bf16_tn_wide for the reduction over rows), which fill LDS with direct-to-LDS
// loads.  Everything else (narrow output layers, ragged K, two-segment GraphSAGE products) runs
// on the kernel described next.
//
// A workgroup of 4 wavefronts (2 x 2) owns a BM x BN tile of C and walks K in steps of 32.
// An MFMA lane consumes eight consecutive k of its row as one 16-byte register group.
// Operands that are k-contiguous in memory are kept [row][k] in LDS and fetched with one
// 16-byte read per fragment.  Operands that are row-contiguous in memory (W in the forward
// product, both operands of Z^T dY) are kept as they come, [k][row], and a fragment is
// gathered with eight 2-byte reads down a column; consecutive lanes then read consecutive
// rows, which is conflict-free, whereas transposing on the way into LDS would put the sixteen
// lanes of a k-row on one bank.
#include "gnn_internal.h"
#include <cstdlib>

namespace gnnmi {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint16_t bf16_t;

constexpr int kThreads = 256;
constexpr int BK = 32;
constexpr int PF = 1;         // tiles of global loads in flight per thread (2 and 3: occupancy falls
                              // from 3 to 2 waves per SIMD, 20-30 % slower)
constexpr int LDK = BK + 8;   // k-fast tiles: [row][k], row stride 80 bytes (conflict-free 16-byte reads)
constexpr int XPAD = 4;       // k-slow tiles: [k][row], row stride BT + 4 elements

__device__ inline float bf16_to_float(uint32_t h) { return __uint_as_float(h << 16); }
__device__ inline uint32_t float_to_bf16(float f)
{
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// two floats rounded to nearest even and packed (lo | hi << 16): one conversion instruction
__device__ inline uint32_t pack_bf16(float lo, float hi)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float floatx2 __attribute__((ext_vector_type(2)));
    const floatx2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
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
        if (VEC) {
            // unconditional load from a clamped (always valid) address, zeroed afterwards:
            // without branches the compiler can keep several tiles of loads in flight
            const bf16_t* q = p + (sidx < nslow ? sidx : nslow - 1) * ld + (k < kend ? k : k0);
            const uint4 x = *reinterpret_cast<const uint4*>(q);
            v = x;   // rows / k past the end are zeroed when the tile goes to LDS
        } else if (sidx < nslow) {
            const bf16_t* q = p + sidx * ld + k;
            {
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
        if (VEC) {
            const bf16_t* q = p + (k < kend ? k : k0) * ld + (f < nfast ? f : fast0);
            const uint4 x = *reinterpret_cast<const uint4*>(q);
            v = x;   // rows / k past the end are zeroed when the tile goes to LDS
        } else if (k < kend) {
            const bf16_t* q = p + k * ld + f;
            {
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
// k-slow tiles stay [k][x] in LDS: two 8-byte stores per vector (rows are 8-byte aligned)
template <int BT>
__device__ inline void store_kslow(bf16_t* S, const uint4 (&r)[BT / 64])
{
    constexpr int TPR = BT / 8;
    constexpr int KPP = kThreads / TPR;
    const int t = threadIdx.x;
    const int fq = (t % TPR) * 8;
#pragma unroll
    for (int i = 0; i < BT / 64; ++i) {
        bf16_t* dst = S + (t / TPR + KPP * i) * (BT + XPAD) + fq;
        *reinterpret_cast<uint2*>(dst) = make_uint2(r[i].x, r[i].y);
        *reinterpret_cast<uint2*>(dst + 4) = make_uint2(r[i].z, r[i].w);
    }
}

// The eight consecutive k (k8 .. k8 + 7) of row x as one MFMA operand register group.
template <int BT, bool KFAST>
__device__ inline bf16x8 load_fragment(const bf16_t* S, int x, int k8)
{
    if (KFAST) {
        return *reinterpret_cast<const bf16x8*>(S + x * LDK + k8);
    } else {
        union { bf16_t h[8]; bf16x8 v; } u;
#pragma unroll
        for (int j = 0; j < 8; ++j) u.h[j] = S[(k8 + j) * (BT + XPAD) + x];
        return u.v;
    }
}

// Zero the vectors of a tile that lie past the end of the matrix (their loads were clamped to
// valid addresses).  Done when the registers are written to LDS, not at load time, so that the
// loads of several tiles stay in flight.
template <int BT>
__device__ inline void mask_kfast(int64_t slow0, int64_t nslow, int64_t k0, int64_t kend, uint4 (&r)[BT / 64])
{
    const int t = threadIdx.x;
    const int64_t k = k0 + (t & 3) * 8;
#pragma unroll
    for (int i = 0; i < BT / 64; ++i)
        if (!(slow0 + (t >> 2) + 64 * i < nslow && k < kend)) r[i] = make_uint4(0, 0, 0, 0);
}
template <int BT>
__device__ inline void mask_kslow(int64_t k0, int64_t kend, int64_t fast0, int64_t nfast, uint4 (&r)[BT / 64])
{
    constexpr int TPR = BT / 8;
    constexpr int KPP = kThreads / TPR;
    const int t = threadIdx.x;
    const int64_t f = fast0 + (t % TPR) * 8;
#pragma unroll
    for (int i = 0; i < BT / 64; ++i)
        if (!(k0 + t / TPR + KPP * i < kend && f < nfast)) r[i] = make_uint4(0, 0, 0, 0);
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
    int32_t nt_1d;           // > 0: one-dimensional grid over (M tile, N tile), see tile_of_block
};

// Which tile a workgroup of a one-dimensional grid owns.  Workgroups are dealt to the 8 XCDs
// round-robin, each XCD with its own L2: block b runs on XCD b % 8 as that XCD's (b / 8)-th
// workgroup.  The workgroups of one XCD walk all N tiles of an M tile before the next M tile,
// so the rows of A they share are fetched into that L2 once instead of once per N tile.
__device__ inline bool tile_of_block(int64_t b, int64_t mt, int32_t nt, int64_t& mtile, int32_t& ntile)
{
    const int64_t slot = b >> 3;
    ntile = (int32_t)(slot % nt);
    mtile = (slot / nt) * 8 + (b & 7);
    return mtile < mt;
}

template <int BM, int BN, bool A_KFAST, bool B_KFAST, bool VEC_A, bool VEC_B>
__global__ __launch_bounds__(kThreads) void k_gemm_bf16(const Args g)
{
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int A_TILE = A_KFAST ? BM * LDK : BK * (BM + XPAD);
    constexpr int B_TILE = B_KFAST ? BN * LDK : BK * (BN + XPAD);
    __shared__ __attribute__((aligned(16))) bf16_t As[2][A_TILE];
    __shared__ __attribute__((aligned(16))) bf16_t Bs[2][B_TILE];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wm0 = (wave >> 1) * WM, wn0 = (wave & 1) * WN;
    int64_t mtile = blockIdx.x;
    int32_t ntile = blockIdx.y;
    if (g.nt_1d > 0 && !tile_of_block(blockIdx.x, (g.m + BM - 1) / BM, g.nt_1d, mtile, ntile)) return;
    const int64_t m0 = mtile * BM;
    const int32_t n0 = ntile * BN;

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

    // Register ring of PF tiles: the global loads of tile t + PF are issued while tile t is
    // multiplied, so that a load has PF tile-times to arrive (one tile-time is far shorter than
    // the memory latency, above all with the fast bf16 MFMA).
    uint4 ra[PF][BM / 64], rb[PF][BN / 64];
    auto load_tile = [&](int64_t t, uint4 (&ra)[BM / 64], uint4 (&rb)[BN / 64]) {
        const int seg = t < tiles0 ? 0 : 1;
        const int64_t k0 = seg == 0 ? kbeg + t * BK : (t - tiles0) * BK;
        const int64_t kend = seg == 0 ? kend0 : (int64_t)g.kseg[1];
        if (A_KFAST) load_kfast<BM, VEC_A>(g.a[seg], g.lda[seg], m0, g.m, k0, kend, ra);
        else load_kslow<BM, VEC_A>(g.a[seg], g.lda[seg], k0, kend, m0, g.m, ra);
        if (B_KFAST) load_kfast<BN, VEC_B>(g.b[seg], g.ldb[seg], n0, g.n, k0, kend, rb);
        else load_kslow<BN, VEC_B>(g.b[seg], g.ldb[seg], k0, kend, n0, g.n, rb);
    };
    auto store_tile = [&](int buf, int64_t t, const uint4 (&ra_in)[BM / 64], const uint4 (&rb_in)[BN / 64]) {
        const int seg = t < tiles0 ? 0 : 1;
        const int64_t k0 = seg == 0 ? kbeg + t * BK : (t - tiles0) * BK;
        const int64_t kend = seg == 0 ? kend0 : (int64_t)g.kseg[1];
        uint4 ra[BM / 64], rb[BN / 64];
#pragma unroll
        for (int i = 0; i < BM / 64; ++i) ra[i] = ra_in[i];
#pragma unroll
        for (int i = 0; i < BN / 64; ++i) rb[i] = rb_in[i];
        if (A_KFAST) { mask_kfast<BM>(m0, g.m, k0, kend, ra); store_kfast<BM>(As[buf], ra); }
        else { mask_kslow<BM>(k0, kend, m0, g.m, ra); store_kslow<BM>(As[buf], ra); }
        if (B_KFAST) { mask_kfast<BN>(n0, g.n, k0, kend, rb); store_kfast<BN>(Bs[buf], rb); }
        else { mask_kslow<BN>(k0, kend, n0, g.n, rb); store_kslow<BN>(Bs[buf], rb); }
    };

#pragma unroll
    for (int d = 0; d < PF; ++d)
        if (ntiles > 0) load_tile(d < ntiles ? d : ntiles - 1, ra[d], rb[d]);
    if (ntiles > 0) store_tile(0, 0, ra[0], rb[0]);
    __syncthreads();
    for (int64_t t0 = 0; t0 < ntiles; t0 += PF) {
#pragma unroll
        for (int dd = 0; dd < PF; ++dd) {
            const int64_t t = t0 + dd;
            if (t >= ntiles) break;
            const int buf = (int)(t & 1);
            // slot dd held tile t, already in LDS; past the end the last tile is fetched again
            // (never used) so that the load stream has no branches
            load_tile(t + PF < ntiles ? t + PF : ntiles - 1, ra[dd], rb[dd]);
            // keep the loads ahead of the MFMA block (the scheduler would sink them to the wait
            // in front of the LDS store)
            __builtin_amdgcn_sched_barrier(0);
        const int half = lane >> 5, xl = lane & 31;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 av[TM], bv[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                av[i] = load_fragment<BM, A_KFAST>(As[buf], wm0 + 32 * i + xl, 16 * ks + 8 * half);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bv[j] = load_fragment<BN, B_KFAST>(Bs[buf], wn0 + 32 * j + xl, 16 * ks + 8 * half);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[j], acc[i][j], 0, 0, 0);
        }
            if (t + 1 < ntiles) store_tile(buf ^ 1, t + 1, ra[(dd + 1) % PF], rb[(dd + 1) % PF]);
            __syncthreads();
        }
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
    static const bool xcd_map = [] {
        const char* e = getenv("GNNMI_GEMM_XCD_MAP");
        return !(e && e[0] == '0');
    }();
#define GNN_GEMM(BM, BN, VA, VB)                                                                \
    do {                                                                                        \
        const int64_t mt = (g.m + BM - 1) / BM;                                                 \
        const int32_t nt = (g.n + BN - 1) / BN;                                                 \
        Args ga = g;                                                                            \
        if (splits == 1 && nt > 1 && xcd_map) {                                                 \
            ga.nt_1d = nt;                                                                      \
            hipLaunchKernelGGL((k_gemm_bf16<BM, BN, A_KFAST, B_KFAST, VA, VB>),                 \
                               dim3((unsigned)((mt + 7) / 8 * 8 * nt)), dim3(kThreads), 0, s, ga); \
        } else {                                                                                \
            hipLaunchKernelGGL((k_gemm_bf16<BM, BN, A_KFAST, B_KFAST, VA, VB>),                 \
                               dim3((unsigned)mt, (unsigned)nt, (unsigned)splits), dim3(kThreads), 0, s, ga); \
        }                                                                                       \
    } while (0)
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

// ---------------------------------------------------------------------------------------------
// Wide variant for the large products with both operands k-contiguous (A [M x K], B [N x K]):
// a 256 x 256 tile per workgroup of 8 wavefronts (2 x 4, 128 x 64 each), K in steps of 64.
// The two LDS stages are filled by direct-to-LDS loads (global_load_lds_dwordx4: 16 bytes per
// lane, a wavefront fills 1 KB of LDS per instruction, no registers and no ds_write involved),
// issued for stage t + 1 right after the barrier that opens stage t.  Inside a tile row (128
// bytes = eight 16-byte chunks) the chunks are permuted by the row number so that the sixteen
// lanes of a fragment read touch every bank once; the permutation is applied on the global
// side, by choosing which chunk a lane fetches.  bf16 results leave through LDS so that a lane
// stores 16 contiguous bytes.
constexpr int WBM = 256, WBN = 256, WBK = 64, WTHREADS = 512;
constexpr int WROWB = WBK * 2;                         // bytes per tile row
constexpr int WSTAGE = (WBM + WBN) * WROWB;            // bytes per stage
constexpr int WTM = 128, WTN = 64;                     // wave tile
constexpr int WCS = WTN * 2 + 16;                      // row stride of a wave's output patch, bytes
constexpr int WLDS = 2 * WSTAGE > 8 * WTM * WCS ? 2 * WSTAGE : 8 * WTM * WCS;

__device__ inline int wide_chunk(int x, int c) { return x * WROWB + ((c ^ ((x >> 1) & 7)) << 4); }

__device__ inline void wide_issue(const bf16_t* __restrict__ p, int64_t ld, int64_t row0, int64_t nrows,
                                  int64_t k0, char* lds_tile, int wave, int lane)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int q = j * 8 + wave;                    // block of 8 rows = 1 KB of LDS
        const int row = q * 8 + (lane >> 3);
        const int c = (lane & 7) ^ ((row >> 1) & 7);   // LDS slot lane & 7 of the row holds chunk c
        int64_t gr = row0 + row;
        gr = gr < nrows ? gr : nrows - 1;              // rows past the end: valid address, result unused
        const bf16_t* src = p + gr * ld + k0 + c * 8;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                         (__attribute__((address_space(3))) void*)(lds_tile + q * 1024), 16, 0, 0);
    }
}

// Stores the 256 x 256 tile held in the accumulators of the eight wavefronts: + bias, max(., 0),
// then bf16 rows through LDS (16 contiguous bytes per lane) or fp32 values straight from the
// MFMA layout.
__device__ inline void wide_store(const Args& g, floatx16 (&acc)[4][2], char* wlds, int64_t m0, int32_t n0,
                                  int wave, int lane, int wm, int wn)
{
    if (g.out_bf16) {
        __syncthreads();                               // every wave is done reading the last stage
        char* patch = wlds + (size_t)wave * WTM * WCS; // private to the wave: [128 rows][64 cols]
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int lc = 32 * j + (lane & 31);
                const int32_t col = n0 + wn * WTN + lc;
                const float bvl = (g.bias && col < g.n) ? g.bias[col] : 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int lr = 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    float v = acc[i][j][r] + bvl;
                    if (g.relu) v = v > 0.f ? v : 0.f;
                    *reinterpret_cast<bf16_t*>(patch + lr * WCS + lc * 2) = (bf16_t)float_to_bf16(v);
                }
            }
        // no barrier: the LDS accesses of one wave complete in order
        const int cq = lane & 7, rr = lane >> 3;       // 8 lanes per row, 8 rows per pass
        const int32_t col0 = n0 + wn * WTN + cq * 8;
#pragma unroll
        for (int ps = 0; ps < WTM / 8; ++ps) {
            const int lr = ps * 8 + rr;
            const int64_t row = m0 + wm * WTM + lr;
            const uint4 v = *reinterpret_cast<const uint4*>(patch + lr * WCS + cq * 16);
            if (row < g.m && col0 + 7 < g.n) {
                *reinterpret_cast<uint4*>(static_cast<bf16_t*>(g.c) + row * g.ldc + col0) = v;
            } else if (row < g.m) {
                const bf16_t* e = reinterpret_cast<const bf16_t*>(&v);
                for (int u = 0; u < 8; ++u)
                    if (col0 + u < g.n) static_cast<bf16_t*>(g.c)[row * g.ldc + col0 + u] = e[u];
            }
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int32_t col = n0 + wn * WTN + 32 * j + (lane & 31);
            if (col >= g.n) continue;
            const float bvl = g.bias ? g.bias[col] : 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = m0 + wm * WTM + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (row >= g.m) continue;
                float v = acc[i][j][r] + bvl;
                if (g.relu) v = v > 0.f ? v : 0.f;
                float* dst = static_cast<float*>(g.c) + row * g.ldc + col;
                if (g.accumulate) v += *dst;
                *dst = v;
            }
        }
}

struct WideFrag {
    bf16x8 a[4], b[2];
};
typedef int v4i32 __attribute__((ext_vector_type(4)));
// The six fragment reads of one 16-deep step as one asm statement.  The compiler does not see
// that their results arrive later, so it places no wait of its own; the kernel waits by count
// (WIDE_WAIT_LDS).  Written as plain loads, a step's reads are waited for right where they are
// issued (the compiler keeps one set of fragment registers), and every step then costs a wave
// two LDS round trips on top of its MFMAs.
// a_addr / b_addr: LDS byte address of this lane's chunk in row block 0 of the A / B tile; the
// other row blocks are 32 rows (4096 bytes) further each.
__device__ inline void wide_frags(WideFrag& f, uint32_t a_addr, uint32_t b_addr)
{
    v4i32 a0, a1, a2, a3, b0, b1;
    asm volatile(
        "ds_read_b128 %0, %6\n\t"
        "ds_read_b128 %4, %7\n\t"
        "ds_read_b128 %1, %6 offset:4096\n\t"
        "ds_read_b128 %5, %7 offset:4096\n\t"
        "ds_read_b128 %2, %6 offset:8192\n\t"
        "ds_read_b128 %3, %6 offset:12288"
        : "=&v"(a0), "=&v"(a1), "=&v"(a2), "=&v"(a3), "=&v"(b0), "=&v"(b1)
        : "v"(a_addr), "v"(b_addr)
        : "memory");
    f.a[0] = __builtin_bit_cast(bf16x8, a0);
    f.a[1] = __builtin_bit_cast(bf16x8, a1);
    f.a[2] = __builtin_bit_cast(bf16x8, a2);
    f.a[3] = __builtin_bit_cast(bf16x8, a3);
    f.b[0] = __builtin_bit_cast(bf16x8, b0);
    f.b[1] = __builtin_bit_cast(bf16x8, b1);
}
__device__ inline void wide_mfma(floatx16 (&acc)[4][2], const WideFrag& f)
{
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b[j], acc[i][j], 0, 0, 0);
}
// waits until at most `pending` of this wavefront's LDS reads are outstanding (6: the step just
// requested; 0: none), and keeps the compiler from moving anything across
#define WIDE_WAIT_LDS(pending)                                             \
    do {                                                                   \
        __builtin_amdgcn_sched_barrier(0);                                 \
        __builtin_amdgcn_s_waitcnt(0xC07F | ((pending) << 8));             \
        __builtin_amdgcn_sched_barrier(0);                                 \
    } while (0)

// The same kernel with the fragment reads of step s + 1 issued before the MFMAs of step s.  The
// barrier that opens stage t + 1 sits before the last step of stage t: by then a wave has read
// all of stage t into registers, so after the barrier it issues the loads of stage t + 2 into
// that buffer, asks for the first fragments of stage t + 1, and only then runs the last step's
// MFMAs.
__global__ __launch_bounds__(WTHREADS) void k_gemm_bf16_wide_pipe(const Args g)
{
    extern __shared__ __attribute__((aligned(1024))) char wlds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    int64_t mtile;
    int32_t ntile;
    if (!tile_of_block(blockIdx.x, (g.m + WBM - 1) / WBM, g.nt_1d, mtile, ntile)) return;
    const int64_t m0 = mtile * WBM;
    const int32_t n0 = ntile * WBN;
    const int nstages = g.kseg[0] / WBK;

    floatx16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    wide_issue(g.a[0], g.lda[0], m0, g.m, 0, wlds, wave, lane);
    wide_issue(g.b[0], g.ldb[0], n0, g.n, 0, wlds + WBM * WROWB, wave, lane);
    if (nstages > 1) {
        wide_issue(g.a[0], g.lda[0], m0, g.m, WBK, wlds + WSTAGE, wave, lane);
        wide_issue(g.b[0], g.ldb[0], n0, g.n, WBK, wlds + WSTAGE + WBM * WROWB, wave, lane);
        __builtin_amdgcn_s_waitcnt(0x0F78);           // vmcnt(8): stage 0 landed, stage 1 may be in flight
    } else {
        __builtin_amdgcn_s_waitcnt(0x0F70);
    }
    __syncthreads();
    // this lane's fragment addresses in buffer 0: step ks is chunk 2 ks + half, stored in slot
    // (2 ks + half) ^ ((x >> 1) & 7) of row x, i.e. 16 * ((half ^ sw) ^ 2 ks) with sw = (xl >> 1) & 7
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)wlds;
    const int xl = lane & 31, half = lane >> 5;
    const uint32_t sw16 = (uint32_t)((half ^ ((xl >> 1) & 7)) << 4);
    const uint32_t a_base = lds0 + (uint32_t)((wm * WTM + xl) * WROWB);
    const uint32_t b_base = lds0 + (uint32_t)(WBM * WROWB + (wn * WTN + xl) * WROWB);
    WideFrag f0, f1;
    wide_frags(f0, a_base + sw16, b_base + sw16);
    WIDE_WAIT_LDS(0);
    for (int t = 0; t < nstages; ++t) {
        const uint32_t cur = (uint32_t)((t & 1) * WSTAGE), nxt = (uint32_t)(((t + 1) & 1) * WSTAGE);
        wide_frags(f1, a_base + cur + (sw16 ^ 32u), b_base + cur + (sw16 ^ 32u));
        WIDE_WAIT_LDS(6);
        wide_mfma(acc, f0);
        wide_frags(f0, a_base + cur + (sw16 ^ 64u), b_base + cur + (sw16 ^ 64u));
        WIDE_WAIT_LDS(6);
        wide_mfma(acc, f1);
        wide_frags(f1, a_base + cur + (sw16 ^ 96u), b_base + cur + (sw16 ^ 96u));
        WIDE_WAIT_LDS(6);
        wide_mfma(acc, f0);
        WIDE_WAIT_LDS(0);                              // all of stage t is in registers
        if (t + 1 < nstages) {
            __builtin_amdgcn_s_waitcnt(0x0F70);       // stage t + 1 landed (this thread's loads)
            __syncthreads();                           // ... everybody's; nobody reads stage t any more
            if (t + 2 < nstages) {
                wide_issue(g.a[0], g.lda[0], m0, g.m, (int64_t)(t + 2) * WBK, wlds + cur, wave, lane);
                wide_issue(g.b[0], g.ldb[0], n0, g.n, (int64_t)(t + 2) * WBK, wlds + cur + WBM * WROWB, wave, lane);
            }
            wide_frags(f0, a_base + nxt + sw16, b_base + nxt + sw16);
            __builtin_amdgcn_sched_barrier(0);
        }
        wide_mfma(acc, f1);
        WIDE_WAIT_LDS(0);                              // f0 is there before the values cross the loop edge
    }
    wide_store(g, acc, wlds, m0, n0, wave, lane, wm, wn);
}

// requires: one K segment, K a multiple of 64, 16-byte aligned rows of A and B
__global__ __launch_bounds__(WTHREADS) void k_gemm_bf16_wide(const Args g)
{
    extern __shared__ __attribute__((aligned(1024))) char wlds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 2, wn = wave & 3;
    int64_t mtile;
    int32_t ntile;
    if (!tile_of_block(blockIdx.x, (g.m + WBM - 1) / WBM, g.nt_1d, mtile, ntile)) return;
    const int64_t m0 = mtile * WBM;
    const int32_t n0 = ntile * WBN;
    const int nstages = g.kseg[0] / WBK;

    floatx16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    wide_issue(g.a[0], g.lda[0], m0, g.m, 0, wlds, wave, lane);
    wide_issue(g.b[0], g.ldb[0], n0, g.n, 0, wlds + WBM * WROWB, wave, lane);
    for (int t = 0; t < nstages; ++t) {
        const int buf = t & 1;
        __builtin_amdgcn_s_waitcnt(0x0F70);           // vmcnt(0): this thread's loads of stage t landed
        __syncthreads();                               // everybody's did; stage t - 1 is no longer read
        if (t + 1 < nstages) {
            char* nxt = wlds + (buf ^ 1) * WSTAGE;
            wide_issue(g.a[0], g.lda[0], m0, g.m, (int64_t)(t + 1) * WBK, nxt, wave, lane);
            wide_issue(g.b[0], g.ldb[0], n0, g.n, (int64_t)(t + 1) * WBK, nxt + WBM * WROWB, wave, lane);
        }
        const char* As = wlds + buf * WSTAGE;
        const char* Bs = As + WBM * WROWB;
        const int xl = lane & 31, half = lane >> 5;
#pragma unroll
        for (int ks = 0; ks < WBK / 16; ++ks) {
            bf16x8 av[4], bv[2];
            const int c = 2 * ks + half;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                av[i] = *reinterpret_cast<const bf16x8*>(As + wide_chunk(wm * WTM + 32 * i + xl, c));
#pragma unroll
            for (int j = 0; j < 2; ++j)
                bv[j] = *reinterpret_cast<const bf16x8*>(Bs + wide_chunk(wn * WTN + 32 * j + xl, c));
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[j], acc[i][j], 0, 0, 0);
        }
    }

    wide_store(g, acc, wlds, m0, n0, wave, lane, wm, wn);
}

// ---------------------------------------------------------------------------------------------
// The same product on a persistent grid, for bf16 results: one workgroup per CU walks its tiles
// (tile_of_block order, a grid stride apart) in one continuous sequence of K stages, so that
//   * the first stage of the next tile is loaded while the last stage of this one is multiplied
//     (no pipeline fill per tile), and
//   * a finished tile leaves the accumulators as packed bf16 pairs (64 registers), and each K
//     stage of the next tile stores one sixteenth of it: 8 rows of the wavefront's columns,
//     straight from the registers in 64-byte pieces (the stores cost the loop nothing; a turn
//     through LDS to make them 16 bytes per lane cost 700 cycles a stage in waits).
// What this is for: a tile's 128 KB of results written in one burst by every CU at the same time
// (the tiles of a launch run in step) leaves at the chip's write rate, and the store instructions
// stall at issue meanwhile - a quarter of the tile's time with K = 1024.  Spread over the next
// tile's stages the same bytes leave while the matrix pipe works.
constexpr int PLDS = 2 * WSTAGE;

// Byte offsets of this lane's four 16-byte pieces of a stage tile, from the tile's first row
// (rows past the end: the last valid row, whose values are never used).
__device__ inline void persist_offsets(int64_t ld, int64_t row0, int64_t nrows, int wave, int lane, uint32_t (&off)[4])
{
    const int64_t last = nrows - 1 - row0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = (j * 8 + wave) * 8 + (lane >> 3);
        const int c = (lane & 7) ^ ((row >> 1) & 7);   // LDS slot lane & 7 of the row holds chunk c
        const int64_t rl = row < last ? row : last;
        off[j] = (uint32_t)((rl * ld + c * 8) * 2);
    }
}
// One operand tile of a stage; base: the tile's first row at this stage's k (uniform).
__device__ inline void persist_issue(const bf16_t* base, const uint32_t (&off)[4], char* lds_tile, int wave)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int q = j * 8 + wave;                    // block of 8 rows = 1 KB of LDS
        const char* src = reinterpret_cast<const char*>(base) + off[j];
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                         (__attribute__((address_space(3))) void*)(lds_tile + q * 1024), 16, 0, 0);
    }
}

struct ParkedTile {
    uint32_t v[64];       // (i, j, r even | r odd << 16): index (i * 2 + j) * 8 + r / 2
    int64_t m0;
    int32_t n0;
};

// Stores chunk `chunk` (0..15) of the parked tile: rows 8 chunk .. + 7 of the wavefront's 128, its
// 64 columns, straight from the MFMA layout: lane (half, xl) holds column 32 j + xl of rows
// 4 half + 2 h and + 1, so a store instruction writes 64 contiguous bytes of two rows, and the two
// column blocks complete each 128-byte line right after one another.  Only the choice of the four
// registers depends on the chunk at compile time.
__device__ inline void persist_store(const Args& g, const ParkedTile& pk, int chunk, int lane, int wm, int wn)
{
    uint32_t pr[2][2];                                 // [j][h]
    switch (chunk) {
#define GNN_CHUNK(C)                                                       \
    case C:                                                                \
        pr[0][0] = pk.v[((C) / 4 * 2 + 0) * 8 + 2 * ((C) % 4)];            \
        pr[0][1] = pk.v[((C) / 4 * 2 + 0) * 8 + 2 * ((C) % 4) + 1];        \
        pr[1][0] = pk.v[((C) / 4 * 2 + 1) * 8 + 2 * ((C) % 4)];            \
        pr[1][1] = pk.v[((C) / 4 * 2 + 1) * 8 + 2 * ((C) % 4) + 1];        \
        break;
        GNN_CHUNK(0) GNN_CHUNK(1) GNN_CHUNK(2) GNN_CHUNK(3) GNN_CHUNK(4) GNN_CHUNK(5) GNN_CHUNK(6) GNN_CHUNK(7)
        GNN_CHUNK(8) GNN_CHUNK(9) GNN_CHUNK(10) GNN_CHUNK(11) GNN_CHUNK(12) GNN_CHUNK(13) GNN_CHUNK(14) GNN_CHUNK(15)
#undef GNN_CHUNK
        default: return;
    }
    const int half = lane >> 5, xl = lane & 31;
    const int64_t row0 = pk.m0 + wm * WTM + 8 * chunk + 4 * half;
    const int32_t col0 = pk.n0 + wn * WTN + xl;
    bf16_t* cp = static_cast<bf16_t*>(g.c) + row0 * g.ldc + col0;
    const bool interior = pk.m0 + WBM <= g.m && pk.n0 + WBN <= g.n;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            if (!interior && col0 + 32 * j >= g.n) continue;
            if (interior || row0 + 2 * h < g.m) cp[(2 * h) * g.ldc + 32 * j] = (bf16_t)(pr[j][h] & 0xFFFFu);
            if (interior || row0 + 2 * h + 1 < g.m) cp[(2 * h + 1) * g.ldc + 32 * j] = (bf16_t)(pr[j][h] >> 16);
        }
}

// requires: one K segment, K a multiple of 64, 16-byte aligned rows of A and B, bf16 result
// without accumulation; total = padded number of linear tile indices
__global__ __launch_bounds__(WTHREADS) void k_gemm_bf16_persist(const Args g, const int32_t total)
{
    extern __shared__ __attribute__((aligned(1024))) char wlds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: kept in scalar registers
    const int wm = wave >> 2, wn = wave & 3;
    const int32_t mt = (int32_t)((g.m + WBM - 1) / WBM);
    const int nstages = g.kseg[0] / WBK;

    // the tile of linear index `from`, or of the next index a grid stride further that owns one
    // (padding indices own none); same order as tile_of_block
    auto next_tile = [&](int32_t from, int32_t& mtile, int32_t& ntile) {
        for (; from < total; from += (int32_t)gridDim.x) {
            const int32_t slot = from >> 3;
            ntile = slot % g.nt_1d;
            mtile = slot / g.nt_1d * 8 + (from & 7);
            if (mtile < mt) break;
        }
        return from;
    };
    int32_t mtile = 0, mtile_n = 0;
    int32_t ntile = 0, ntile_n = 0;
    int32_t idx = next_tile((int32_t)blockIdx.x, mtile, ntile);
    if (idx >= total) return;

    floatx16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    ParkedTile pk;
#pragma unroll
    for (int q = 0; q < 64; ++q) pk.v[q] = 0u;
    pk.m0 = 0;
    pk.n0 = 0;
    bool parked = false;

    int buf = 0;
    uint32_t offa[4], offb[4];
    persist_offsets(g.lda[0], (int64_t)mtile * WBM, g.m, wave, lane, offa);
    persist_offsets(g.ldb[0], (int64_t)ntile * WBN, g.n, wave, lane, offb);
    persist_issue(g.a[0] + (int64_t)mtile * WBM * g.lda[0], offa, wlds, wave);
    persist_issue(g.b[0] + (int64_t)ntile * WBN * g.ldb[0], offb, wlds + WBM * WROWB, wave);
    const int xl = lane & 31, half = lane >> 5;
    while (true) {
        const int32_t idx_n = next_tile(idx + (int32_t)gridDim.x, mtile_n, ntile_n);
        const bool has_next = idx_n < total;
        const int64_t m0 = (int64_t)mtile * WBM;
        const int32_t n0 = ntile * WBN;
        int chunk = 0, due = 0;                        // 16 chunks spread evenly over the stages
        for (int t = 0; t < nstages; ++t) {
            __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0): this thread's loads of the stage landed
            __syncthreads();                           // everybody's did; the other buffer is no longer read
            char* nxt = wlds + (buf ^ 1) * WSTAGE;
            if (t + 1 < nstages) {
                persist_issue(g.a[0] + m0 * g.lda[0] + (int64_t)(t + 1) * WBK, offa, nxt, wave);
                persist_issue(g.b[0] + (int64_t)n0 * g.ldb[0] + (int64_t)(t + 1) * WBK, offb, nxt + WBM * WROWB, wave);
            } else if (has_next) {
                // (the tile numbers pass through an empty asm so that none of this is computed,
                // and kept in registers, before the loop)
                int32_t mn = mtile_n, nn = ntile_n;
                asm volatile("" : "+s"(mn), "+s"(nn));
                persist_offsets(g.lda[0], (int64_t)mn * WBM, g.m, wave, lane, offa);
                persist_offsets(g.ldb[0], (int64_t)nn * WBN, g.n, wave, lane, offb);
                persist_issue(g.a[0] + (int64_t)mn * WBM * g.lda[0], offa, nxt, wave);
                persist_issue(g.b[0] + (int64_t)nn * WBN * g.ldb[0], offb, nxt + WBM * WROWB, wave);
            }
            const char* As = wlds + buf * WSTAGE;
            const char* Bs = As + WBM * WROWB;
#pragma unroll
            for (int ks = 0; ks < WBK / 16; ++ks) {
                bf16x8 av[4], bv[2];
                const int c = 2 * ks + half;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    av[i] = *reinterpret_cast<const bf16x8*>(As + wide_chunk(wm * WTM + 32 * i + xl, c));
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    bv[j] = *reinterpret_cast<const bf16x8*>(Bs + wide_chunk(wn * WTN + 32 * j + xl, c));
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[j], acc[i][j], 0, 0, 0);
                // one sixteenth of the parked tile per stage (more when K < 1024), after a
                // step's MFMAs are issued; the two wavefronts of a SIMD (w and w + 4: the two
                // values of wm) at different steps
                if (ks == (wm == 1 ? 2 : 0) && parked)
                    for (due += 16; due >= nstages; due -= nstages) persist_store(g, pk, chunk++, lane, wm, wn);
            }
            buf ^= 1;
        }
        // the tile is complete: + bias, max(., 0), round, park; the accumulators start over
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int32_t col = n0 + wn * WTN + 32 * j + (lane & 31);
            const float bvl = (g.bias && col < g.n) ? g.bias[col] : 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    float v0 = acc[i][j][r] + bvl, v1 = acc[i][j][r + 1] + bvl;
                    if (g.relu) {
                        v0 = v0 > 0.f ? v0 : 0.f;
                        v1 = v1 > 0.f ? v1 : 0.f;
                    }
                    pk.v[(i * 2 + j) * 8 + r / 2] = pack_bf16(v0, v1);
                    acc[i][j][r] = 0.f;
                    acc[i][j][r + 1] = 0.f;
                }
        }
        pk.m0 = m0;
        pk.n0 = n0;
        parked = true;
        if (!has_next) break;
        idx = idx_n;
        mtile = mtile_n;
        ntile = ntile_n;
    }
    for (int ch = 0; ch < 16; ++ch) persist_store(g, pk, ch, lane, wm, wn);
}

// Whether the wide kernel can take this product (both operands k-contiguous is the caller's business).
bool wide_ok(const Args& g)
{
    static const bool enabled = [] {
        const char* e = getenv("GNNMI_GEMM_WIDE");
        return !(e && e[0] == '0');
    }();
    if (!enabled || g.kseg[1] != 0 || g.split_chunk != 0) return false;
    if (g.m < 2 * WBM || g.n < WBN || g.kseg[0] < WBK || g.kseg[0] % WBK != 0) return false;
    if (!aligned16(g.a[0]) || !aligned16(g.b[0]) || g.lda[0] % 8 != 0 || g.ldb[0] % 8 != 0) return false;
    if (g.out_bf16 && (!aligned16(g.c) || g.ldc % 8 != 0)) return false;
    return true;
}

bool launch_wide(const Args& g, hipStream_t s)
{
    static const bool attr_ok = hipFuncSetAttribute((const void*)k_gemm_bf16_wide,
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, WLDS) == hipSuccess;
    static const bool persist_ok = hipFuncSetAttribute((const void*)k_gemm_bf16_persist,
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, PLDS) == hipSuccess;
    static const bool persist = [] {
        const char* e = getenv("GNNMI_GEMM_PERSIST");
        return !(e && e[0] == '0');
    }();
    // one workgroup fits a CU (LDS), and the grid is one workgroup per CU
    static const int cus = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8)
            return 0;
        return n / 8 * 8;
    }();
    const int64_t mt = (g.m + WBM - 1) / WBM;
    const int32_t nt = (g.n + WBN - 1) / WBN;
    Args ga = g;
    ga.nt_1d = nt;
    const int64_t total = (mt + 7) / 8 * 8 * nt;
    if (persist && persist_ok && cus > 0 && g.out_bf16 && !g.accumulate && total < (1 << 30)) {
        const int64_t grid = total < cus ? total : cus;
        hipLaunchKernelGGL(k_gemm_bf16_persist, dim3((unsigned)grid), dim3(WTHREADS), PLDS, s, ga, (int32_t)total);
        return true;
    }
    if (!attr_ok) return false;
    static const bool pipe_ok = hipFuncSetAttribute((const void*)k_gemm_bf16_wide_pipe,
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, WLDS) == hipSuccess;
    static const bool pipe = [] {
        const char* e = getenv("GNNMI_GEMM_PIPE");
        return !(e && e[0] == '0');
    }();
    if (pipe && pipe_ok)
        hipLaunchKernelGGL(k_gemm_bf16_wide_pipe, dim3((unsigned)total), dim3(WTHREADS), WLDS, s, ga);
    else
        hipLaunchKernelGGL(k_gemm_bf16_wide, dim3((unsigned)total), dim3(WTHREADS), WLDS, s, ga);
    return true;
}

__global__ __launch_bounds__(256) void k_transpose_bf16(const bf16_t* __restrict__ src, int64_t ld, int32_t k,
                                                        int32_t n, bf16_t* __restrict__ dst)
{
    __shared__ bf16_t tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;     // 32 x 8
    const int32_t k0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
    for (int i = ty; i < 32; i += 8)
        tile[i][tx] = (k0 + i < k && n0 + tx < n) ? src[(int64_t)(k0 + i) * ld + n0 + tx] : (bf16_t)0;
    __syncthreads();
    for (int i = ty; i < 32; i += 8)
        if (n0 + i < n && k0 + tx < k) dst[(int64_t)(n0 + i) * k + k0 + tx] = tile[tx][i];
}

// ---------------------------------------------------------------------------------------------
// Wide variant of the reduction over rows, C[m][n] = sum_k A[k][m] B[k][n] (grad W = Z^T dY):
// the same 256 x 256 tile, 64 k-rows per stage and direct-to-LDS loads.  Both operands arrive
// [k][m] (m contiguous), the MFMA wants eight consecutive k per lane: fragments are fetched
// with the LDS transpose read (ds_read_b64_tr_b16).  Within a group of 16 lanes, lane j hands
// in the address of four consecutive 16-bit elements, taken as row j / 4, columns
// 4 (j % 4) .. + 3 of a 4 x 16 block, and lane i receives column i of that block - here rows
// are k and columns are m, so a lane gets four consecutive k of its m; two reads make the
// operand.  The 16-byte chunks of a k-row are permuted by the row number so that the four
// k-rows of one read fall into different banks (applied on the global side, as above).
// K is split over blockIdx.z into fp32 partial tiles, reduced afterwards in a fixed order.
typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef short v8i16 __attribute__((ext_vector_type(8)));
constexpr int TROWB = WBM * 2;                         // bytes per k-row of an operand tile
constexpr int TOP = WBK * TROWB;                       // bytes per operand tile
constexpr int TSTAGE = 2 * TOP;
constexpr int TLDS = 2 * TSTAGE;

struct ArgsT {
    const bf16_t* a;
    const bf16_t* b;
    int64_t lda, ldb;
    float* partial;            // [splits][m][n]
    int32_t m, n;
    int64_t k;                 // rows covered, a multiple of 64
    int64_t chunk;             // rows per split, a multiple of 64
    int32_t splits;            // > 0: one-dimensional grid, see k_gemm_bf16_tn_wide
};

__device__ inline int tn_off(int k, int mcol)          // byte offset of element (k, mcol), mcol % 4 == 0
{
    return k * TROWB + ((((mcol >> 3) ^ ((k & 3) << 1)) << 4) | ((mcol & 4) << 1));
}

__device__ inline void tn_issue(const bf16_t* __restrict__ p, int64_t ld, int64_t krow0, int32_t col0,
                                int32_t ncols, char* lds_tile, int wave, int lane)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int q = j * 8 + wave;                    // two k-rows = 1 KB of LDS
        const int k = 2 * q + (lane >> 5);
        const int mc = (lane & 31) ^ ((k & 3) << 1);
        int32_t col = col0 + mc * 8;
        col = col + 8 <= ncols ? col : 0;              // chunks past the end: valid address, result unused
        const bf16_t* src = p + (krow0 + k) * ld + col;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                         (__attribute__((address_space(3))) void*)(lds_tile + q * 1024), 16, 0, 0);
    }
}

// eight consecutive k (k8 .. k8 + 7) of this lane's row in the 32-column block starting at c0
__device__ inline bf16x8 tn_fragment(const char* tile, int k8, int c0, int lane)
{
    const int j = lane & 15, grp = lane >> 4;
    const int mcol = c0 + 16 * (grp & 1) + 4 * (j & 3);
    const int k = k8 + (j >> 2);
    const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) v4i16*)(tile + tn_off(k, mcol)));
    const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) v4i16*)(tile + tn_off(k + 4, mcol)));
    v8i16 r;
    r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
    r[4] = hi[0]; r[5] = hi[1]; r[6] = hi[2]; r[7] = hi[3];
    return __builtin_bit_cast(bf16x8, r);
}

// requires: m, n multiples of 8; rows of A and B 16-byte aligned; k and chunk multiples of 64
__global__ __launch_bounds__(WTHREADS) void k_gemm_bf16_tn_wide(const ArgsT g)
{
    extern __shared__ __attribute__((aligned(1024))) char wlds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 2, wn = wave & 3;
    // One-dimensional grid (splits > 0): workgroups are dealt to the 8 XCDs round-robin, and
    // every tile of one K split runs on the same XCD, so the 64-row stages of A and B that the
    // tiles of a split share are fetched into that XCD's L2 once instead of once per tile.
    int32_t bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
    if (g.splits > 0) {
        const int32_t mt = (g.m + WBM - 1) / WBM, nt = (g.n + WBN - 1) / WBN, tiles = mt * nt;
        const int32_t slot = blockIdx.x >> 3, xcd = blockIdx.x & 7;
        bz = (slot / tiles) * 8 + xcd;
        if (bz >= g.splits) return;
        const int32_t tile = slot % tiles;
        bx = tile % mt;
        by = tile / mt;
    }
    const int32_t m0 = bx * WBM, n0 = by * WBN;
    const int64_t kbeg = (int64_t)bz * g.chunk;
    const int64_t kend = kbeg + g.chunk < g.k ? kbeg + g.chunk : g.k;
    const int nstages = kend > kbeg ? (int)((kend - kbeg) / WBK) : 0;

    floatx16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    if (nstages > 0) {
        tn_issue(g.a, g.lda, kbeg, m0, g.m, wlds, wave, lane);
        tn_issue(g.b, g.ldb, kbeg, n0, g.n, wlds + TOP, wave, lane);
    }
    for (int t = 0; t < nstages; ++t) {
        const int buf = t & 1;
        __builtin_amdgcn_s_waitcnt(0x0F70);           // vmcnt(0)
        __syncthreads();
        if (t + 1 < nstages) {
            char* nxt = wlds + (buf ^ 1) * TSTAGE;
            tn_issue(g.a, g.lda, kbeg + (int64_t)(t + 1) * WBK, m0, g.m, nxt, wave, lane);
            tn_issue(g.b, g.ldb, kbeg + (int64_t)(t + 1) * WBK, n0, g.n, nxt + TOP, wave, lane);
        }
        const char* As = wlds + buf * TSTAGE;
        const char* Bs = As + TOP;
        const int khalf = (lane >> 5) * 8;
#pragma unroll
        for (int ks = 0; ks < WBK / 16; ++ks) {
            bf16x8 av[4], bv[2];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = tn_fragment(As, 16 * ks + khalf, wm * WTM + 32 * i, lane);
#pragma unroll
            for (int j = 0; j < 2; ++j) bv[j] = tn_fragment(Bs, 16 * ks + khalf, wn * WTN + 32 * j, lane);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[j], acc[i][j], 0, 0, 0);
        }
    }
    float* out = g.partial + (int64_t)bz * g.m * g.n;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int32_t col = n0 + wn * WTN + 32 * j + (lane & 31);
            if (col >= g.n) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int32_t row = m0 + wm * WTM + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (row < g.m) out[(int64_t)row * g.n + col] = acc[i][j][r];
            }
        }
}

bool wide_tn_ok(const void* a, int64_t lda, const void* b, int64_t ldb, int32_t m, int32_t n, int64_t kdim)
{
    static const bool enabled = [] {
        const char* e = getenv("GNNMI_GEMM_WIDE");
        return !(e && e[0] == '0');
    }();
    return enabled && m >= WBM && n >= WBN && m % 8 == 0 && n % 8 == 0 && kdim >= 64 * WBK && aligned16(a) &&
           aligned16(b) && lda % 8 == 0 && ldb % 8 == 0;
}

int wide_tn_splits(int64_t kdim, int32_t m, int32_t n)
{
    const int64_t tiles = (int64_t)((m + WBM - 1) / WBM) * ((n + WBN - 1) / WBN);
    int64_t want = (512 + tiles - 1) / tiles;          // two workgroups per CU over the launch
    const int64_t most = kdim / (16 * WBK);            // at least 16 stages per split
    int64_t sp = want < most ? want : most;
    sp = sp > 64 ? 64 : sp;
    return (int)(sp < 1 ? 1 : sp);
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
                         int64_t m, int32_t n, const GemmEpilogue& ep, hipStream_t s, void* bt_scratch)
{
    if (bt_scratch && nseg == 1) {
        // large product: transpose B (the weights, small) and take the wide kernel
        Args w{};
        w.a[0] = w.a[1] = (const bf16_t*)segs[0].a; w.lda[0] = w.lda[1] = segs[0].lda;
        w.b[0] = w.b[1] = (const bf16_t*)bt_scratch; w.ldb[0] = w.ldb[1] = segs[0].k;
        w.kseg[0] = segs[0].k;
        w.c = c; w.ldc = ldc; w.m = m; w.n = n; w.out_bf16 = out_bf16;
        w.bias = ep.bias; w.relu = ep.relu; w.accumulate = ep.accumulate;
        if (wide_ok(w)) {
            hipLaunchKernelGGL(k_transpose_bf16, dim3((unsigned)((n + 31) / 32), (unsigned)((segs[0].k + 31) / 32)),
                               dim3(256), 0, s, (const bf16_t*)segs[0].b, segs[0].ldb, segs[0].k, n,
                               (bf16_t*)bt_scratch);
            if (launch_wide(w, s)) return;
        }
    }
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
    if (wide_ok(g) && launch_wide(g, s)) return;
    launch<true, true>(g, 1, s);
}

void launch_gemm_bf16_tn(const void* a, int64_t lda, const void* b, int64_t ldb, float* c,
                         int64_t ldc, int32_t m, int32_t n, int64_t kdim, float* partial,
                         hipStream_t s)
{
    if (kdim <= 0 || m <= 0 || n <= 0) return;
    if (wide_tn_ok(a, lda, b, ldb, m, n, kdim)) {
        static const bool attr_ok = hipFuncSetAttribute((const void*)k_gemm_bf16_tn_wide,
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, TLDS) == hipSuccess;
        if (attr_ok) {
            // whole stages of 64 rows on the wide kernel, the last rows (fewer than 64) below
            ArgsT w{};
            w.a = (const bf16_t*)a; w.lda = lda; w.b = (const bf16_t*)b; w.ldb = ldb;
            w.partial = partial; w.m = m; w.n = n;
            w.k = kdim / WBK * WBK;
            const int want = wide_tn_splits(kdim, m, n);
            w.chunk = (w.k / WBK + want - 1) / want * WBK;
            const int sp = (int)((w.k + w.chunk - 1) / w.chunk);
            static const bool by_split = [] {
                const char* e = getenv("GNNMI_GEMM_TN_XCD");
                return !(e && e[0] == '0');
            }();
            const unsigned mt = (unsigned)((m + WBM - 1) / WBM), nt = (unsigned)((n + WBN - 1) / WBN);
            if (by_split && mt * nt > 1) {
                w.splits = sp;
                hipLaunchKernelGGL(k_gemm_bf16_tn_wide, dim3((unsigned)((sp + 7) / 8 * 8) * mt * nt), dim3(WTHREADS),
                                   TLDS, s, w);
            } else {
                w.splits = 0;
                hipLaunchKernelGGL(k_gemm_bf16_tn_wide, dim3(mt, nt, (unsigned)sp), dim3(WTHREADS), TLDS, s, w);
            }
            launch_reduce_partials(partial, sp, (int64_t)m * n, c, ldc, m, n, s);
            if (w.k == kdim) return;
            a = (const bf16_t*)a + w.k * lda;
            b = (const bf16_t*)b + w.k * ldb;
            kdim -= w.k;
        }
    }
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

int64_t gemm_bf16_tn_partial_floats(int64_t kdim, int32_t m, int32_t n)
{
    const int64_t narrow = (int64_t)gemm_tn_splits(kdim, m, n) * m * n;
    const int64_t wide = (int64_t)wide_tn_splits(kdim, m, n) * m * n;
    return narrow > wide ? narrow : wide;
}

void launch_to_bf16(const float* src, void* dst, int64_t n, hipStream_t s)
{
    if (n <= 0) return;
    int64_t blocks = (n + 255) / 256;
    blocks = blocks > 16384 ? 16384 : blocks;
    hipLaunchKernelGGL(k_to_bf16, dim3((unsigned)blocks), dim3(256), 0, s, src, (bf16_t*)dst, n);
}

}  // namespace gnnmi
