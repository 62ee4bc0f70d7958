// Dense contractions of the path on the fp32 matrix cores (v_mfma_f32_32x32x2_f32), gfx950.
//
//   forward   A_p^l  = act( Z_p W^l (+ X_p W_s^l) + b^l )        [n_p x d_in] [d_in x d_out]
//   backward  dZ_p   = dY_p (W^l)^T                              [n_p x d_out][d_out x d_in]
//             grad W^l += Z_p^T dY_p                             reduction over the n_p rows
//
// One workgroup of 4 wavefronts (2 x 2) owns a BM x BN tile of C.  K is walked in steps of 16
// through a double-buffered LDS stage.  An operand whose k index is the contiguous one in
// memory is kept [x][k] in LDS (chunks rotated per row, see kf_chunk) and an MFMA lane fetches
// eight k of its row with two 16-byte reads; an operand whose m (or n) index is contiguous is
// kept [k][x], so that the 32 lanes feeding one MFMA operand column read 32 consecutive floats.
// Widths that are not multiples of 4 floats (e.g. 47 classes) take a scalar-load variant of the
// same kernel; tails in M, N and K are zero-filled in LDS, never in memory.
#include "gnn_internal.h"
#include <cstdlib>

namespace gnnmi {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int BK = 16;
constexpr int PF = 1;   // stages of global loads in flight per thread; 2 and 3 measured slower, also on
                        // the narrow (48-wide) contractions: those are bound by the MFMA work of
                        // their padded 64-wide tile, not by loads in flight
constexpr int SUB = 1;  // k-tiles of BK per LDS stage (one barrier per stage); 2 measured slower:
                        // the forward contraction loses more to the larger LDS footprint than
                        // the halved barrier count gains
constexpr int PAD = 4;

struct Operand {         // a matrix operand restricted to one K segment
    const float* p;
    int64_t ld;
};

// Tile whose k index is the contiguous one in memory: (slow = m or n, fast = k).
// Thread t covers slow = t / 4 + 64 i, k = 4 (t % 4) .. + 3.
template <int BT, bool VEC>
__device__ inline void load_kfast(const float* __restrict__ p, int64_t ld, int64_t slow0,
                                  int64_t nslow, int32_t k0, int32_t kend, float4 (&r)[BT / 64])
{
    const int t = threadIdx.x;
    const int kq = (t & 3) * 4;
#pragma unroll
    for (int i = 0; i < BT / 64; ++i) {
        const int64_t sidx = slow0 + (t >> 2) + 64 * i;
        const int32_t k = k0 + kq;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (VEC) {
            // unconditional load from a clamped (always valid) address, zeroed afterwards:
            // without branches the compiler can keep several tiles of loads in flight
            const float* q = p + (sidx < nslow ? sidx : nslow - 1) * ld + (k < kend ? k : k0);
            const float4 x = *reinterpret_cast<const float4*>(q);
            v = x;   // rows / k past the end are zeroed when the tile goes to LDS
        } else if (sidx < nslow) {
            const float* q = p + sidx * ld + k;
            {
                if (k + 0 < kend) v.x = q[0];
                if (k + 1 < kend) v.y = q[1];
                if (k + 2 < kend) v.z = q[2];
                if (k + 3 < kend) v.w = q[3];
            }
        }
        r[i] = v;
    }
}
// k-fast tiles are kept [x][k] in LDS: one 16-byte store per register, and an MFMA lane later
// fetches eight consecutive k of its row with two 16-byte reads.  Rows are BK floats apart and
// the four 16-byte chunks of row x are rotated by x / 4: sixteen consecutive lanes then touch
// all 64 banks exactly once both when storing (4 rows x 4 chunks) and when reading (16 rows,
// one chunk each); a padded row stride can satisfy only one of the two.
constexpr int KF_LD = BK;
__device__ inline int kf_chunk(int x, int chunk) { return 4 * ((chunk + (x >> 2)) & 3); }
template <int BT>
__device__ inline void store_kfast(float* S, const float4 (&r)[BT / 64])
{
    const int t = threadIdx.x;
#pragma unroll
    for (int i = 0; i < BT / 64; ++i) {
        const int x = (t >> 2) + 64 * i;
        *reinterpret_cast<float4*>(S + x * KF_LD + kf_chunk(x, t & 3)) = r[i];
    }
}

// Tile whose m (or n) index is the contiguous one: (slow = k, fast = m or n).
// Thread t covers k = t / (BT/4) + (1024/BT) i, fast = 4 (t % (BT/4)) .. + 3.
template <int BT, bool VEC>
__device__ inline void load_kslow(const float* __restrict__ p, int64_t ld, int64_t k0, int64_t kend,
                                  int64_t fast0, int64_t nfast, float4 (&r)[BT / 64])
{
    constexpr int TPR = BT / 4;           // threads per k row
    constexpr int KPP = kThreads / TPR;   // k rows per pass
    const int t = threadIdx.x;
    const int fq = (t % TPR) * 4;
#pragma unroll
    for (int i = 0; i < BT / 64; ++i) {
        const int64_t k = k0 + t / TPR + KPP * i;
        const int64_t f = fast0 + fq;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (VEC) {
            const float* q = p + (k < kend ? k : k0) * ld + (f < nfast ? f : fast0);
            const float4 x = *reinterpret_cast<const float4*>(q);
            v = x;   // rows / k past the end are zeroed when the tile goes to LDS
        } else if (k < kend) {
            const float* q = p + k * ld + f;
            {
                if (f + 0 < nfast) v.x = q[0];
                if (f + 1 < nfast) v.y = q[1];
                if (f + 2 < nfast) v.z = q[2];
                if (f + 3 < nfast) v.w = q[3];
            }
        }
        r[i] = v;
    }
}
template <int BT>
__device__ inline void store_kslow(float* S, const float4 (&r)[BT / 64])
{
    constexpr int TPR = BT / 4;
    constexpr int KPP = kThreads / TPR;
    const int t = threadIdx.x;
    const int fq = (t % TPR) * 4;
#pragma unroll
    for (int i = 0; i < BT / 64; ++i)
        *reinterpret_cast<float4*>(S + (t / TPR + KPP * i) * (BT + PAD) + fq) = r[i];
}

// Fragment of one operand for a whole BK = 16 tile: f[j] is the value this lane feeds to the
// j-th MFMA k-step.  The two half-waves of a 32x32x2 MFMA supply k = 0 and k = 1 of a step;
// here half h supplies k = 8 h + j of the tile at step j (the k order inside a tile is free
// as long as A and B agree), which makes a k-fast row fragment eight consecutive floats.
template <int BT, bool KFAST>
__device__ inline void load_fragment(const float* S, int x, int half, float (&f)[8])
{
    if (KFAST) {
        const float4 lo = *reinterpret_cast<const float4*>(S + x * KF_LD + kf_chunk(x, 2 * half));
        const float4 hi = *reinterpret_cast<const float4*>(S + x * KF_LD + kf_chunk(x, 2 * half + 1));
        f[0] = lo.x; f[1] = lo.y; f[2] = lo.z; f[3] = lo.w;
        f[4] = hi.x; f[5] = hi.y; f[6] = hi.z; f[7] = hi.w;
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) f[j] = S[(8 * half + j) * (BT + PAD) + x];
    }
}

// Zero the vectors of a tile that lie past the end of the matrix (their loads were clamped to
// valid addresses).  Done when the registers are written to LDS, not at load time, so that the
// loads of several tiles stay in flight.
template <int BT>
__device__ inline void mask_kfast(int64_t slow0, int64_t nslow, int64_t k0, int64_t kend, float4 (&r)[BT / 64])
{
    const int t = threadIdx.x;
    const int64_t k = k0 + (t & 3) * 4;
#pragma unroll
    for (int i = 0; i < BT / 64; ++i)
        if (!(slow0 + (t >> 2) + 64 * i < nslow && k < kend)) r[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}
template <int BT>
__device__ inline void mask_kslow(int64_t k0, int64_t kend, int64_t fast0, int64_t nfast, float4 (&r)[BT / 64])
{
    constexpr int TPR = BT / 4;
    constexpr int KPP = kThreads / TPR;
    const int t = threadIdx.x;
    const int64_t f = fast0 + (t % TPR) * 4;
#pragma unroll
    for (int i = 0; i < BT / 64; ++i)
        if (!(k0 + t / TPR + KPP * i < kend && f < nfast)) r[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

struct GemmArgs {
    Operand a[2], b[2];      // up to two K segments
    int32_t kseg[2];         // K of each segment (second may be 0)
    float* c;
    int64_t ldc;
    int64_t m;               // rows of C
    int32_t n;               // columns of C
    const float* bias;
    int32_t relu;
    int32_t accumulate;
    int64_t split_chunk;     // K per split (multiple of BK); 0 = no split
    int64_t split_stride;    // elements between the partial C of consecutive splits
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

// A_KFAST: A(m,k) = a[m*lda + k]   (else a[k*lda + m])
// B_KFAST: B(k,n) = b[n*ldb + k]   (else b[k*ldb + n])
template <int BM, int BN, bool A_KFAST, bool B_KFAST, bool VEC_A, bool VEC_B>
__global__ __launch_bounds__(kThreads) void k_gemm(const GemmArgs g)
{
    constexpr int WM = BM / 2, WN = BN / 2;   // wave tile
    constexpr int TM = WM / 32, TN = WN / 32; // 32x32 MFMA tiles per wave
    constexpr int A_TILE = A_KFAST ? BM * KF_LD : BK * (BM + PAD);
    constexpr int B_TILE = B_KFAST ? BN * KF_LD : BK * (BN + PAD);
    __shared__ __attribute__((aligned(16))) float As[2][SUB * A_TILE];
    __shared__ __attribute__((aligned(16))) float Bs[2][SUB * B_TILE];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wm0 = (wave >> 1) * WM, wn0 = (wave & 1) * WN;
    int64_t mtile = blockIdx.x;
    int32_t ntile = blockIdx.y;
    if (g.nt_1d > 0 && !tile_of_block(blockIdx.x, (g.m + BM - 1) / BM, g.nt_1d, mtile, ntile)) return;
    const int64_t m0 = mtile * BM;
    const int32_t n0 = ntile * BN;

    // K range of this workgroup (split-K only with a single segment)
    int64_t kbeg = 0, kend0 = g.kseg[0];
    float* cbase = g.c;
    if (g.split_chunk > 0) {
        kbeg = (int64_t)blockIdx.z * g.split_chunk;
        kend0 = kbeg + g.split_chunk < kend0 ? kbeg + g.split_chunk : kend0;
        cbase += (int64_t)blockIdx.z * g.split_stride;
    }
    // a stage is SUB consecutive k-tiles of one segment (tiles past the segment's end are zero)
    constexpr int SK = BK * SUB;
    const int64_t tiles0 = kend0 > kbeg ? (kend0 - kbeg + SK - 1) / SK : 0;
    const int64_t tiles1 = (g.kseg[1] + SK - 1) / SK;
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
    float4 ra[PF][SUB][BM / 64], rb[PF][SUB][BN / 64];
    auto load_tile = [&](int64_t t, float4 (&ra)[SUB][BM / 64], float4 (&rb)[SUB][BN / 64]) {
        const int seg = t < tiles0 ? 0 : 1;
        const int64_t ks = seg == 0 ? kbeg + t * SK : (t - tiles0) * SK;
        const int64_t kend = seg == 0 ? kend0 : (int64_t)g.kseg[1];
#pragma unroll
        for (int u = 0; u < SUB; ++u) {
            // a tile wholly past the end is fetched from the segment's first tile and zeroed later
            const int64_t k0 = ks + u * BK < kend ? ks + u * BK : ks;
            if (A_KFAST) load_kfast<BM, VEC_A>(g.a[seg].p, g.a[seg].ld, m0, g.m, (int32_t)k0, (int32_t)kend, ra[u]);
            else load_kslow<BM, VEC_A>(g.a[seg].p, g.a[seg].ld, k0, kend, m0, g.m, ra[u]);
            if (B_KFAST) load_kfast<BN, VEC_B>(g.b[seg].p, g.b[seg].ld, n0, g.n, (int32_t)k0, (int32_t)kend, rb[u]);
            else load_kslow<BN, VEC_B>(g.b[seg].p, g.b[seg].ld, k0, kend, n0, g.n, rb[u]);
        }
    };
    auto store_tile = [&](int buf, int64_t t, const float4 (&ra_in)[SUB][BM / 64],
                          const float4 (&rb_in)[SUB][BN / 64]) {
        const int seg = t < tiles0 ? 0 : 1;
        const int64_t ks = seg == 0 ? kbeg + t * SK : (t - tiles0) * SK;
        const int64_t kend = seg == 0 ? kend0 : (int64_t)g.kseg[1];
#pragma unroll
        for (int u = 0; u < SUB; ++u) {
            const bool live = ks + u * BK < kend;
            const int64_t k0 = live ? ks + u * BK : ks;
            const int64_t ke = live ? kend : ks;        // an empty range zeroes the whole tile
            float4 ra[BM / 64], rb[BN / 64];
#pragma unroll
            for (int i = 0; i < BM / 64; ++i) ra[i] = ra_in[u][i];
#pragma unroll
            for (int i = 0; i < BN / 64; ++i) rb[i] = rb_in[u][i];
            if (A_KFAST) { mask_kfast<BM>(m0, g.m, k0, ke, ra); store_kfast<BM>(As[buf] + u * A_TILE, ra); }
            else { mask_kslow<BM>(k0, ke, m0, g.m, ra); store_kslow<BM>(As[buf] + u * A_TILE, ra); }
            if (B_KFAST) { mask_kfast<BN>(n0, g.n, k0, ke, rb); store_kfast<BN>(Bs[buf] + u * B_TILE, rb); }
            else { mask_kslow<BN>(k0, ke, n0, g.n, rb); store_kslow<BN>(Bs[buf] + u * B_TILE, rb); }
        }
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
            // slot dd held stage t, already in LDS; past the end the last stage is fetched again
            // (never used) so that the load stream has no branches
            load_tile(t + PF < ntiles ? t + PF : ntiles - 1, ra[dd], rb[dd]);
            // keep the loads where they are: left alone, the scheduler sinks them below the
            // MFMA block, right in front of the wait that precedes the LDS store
            __builtin_amdgcn_sched_barrier(0);
            const int half = lane >> 5, xl = lane & 31;
#pragma unroll
            for (int u = 0; u < SUB; ++u) {
                float af[TM][8], bf[TN][8];
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    load_fragment<BM, A_KFAST>(As[buf] + u * A_TILE, wm0 + 32 * i + xl, half, af[i]);
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    load_fragment<BN, B_KFAST>(Bs[buf] + u * B_TILE, wn0 + 32 * j + xl, half, bf[j]);
#pragma unroll
                for (int st = 0; st < 8; ++st)
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i][st], bf[j][st], acc[i][j], 0, 0, 0);
            }
            if (t + 1 < ntiles) store_tile(buf ^ 1, t + 1, ra[(dd + 1) % PF], rb[(dd + 1) % PF]);
            __syncthreads();
        }
    }

    // epilogue: lane holds C[8 (r/4) + 4 (lane/32) + r%4][lane%32] of each 32x32 tile
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int32_t col = n0 + wn0 + 32 * j + (lane & 31);
            if (col >= g.n) continue;
            const float bv = g.bias ? g.bias[col] : 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = m0 + wm0 + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (row >= g.m) continue;
                float v = acc[i][j][r] + bv;
                if (g.relu) v = v > 0.f ? v : 0.f;
                float* dst = cbase + row * g.ldc + col;
                if (g.accumulate) v += *dst;
                *dst = v;
            }
        }
}

// c[i] += sum_s partial[s * stride + i].  A block covers 64 groups of four consecutive
// elements; its four wavefronts each add a quarter of the splits (ascending, eight loads in
// flight) and the four sums are combined through LDS in wavefront order, so the result does
// not depend on timing.  (One thread per group over all splits left most of the chip idle: a
// 256 x 256 gradient is only 64 such blocks of 256 threads.)
__global__ __launch_bounds__(256) void k_reduce_partials(const float* __restrict__ partial,
                                                         int32_t splits, int64_t stride,
                                                         float* __restrict__ c, int64_t ldc,
                                                         int32_t m, int32_t n)
{
    constexpr int U = 8;
    __shared__ float4 sm[4][64];
    const int64_t total = (int64_t)m * n;
    const int grp = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int64_t i = ((int64_t)blockIdx.x * 64 + grp) * 4;
    const int32_t per = (splits + 3) / 4;
    const int32_t zb = q * per, ze = zb + per < splits ? zb + per : splits;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    if (i < total) {
        const bool full = (i + 3 < total) && (stride % 4 == 0);
        if (full) {
            for (int32_t z0 = zb; z0 < ze; z0 += U) {
                float4 x[U];
#pragma unroll
                for (int u = 0; u < U; ++u)
                    x[u] = z0 + u < ze
                               ? *reinterpret_cast<const float4*>(partial + (int64_t)(z0 + u) * stride + i)
                               : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int u = 0; u < U; ++u) { acc[0] += x[u].x; acc[1] += x[u].y; acc[2] += x[u].z; acc[3] += x[u].w; }
            }
        } else {
            for (int32_t z = zb; z < ze; ++z)
                for (int e = 0; e < 4; ++e)
                    if (i + e < total) acc[e] += partial[(int64_t)z * stride + i + e];
        }
    }
    sm[q][grp] = make_float4(acc[0], acc[1], acc[2], acc[3]);
    __syncthreads();
    if (q != 0 || i >= total) return;
    float4 t = sm[0][grp];
    for (int w = 1; w < 4; ++w) { t.x += sm[w][grp].x; t.y += sm[w][grp].y; t.z += sm[w][grp].z; t.w += sm[w][grp].w; }
    const float out[4] = {t.x, t.y, t.z, t.w};
    for (int e = 0; e < 4; ++e) {
        const int64_t j2 = i + e;
        if (j2 >= total) break;
        const int64_t r = j2 / n, cc = j2 - r * n;
        c[r * ldc + cc] += out[e];
    }
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

template <bool A_KFAST, bool B_KFAST>
void launch_gemm(const GemmArgs& g, int splits, hipStream_t s)
{
    if (g.m <= 0 || g.n <= 0) return;
    // float4 loads need 16-byte aligned rows, and the contiguous index of the operand (k for a
    // k-fast operand, m or n otherwise) must consist of whole float4s; decided per operand
    bool va = true, vb = true;
    for (int i = 0; i < 2; ++i) {
        if (g.kseg[i] == 0) continue;
        va = va && aligned16(g.a[i].p) && g.a[i].ld % 4 == 0 && (!A_KFAST || g.kseg[i] % 4 == 0);
        vb = vb && aligned16(g.b[i].p) && g.b[i].ld % 4 == 0 && (!B_KFAST || g.kseg[i] % 4 == 0);
    }
    // (an operand whose m or n index is the contiguous one needs no such condition: its rows are
    // ld >= m (or n) floats long with ld a multiple of 4, so the last vector of a row stays inside
    // the row; what it reads past m (or n) only reaches columns of C that are never stored)
    const bool big_m = g.m > 64, big_n = g.n > 64;
    static const bool xcd_map = [] {
        const char* e = getenv("GNNMI_GEMM_XCD_MAP");
        return !(e && e[0] == '0');
    }();
#define GNN_GEMM(BM, BN, VA, VB)                                                                \
    do {                                                                                        \
        const int64_t mt = (g.m + BM - 1) / BM;                                                 \
        const int32_t nt = (g.n + BN - 1) / BN;                                                 \
        GemmArgs ga = g;                                                                        \
        if (splits == 1 && nt > 1 && xcd_map) {                                                 \
            ga.nt_1d = nt;                                                                      \
            hipLaunchKernelGGL((k_gemm<BM, BN, A_KFAST, B_KFAST, VA, VB>),                      \
                               dim3((unsigned)((mt + 7) / 8 * 8 * nt)), dim3(kThreads), 0, s, ga); \
        } else {                                                                                \
            hipLaunchKernelGGL((k_gemm<BM, BN, A_KFAST, B_KFAST, VA, VB>),                      \
                               dim3((unsigned)mt, (unsigned)nt, (unsigned)splits), dim3(kThreads), 0, s, ga); \
        }                                                                                       \
    } while (0)
    // the last 128-wide column tile would be less than half used: 64-wide tiles waste less
    // (172 columns: 192 computed instead of 256, 0.55 -> 0.42 ms on 780 k rows)
    const bool tail64 = splits == 1 && (g.n + 63) / 64 * 64 < (g.n + 127) / 128 * 128;
    // short K: the product is bound by its loads and stores, 64-row tiles keep more workgroups
    // per CU in flight (+5 % at K = 128)
    const bool small_k = splits == 1 && g.kseg[0] + g.kseg[1] <= 128;
#define GNN_GEMM_TILE(VA, VB)                                     \
    do {                                                          \
        if (big_m && big_n && tail64) GNN_GEMM(128, 64, VA, VB);  \
        else if (small_k && big_n) GNN_GEMM(64, 128, VA, VB);     \
        else if (big_m && big_n) GNN_GEMM(128, 128, VA, VB);      \
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

}  // namespace

void launch_gemm_nn(const GemmSeg* segs, int nseg, float* c, int64_t ldc, int64_t m, int32_t n,
                    const GemmEpilogue& ep, hipStream_t s)
{
    GemmArgs g{};
    for (int i = 0; i < 2; ++i) {
        if (i < nseg) {
            g.a[i] = {segs[i].a, segs[i].lda};
            g.b[i] = {segs[i].b, segs[i].ldb};
            g.kseg[i] = segs[i].k;
        } else {
            g.a[i] = g.a[0];
            g.b[i] = g.b[0];
            g.kseg[i] = 0;
        }
    }
    g.c = c; g.ldc = ldc; g.m = m; g.n = n;
    g.bias = ep.bias; g.relu = ep.relu; g.accumulate = ep.accumulate;
    launch_gemm<true, false>(g, 1, s);
}

void launch_gemm_nt(const float* a, int64_t lda, const float* b, int64_t ldb, float* c,
                    int64_t ldc, int64_t m, int32_t n, int32_t k, const GemmEpilogue& ep,
                    hipStream_t s)
{
    GemmArgs g{};
    g.a[0] = g.a[1] = {a, lda};
    g.b[0] = g.b[1] = {b, ldb};
    g.kseg[0] = k; g.kseg[1] = 0;
    g.c = c; g.ldc = ldc; g.m = m; g.n = n;
    g.bias = ep.bias; g.relu = ep.relu; g.accumulate = ep.accumulate;
    launch_gemm<true, true>(g, 1, s);
}

void launch_gemm_nt2(const GemmSeg* segs, int nseg, float* c, int64_t ldc, int64_t m, int32_t n,
                     const GemmEpilogue& ep, hipStream_t s)
{
    GemmArgs g{};
    for (int i = 0; i < 2; ++i) {
        const GemmSeg& sg = segs[i < nseg ? i : 0];
        g.a[i] = {sg.a, sg.lda};
        g.b[i] = {sg.b, sg.ldb};
        g.kseg[i] = i < nseg ? sg.k : 0;
    }
    g.c = c; g.ldc = ldc; g.m = m; g.n = n;
    g.bias = ep.bias; g.relu = ep.relu; g.accumulate = ep.accumulate;
    launch_gemm<true, true>(g, 1, s);
}

int gemm_tn_splits(int64_t kdim, int32_t m, int32_t n)
{
    const int64_t tiles = (int64_t)((m + 127) / 128) * ((n + 127) / 128);
    int64_t want = (512 + tiles - 1) / tiles;           // ~2 workgroups per CU
    int64_t most = (kdim + 16 * BK - 1) / (16 * BK);    // at least 16 k-steps per split
    int64_t sp = want < most ? want : most;
    return (int)(sp < 1 ? 1 : sp);
}

void launch_gemm_tn(const float* a, int64_t lda, const float* b, int64_t ldb, float* c,
                    int64_t ldc, int32_t m, int32_t n, int64_t kdim, float* partial,
                    hipStream_t s)
{
    if (kdim <= 0 || m <= 0 || n <= 0) return;
    const int splits = gemm_tn_splits(kdim, m, n);
    int64_t chunk = (kdim + splits - 1) / splits;
    chunk = (chunk + BK - 1) / BK * BK;
    GemmArgs g{};
    g.a[0] = g.a[1] = {a, lda};
    g.b[0] = g.b[1] = {b, ldb};
    g.kseg[0] = (int32_t)kdim; g.kseg[1] = 0;
    g.c = partial; g.ldc = n; g.m = m; g.n = n;
    g.split_chunk = chunk;
    g.split_stride = (int64_t)m * n;
    launch_gemm<false, false>(g, splits, s);
    launch_reduce_partials(partial, splits, (int64_t)m * n, c, ldc, m, n, s);
}

void launch_reduce_partials(const float* partial, int splits, int64_t stride, float* c, int64_t ldc,
                            int32_t m, int32_t n, hipStream_t s)
{
    int64_t blocks = ((int64_t)m * n + 255) / 256;
    hipLaunchKernelGGL(k_reduce_partials, dim3((unsigned)blocks), dim3(256), 0, s, partial, splits,
                       stride, c, ldc, m, n);
}

}  // namespace gnnmi
