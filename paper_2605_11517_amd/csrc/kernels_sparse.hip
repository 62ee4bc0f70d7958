// HBM-bound kernels of the path: boundary gather, CSR aggregation (forward, recompute and
// transposed), scatter-add.  gfx950, wave64.
//
//   gather      staging[i,:] = A^{l-1}[B_p[i],:]                       (Gather / regather step)
//   spmm        Z_p[v,:] = scale_v * sum_{e in row v} w_e * src(col_e)  (aggregation along T_p)
//   scatter-add grad A^{l-1}[owner(i),:] += grad GA_p[i,:]              (scatter-accumulate step)
#include <cstdlib>

#include "gnn_internal.h"

namespace gnnmi {
namespace {

constexpr int kBlock = 256;
constexpr int kWave = 64;

// ---------------------------------------------------------------------------------------------
// row copies through an index list.  A row is `vpr` vectors of type V.  G lanes share a row and
// walk it in steps of G vectors; each group keeps UNROLL rows in flight.
// ---------------------------------------------------------------------------------------------
template <typename V, int G, bool SCATTER>
__global__ __launch_bounds__(kBlock) void k_move_rows(const V* __restrict__ src,
                                                      const int32_t* __restrict__ idx,
                                                      V* __restrict__ dst, int64_t rows,
                                                      int32_t vpr)
{
    constexpr int UNROLL = 4;
    const int lane = threadIdx.x % G;
    const int64_t group = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / G;
    const int64_t ngroups = (int64_t)gridDim.x * kBlock / G;
    for (int64_t r0 = group * UNROLL; r0 < rows; r0 += ngroups * UNROLL) {
        int64_t from[UNROLL], to[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            int64_t r = r0 + u;
            int64_t m = r < rows ? (int64_t)idx[r] : 0;
            from[u] = SCATTER ? r : m;
            to[u] = SCATTER ? m : r;
        }
        for (int j = lane; j < vpr; j += G) {
            V val[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
                if (r0 + u < rows) val[u] = src[from[u] * vpr + j];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
                if (r0 + u < rows) dst[to[u] * vpr + j] = val[u];
        }
    }
}

template <typename V, bool SCATTER>
void move_rows_typed(const void* src, const int32_t* idx, void* dst, int64_t rows, int32_t vpr,
                     hipStream_t s)
{
    if (rows <= 0 || vpr <= 0) return;
    auto launch = [&](auto gtag) {
        constexpr int G = decltype(gtag)::value;
        int64_t groups_needed = (rows + 3) / 4;
        int64_t blocks = (groups_needed * G + kBlock - 1) / kBlock;
        blocks = blocks < 1 ? 1 : (blocks > 65536 ? 65536 : blocks);
        hipLaunchKernelGGL((k_move_rows<V, G, SCATTER>), dim3((unsigned)blocks), dim3(kBlock), 0, s,
                           (const V*)src, idx, (V*)dst, rows, vpr);
    };
    if (vpr <= 8) launch(std::integral_constant<int, 8>{});
    else if (vpr <= 16) launch(std::integral_constant<int, 16>{});
    else if (vpr <= 32) launch(std::integral_constant<int, 32>{});
    else launch(std::integral_constant<int, 64>{});
}

template <bool SCATTER>
void move_rows(const void* src, const int32_t* idx, void* dst, int64_t rows, int64_t row_bytes,
               hipStream_t s)
{
    // the widest vector that divides the row and that both base addresses are aligned to
    const uint64_t al = (uint64_t)row_bytes | (uint64_t)reinterpret_cast<uintptr_t>(src) |
                        (uint64_t)reinterpret_cast<uintptr_t>(dst);
    if (al % 16 == 0)
        move_rows_typed<float4, SCATTER>(src, idx, dst, rows, (int32_t)(row_bytes / 16), s);
    else if (al % 4 == 0)
        move_rows_typed<uint32_t, SCATTER>(src, idx, dst, rows, (int32_t)(row_bytes / 4), s);
    else if (al % 2 == 0)
        move_rows_typed<uint16_t, SCATTER>(src, idx, dst, rows, (int32_t)(row_bytes / 2), s);
    else
        move_rows_typed<uint8_t, SCATTER>(src, idx, dst, rows, (int32_t)row_bytes, s);
}

// ---------------------------------------------------------------------------------------------
// CSR aggregation, one wavefront per work item.
//
// Work items come from a host-built plan so that every wavefront sees about the same number of
// entries whatever the degree distribution: an item is either a range of consecutive short
// rows (results written directly) or one segment of a long row (partial sum written to
// `partial`, combined afterwards in segment order, which keeps the result deterministic).
//
// Inside a row the 64 lanes are split into S = 64 / G slots of G lanes.  A slot owns one entry
// at a time and its lanes read that source row as float4 (16 B per lane, a full row of
// d <= 4 G floats per slot in one coalesced request); NV > 1 covers wider rows.  The wave
// loads 64 column indices and weights with one coalesced read each and hands them to the slots
// with cross-lane reads, so the index stream costs 4-8 B per entry and the feature rows
// dominate.  Slot partial sums are combined with xor-shuffles at the end of the row.
// ---------------------------------------------------------------------------------------------
struct SpmmArgs {
    const int64_t* rp;
    const int32_t* col;
    const float* w;
    int64_t wss = 0;        // column-sliced launches: the entry weights of slice s start at w + s wss
    const float* rowscale;
    const void* a_rows;     // element type TIn
    int64_t n_a;
    const void* b_rows;
    void* out;              // element type TOut
    int32_t d, ld;          // d: columns handled by this launch; ld: row stride (elements)
    SpmmItems it;
    float* partial;         // always fp32
    // optional fused scatter-accumulate (fp32 output only): row r is ADDED to output row
    // map_base + r when r < map_n_own, else to row map_idx[r - map_n_own]; map_n_own < 0 = off
    int64_t map_n_own, map_base;
    const int32_t* map_idx;
    const uint32_t* map_first;   // optional bit per row: set = store, do not add
    // applied to what is stored: + bias[column] (pointer already at this launch's first column),
    // then max(., 0)
    const float* bias;
    int32_t relu;
    __device__ int64_t out_row(int32_t r) const
    {
        if (map_n_own < 0) return r;
        return r < map_n_own ? map_base + r : (int64_t)map_idx[r - map_n_own];
    }
    __device__ bool adds(int32_t r) const
    {
        if (map_n_own < 0) return false;
        if (!map_first) return true;
        return ((map_first[r >> 5] >> (r & 31)) & 1u) == 0u;
    }
};

// 16-byte vectors of the storage types: 4 floats or 8 bfloat16 (kept as raw uint16_t).
template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int EPV = 4;
    __device__ static inline void unpack(const uint4& v, float (&f)[4])
    {
        f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
        f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    }
    __device__ static inline uint4 pack(const float (&f)[4])
    {
        return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]),
                          __float_as_uint(f[3]));
    }
    __device__ static inline float load(const float* p) { return *p; }
    __device__ static inline void store(float* p, float v) { *p = v; }
};
__device__ inline float bf16_to_float(uint32_t h) { return __uint_as_float(h << 16); }
__device__ inline uint32_t float_to_bf16(float f)   // round to nearest even
{
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
template <> struct Elem<uint16_t> {
    static constexpr int EPV = 8;
    __device__ static inline void unpack(const uint4& v, float (&f)[8])
    {
        f[0] = bf16_to_float(v.x & 0xFFFFu); f[1] = bf16_to_float(v.x >> 16);
        f[2] = bf16_to_float(v.y & 0xFFFFu); f[3] = bf16_to_float(v.y >> 16);
        f[4] = bf16_to_float(v.z & 0xFFFFu); f[5] = bf16_to_float(v.z >> 16);
        f[6] = bf16_to_float(v.w & 0xFFFFu); f[7] = bf16_to_float(v.w >> 16);
    }
    __device__ static inline uint4 pack(const float (&f)[8])
    {
        return make_uint4(float_to_bf16(f[0]) | (float_to_bf16(f[1]) << 16),
                          float_to_bf16(f[2]) | (float_to_bf16(f[3]) << 16),
                          float_to_bf16(f[4]) | (float_to_bf16(f[5]) << 16),
                          float_to_bf16(f[6]) | (float_to_bf16(f[7]) << 16));
    }
    __device__ static inline float load(const uint16_t* p) { return bf16_to_float(*p); }
    __device__ static inline void store(uint16_t* p, float v) { *p = (uint16_t)float_to_bf16(v); }
};

// acc[v][i] += sum over entries [e_begin, e_end) of w_e * src(col_e)[(v*G + lane%G)*EPV + i]
template <typename TIn, int G, int NV, bool VEC>
__device__ inline void spmm_accumulate(const SpmmArgs& g, int64_t e_begin, int64_t e_end, int lane,
                                       float (&acc)[NV][Elem<TIn>::EPV])
{
    constexpr int EPV = Elem<TIn>::EPV;
    constexpr int S = kWave / G;
    constexpr int UNROLL = (NV == 1) ? 8 : 4;   // source rows in flight per slot
    const int slot = lane / G;
    const int gl = lane % G;
    const TIn* a_rows = static_cast<const TIn*>(g.a_rows);
    const TIn* b_rows = static_cast<const TIn*>(g.b_rows);
    // column offsets of this lane's vectors; lanes past the row end read column 0 (their sums
    // are never stored), so that every load below is unconditional and the compiler can keep
    // all of them in flight
    int cv[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int c = (v * G + gl) * EPV;
        cv[v] = c < g.d ? c : 0;
    }
    // index/weight chunk of the first 64 entries; the next chunk is fetched while this one is
    // being consumed
    int32_t my_c = 0;
    float my_w = 0.f;
    if (e_begin + lane < e_end) {
        my_c = g.col[e_begin + lane];
        my_w = g.w ? g.w[e_begin + lane] : 1.f;
    }
    for (int64_t e0 = e_begin; e0 < e_end; e0 += kWave) {
        const int cnt = (int)((e_end - e0) < kWave ? (e_end - e0) : kWave);
        const int32_t cur_c = my_c;
        const float cur_w = my_w;
        if (e0 + kWave + lane < e_end) {
            my_c = g.col[e0 + kWave + lane];
            my_w = g.w ? g.w[e0 + kWave + lane] : 1.f;
        }
        for (int j0 = 0; j0 < cnt; j0 += S * UNROLL) {
            const TIn* src[UNROLL];
            float ww[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int j = j0 + u * S + slot;
                const int jj = j < cnt ? j : cnt - 1;     // stay on a valid entry
                const int32_t c = __shfl(cur_c, jj, kWave);
                const float wt = __shfl(cur_w, jj, kWave);
                ww[u] = j < cnt ? wt : 0.f;
                src[u] = (c < g.n_a) ? a_rows + (int64_t)c * g.ld
                                     : b_rows + ((int64_t)c - g.n_a) * g.ld;
            }
            if (VEC) {
                uint4 x[UNROLL][NV];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u)
#pragma unroll
                    for (int v = 0; v < NV; ++v)
                        x[u][v] = *reinterpret_cast<const uint4*>(src[u] + cv[v]);
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) {
                    const bool on = (j0 + u * S + slot) < cnt;
#pragma unroll
                    for (int v = 0; v < NV; ++v) {
                        float f[EPV];
                        Elem<TIn>::unpack(x[u][v], f);
#pragma unroll
                        for (int i = 0; i < EPV; ++i) acc[v][i] += on ? ww[u] * f[i] : 0.f;
                    }
                }
            } else {
#pragma unroll
                for (int u = 0; u < UNROLL; ++u)
#pragma unroll
                    for (int v = 0; v < NV; ++v)
#pragma unroll
                        for (int i = 0; i < EPV; ++i) {
                            int c = (v * G + gl) * EPV + i;
                            if (c < g.d && ww[u] != 0.f) acc[v][i] += ww[u] * Elem<TIn>::load(src[u] + c);
                        }
            }
        }
    }
    // combine the slots
#pragma unroll
    for (int m = G; m < kWave; m <<= 1)
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int i = 0; i < EPV; ++i) acc[v][i] += __shfl_xor(acc[v][i], m, kWave);
}

// Lanes 0..G-1 write sc * acc as elements of type TOut; each lane owns EPV consecutive
// columns per vector, which is a whole 16-byte store for TOut = TIn and two for fp32 output of
// a bf16 input.
template <typename TOut, int EPV, int G, int NV, bool VEC>
__device__ inline void spmm_store(TOut* o, int32_t d, int lane, float sc, const float (&acc)[NV][EPV],
                                  bool add, const float* bias, bool relu)
{
    if (lane >= G) return;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int c0 = (v * G + lane) * EPV;
        if (VEC) {
            if (c0 >= d) continue;
            constexpr int OPV = Elem<TOut>::EPV;      // elements per 16-byte output vector
#pragma unroll
            for (int h = 0; h < EPV / OPV; ++h) {
                float f[OPV];
#pragma unroll
                for (int i = 0; i < OPV; ++i) f[i] = sc * acc[v][h * OPV + i];
                uint4* dst = reinterpret_cast<uint4*>(o + c0 + h * OPV);
                if (add) {
                    float old[OPV];
                    Elem<TOut>::unpack(*dst, old);
#pragma unroll
                    for (int i = 0; i < OPV; ++i) f[i] += old[i];
                }
                if (bias) {
#pragma unroll
                    for (int i = 0; i < OPV; ++i) f[i] += bias[c0 + h * OPV + i];
                }
                if (relu) {
#pragma unroll
                    for (int i = 0; i < OPV; ++i) f[i] = f[i] > 0.f ? f[i] : 0.f;
                }
                *dst = Elem<TOut>::pack(f);
            }
        } else {
#pragma unroll
            for (int i = 0; i < EPV; ++i)
                if (c0 + i < d) {
                    float v2 = sc * acc[v][i];
                    if (add) v2 += Elem<TOut>::load(o + c0 + i);
                    if (bias) v2 += bias[c0 + i];
                    if (relu) v2 = v2 > 0.f ? v2 : 0.f;
                    Elem<TOut>::store(o + c0 + i, v2);
                }
        }
    }
}

template <typename TIn, typename TOut, int G, int NV, bool VEC>
__global__ __launch_bounds__(kBlock) void k_spmm_items(const SpmmArgs g)
{
    constexpr int EPV = Elem<TIn>::EPV;
    const int lane = threadIdx.x % kWave;
    // the item index is the same for the whole wavefront; tell the compiler so that row
    // pointers and item descriptors travel through scalar registers
    const int64_t item = __builtin_amdgcn_readfirstlane(
        (int)(blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave));
    float acc[NV][EPV];
    if (item < g.it.nsegs) {
        // one segment of a long row -> fp32 partial sum
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int i = 0; i < EPV; ++i) acc[v][i] = 0.f;
        const int64_t e0 = g.it.seg_begin[item];
        spmm_accumulate<TIn, G, NV, VEC>(g, e0, e0 + g.it.seg_len[item], lane, acc);
        spmm_store<float, EPV, G, NV, VEC>(g.partial + item * (int64_t)g.ld, g.d, lane, 1.f, acc, false, nullptr,
                                           false);
        return;
    }
    const int64_t ri = item - g.it.nsegs;
    if (ri >= g.it.nranges) return;
    const int32_t r_end = g.it.range_rows[ri + 1];
    for (int32_t row = g.it.range_rows[ri]; row < r_end; ++row) {
        const int64_t e_begin = g.rp[row], e_end = g.rp[row + 1];
        if (e_end - e_begin > kSpmmSegment) continue;  // long row: handled by its segments
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int i = 0; i < EPV; ++i) acc[v][i] = 0.f;
        spmm_accumulate<TIn, G, NV, VEC>(g, e_begin, e_end, lane, acc);
        spmm_store<TOut, EPV, G, NV, VEC>(static_cast<TOut*>(g.out) + g.out_row(row) * (int64_t)g.ld, g.d,
                                          lane, g.rowscale ? g.rowscale[row] : 1.f, acc, g.adds(row),
                                          g.bias, g.relu != 0);
    }
}

// ---------------------------------------------------------------------------------------------
// Column-sliced variant for rows of at least two 128-byte lines.
//
// The row is cut into NS slices of G 16-byte vectors (a multiple of 128 bytes each) and
// workgroup b handles slice b % NS.  Consecutive workgroups are dispatched to consecutive XCDs,
// each with its own L2, so every XCD only ever sees one slice of every source row: the eight L2s
// hold disjoint data instead of eight copies of the same hot rows, which multiplies the number
// of source rows that stay cached by NS.
//
// To keep the per-row cost from growing by the same factor, a wavefront here works on 64 / G
// items at once, one per slot of G lanes.  An item is a long-row segment or a whole short row;
// the host lists the short rows longest first, so the slots of a wavefront run about the same
// number of steps.  Each slot streams its own index/weight chunk (G entries) and walks it with
// up to eight source-slice loads in flight.
// ---------------------------------------------------------------------------------------------
template <typename TIn, typename TOut, int G>
__global__ __launch_bounds__(kBlock) void k_spmm_slots(const SpmmArgs g, int32_t nslices)
{
    constexpr int EPV = Elem<TIn>::EPV;
    constexpr int S = kWave / G;
    constexpr int UNROLL = G < 8 ? G : 8;
    const int lane = threadIdx.x % kWave;
    const int slot = lane / G, gl = lane % G;
    unsigned blk = blockIdx.x;
    // this lane's columns; lanes past the row end (rows narrower than G vectors) read column 0
    // and store nothing
    const int coff_raw = (int)(blk % (unsigned)nslices) * (G * EPV) + gl * EPV;
    const bool live = coff_raw < g.d;
    const int coff = live ? coff_raw : 0;
    const float* wsl = g.w ? g.w + (int64_t)(blk % (unsigned)nslices) * g.wss : nullptr;   // this slice's weights
    blk /= (unsigned)nslices;
    const int64_t item = ((int64_t)blk * (kBlock / kWave) + threadIdx.x / kWave) * S + slot;

    const TIn* a_rows = static_cast<const TIn*>(g.a_rows);
    const TIn* b_rows = static_cast<const TIn*>(g.b_rows);
    int64_t e_begin = 0;
    int32_t len = 0;
    int32_t row = -1;
    bool first_row = false;
    if (item < g.it.nsegs) {
        e_begin = g.it.seg_begin[item];
        len = g.it.seg_len[item];
    } else if (item < g.it.nsegs + g.it.nshort) {
        // (the top bit of an entry of the transposed plan's list marks a row that is first to
        // reach its output row; it counts only where map_first is given)
        const int32_t listed = g.it.rows_sorted[item - g.it.nsegs];
        row = listed & 0x7FFFFFFF;
        first_row = listed < 0;
        e_begin = g.rp[row];
        len = (int32_t)(g.rp[row + 1] - e_begin);
    }
    // the longest slot of the wavefront sets the trip count and lends its entries to finished
    // slots, so that every load below reads a real source row
    int32_t maxlen = len;
    int lead = slot;
#pragma unroll
    for (int m = G; m < kWave; m <<= 1) {
        const int32_t ol = __shfl_xor(maxlen, m, kWave);
        const int os = __shfl_xor(lead, m, kWave);
        if (ol > maxlen || (ol == maxlen && os < lead)) { maxlen = ol; lead = os; }
    }
    float acc[EPV];
#pragma unroll
    for (int i = 0; i < EPV; ++i) acc[i] = 0.f;

    for (int32_t e0 = 0; e0 < maxlen; e0 += G) {
        int32_t my_c = 0;
        float my_w = 0.f;
        if (e0 + gl < len) {
            my_c = g.col[e_begin + e0 + gl];
            my_w = wsl ? wsl[e_begin + e0 + gl] : 1.f;
        }
        const int cnt = len - e0;                     // entries this slot still has (may be <= 0)
        const int lead_cnt = maxlen - e0 < G ? maxlen - e0 : G;
#pragma unroll
        for (int j0 = 0; j0 < G; j0 += UNROLL) {
            if (j0 >= lead_cnt) break;               // uniform across the wavefront
            uint4 x[UNROLL];
            float ww[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int j = j0 + u;
                const bool on = j < cnt;
                const int src_lane = on ? slot * G + j : lead * G + (j < lead_cnt ? j : lead_cnt - 1);
                const int32_t c = __shfl(my_c, src_lane, kWave);
                const float wt = __shfl(my_w, src_lane, kWave);
                ww[u] = on ? wt : 0.f;
                const TIn* src = (c < g.n_a) ? a_rows + (int64_t)c * g.ld : b_rows + ((int64_t)c - g.n_a) * g.ld;
                x[u] = *reinterpret_cast<const uint4*>(src + coff);
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                float f[EPV];
                Elem<TIn>::unpack(x[u], f);
                const bool on = (j0 + u) < cnt;
#pragma unroll
                for (int i = 0; i < EPV; ++i) acc[i] += on ? ww[u] * f[i] : 0.f;
            }
        }
    }
    if (!live) return;
    if (item < g.it.nsegs) {
        float* o = g.partial + item * (int64_t)g.ld + coff;
#pragma unroll
        for (int h = 0; h < EPV / 4; ++h)
            *reinterpret_cast<float4*>(o + 4 * h) =
                make_float4(acc[4 * h], acc[4 * h + 1], acc[4 * h + 2], acc[4 * h + 3]);
    } else if (row >= 0) {
        const float sc = g.rowscale ? g.rowscale[row] : 1.f;
        TOut* o = static_cast<TOut*>(g.out) + g.out_row(row) * (int64_t)g.ld + coff;
        constexpr int OPV = Elem<TOut>::EPV;
        const bool add = g.map_n_own >= 0 && !(g.map_first && first_row);   // fused scatter-accumulate (fp32 output): one slot per row
#pragma unroll
        for (int h = 0; h < EPV / OPV; ++h) {
            float f[OPV];
#pragma unroll
            for (int i = 0; i < OPV; ++i) f[i] = sc * acc[h * OPV + i];
            if (add) {
                float old[OPV];
                Elem<TOut>::unpack(*reinterpret_cast<const uint4*>(o + h * OPV), old);
#pragma unroll
                for (int i = 0; i < OPV; ++i) f[i] += old[i];
            }
            if (g.bias) {
#pragma unroll
                for (int i = 0; i < OPV; ++i) f[i] += g.bias[coff + h * OPV + i];
            }
            if (g.relu) {
#pragma unroll
                for (int i = 0; i < OPV; ++i) f[i] = f[i] > 0.f ? f[i] : 0.f;
            }
            *reinterpret_cast<uint4*>(o + h * OPV) = Elem<TOut>::pack(f);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Variant of k_spmm_slots for operators whose rows hold a handful of entries and whose sources
// are one array of fewer than 2^32 elements (the transposed operator of a sparse directed graph;
// no column slices).  UNR loads in flight per slot instead of eight, 32-bit source offsets, a
// rolled batch loop: 51 registers instead of 95, eight wavefronts per SIMD instead of five - such
// rows are bound by how many of them are in flight, not by bytes.  NV = 2: rows of up to 2 G
// vectors, two vectors per lane.
// ---------------------------------------------------------------------------------------------
template <typename TIn, typename TOut, int G, int UNR, int NV, bool ONE_SRC = true>
__global__ __launch_bounds__(kBlock) void k_spmm_short(const SpmmArgs g, int32_t nslices)
{
    constexpr int EPV = Elem<TIn>::EPV;
    constexpr int S = kWave / G;
    // source rows in flight per slot.  Eight for rows of tens of entries; four for operators whose
    // rows hold three or four entries (the transposed operator of a sparse directed graph): the
    // loads beyond a row's end only repeat its last entry, and the registers they occupy cost
    // occupancy (95 -> 51 registers, 5 -> 8 wavefronts per SIMD), which is what keeps rows in flight
    constexpr int UNROLL = G < UNR ? G : UNR;
    const int lane = threadIdx.x % kWave;
    const int slot = lane / G, gl = lane % G;
    unsigned blk = blockIdx.x;
    // this lane's columns: NV vectors, G vectors apart (NV = 2: rows of up to 2 G vectors without
    // column slices); lanes past the row end read column 0 and store nothing
    int coff[NV];
    bool live[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int raw = (int)(blk % (unsigned)nslices) * (G * EPV) + (v * G + gl) * EPV;
        live[v] = raw < g.d;
        coff[v] = live[v] ? raw : 0;
    }
    const float* wsl = g.w ? g.w + (int64_t)(blk % (unsigned)nslices) * g.wss : nullptr;   // this slice's weights
    blk /= (unsigned)nslices;
    const int64_t item = ((int64_t)blk * (kBlock / kWave) + threadIdx.x / kWave) * S + slot;

    const TIn* a_rows = static_cast<const TIn*>(g.a_rows);
    const TIn* b_rows = static_cast<const TIn*>(g.b_rows);
    int64_t e_begin = 0;
    int32_t len = 0;
    int32_t row = -1;
    bool first_row = false;
    if (item < g.it.nsegs) {
        e_begin = g.it.seg_begin[item];
        len = g.it.seg_len[item];
    } else if (item < g.it.nsegs + g.it.nshort) {
        // (the top bit of an entry of the transposed plan's list marks a row that is first to
        // reach its output row; it counts only where map_first is given)
        const int32_t listed = g.it.rows_sorted[item - g.it.nsegs];
        row = listed & 0x7FFFFFFF;
        first_row = listed < 0;
        e_begin = g.rp[row];
        len = (int32_t)(g.rp[row + 1] - e_begin);
    }
    // the longest slot of the wavefront sets the trip count and lends its entries to finished
    // slots, so that every load below reads a real source row
    int32_t maxlen = len;
    int lead = slot;
#pragma unroll
    for (int m = G; m < kWave; m <<= 1) {
        const int32_t ol = __shfl_xor(maxlen, m, kWave);
        const int os = __shfl_xor(lead, m, kWave);
        if (ol > maxlen || (ol == maxlen && os < lead)) { maxlen = ol; lead = os; }
    }
    float acc[NV][EPV];
#pragma unroll
    for (int v = 0; v < NV; ++v)
#pragma unroll
        for (int i = 0; i < EPV; ++i) acc[v][i] = 0.f;

    for (int32_t e0 = 0; e0 < maxlen; e0 += G) {
        int32_t my_c = 0;
        float my_w = 0.f;
        if (e0 + gl < len) {
            my_c = g.col[e_begin + e0 + gl];
            my_w = wsl ? wsl[e_begin + e0 + gl] : 1.f;
        }
        const int cnt = len - e0;                     // entries this slot still has (may be <= 0)
        const int lead_cnt = maxlen - e0 < G ? maxlen - e0 : G;
        // one batch of UNROLL entries: loads first, then the multiply-adds
        auto batch = [&](int j0) {
            uint4 x[UNROLL][NV];
            float ww[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int j = j0 + u;
                const bool on = j < cnt;
                const int src_lane = on ? slot * G + j : lead * G + (j < lead_cnt ? j : lead_cnt - 1);
                const int32_t c = __shfl(my_c, src_lane, kWave);
                const float wt = __shfl(my_w, src_lane, kWave);
                ww[u] = on ? wt : 0.f;
                if (ONE_SRC) {
                    // one source array (the transposed operator reads the partition's own rows
                    // only) of fewer than 2^32 elements: 32-bit offsets from a uniform base
                    // instead of a 64-bit address per load in flight
                    const uint32_t off = (uint32_t)c * (uint32_t)g.ld;
#pragma unroll
                    for (int v = 0; v < NV; ++v)
                        x[u][v] = *reinterpret_cast<const uint4*>(a_rows + (off + (uint32_t)coff[v]));
                } else {
                    const TIn* src = (c < g.n_a) ? a_rows + (int64_t)c * g.ld : b_rows + ((int64_t)c - g.n_a) * g.ld;
#pragma unroll
                    for (int v = 0; v < NV; ++v) x[u][v] = *reinterpret_cast<const uint4*>(src + coff[v]);
                }
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const bool on = (j0 + u) < cnt;
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    float f[EPV];
                    Elem<TIn>::unpack(x[u][v], f);
#pragma unroll
                    for (int i = 0; i < EPV; ++i) acc[v][i] += on ? ww[u] * f[i] : 0.f;
                }
            }
        };
        if (UNR < 8) {
            // short rows: a rolled loop keeps the register count (and with it the occupancy) low
#pragma unroll 1
            for (int j0 = 0; j0 < G; j0 += UNROLL) {
                if (j0 >= lead_cnt) break;           // uniform across the wavefront
                batch(j0);
            }
        } else {
#pragma unroll
            for (int j0 = 0; j0 < G; j0 += UNROLL) {
                if (j0 >= lead_cnt) break;           // uniform across the wavefront
                batch(j0);
            }
        }
    }
    if (item < g.it.nsegs) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            if (!live[v]) continue;
            float* o = g.partial + item * (int64_t)g.ld + coff[v];
#pragma unroll
            for (int h = 0; h < EPV / 4; ++h)
                *reinterpret_cast<float4*>(o + 4 * h) =
                    make_float4(acc[v][4 * h], acc[v][4 * h + 1], acc[v][4 * h + 2], acc[v][4 * h + 3]);
        }
    } else if (row >= 0) {
        const float sc = g.rowscale ? g.rowscale[row] : 1.f;
        TOut* orow = static_cast<TOut*>(g.out) + g.out_row(row) * (int64_t)g.ld;
        constexpr int OPV = Elem<TOut>::EPV;
        const bool add = g.map_n_own >= 0 && !(g.map_first && first_row);   // fused scatter-accumulate (fp32 output): one slot per row
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            if (!live[v]) continue;
            TOut* o = orow + coff[v];
#pragma unroll
            for (int h = 0; h < EPV / OPV; ++h) {
                float f[OPV];
#pragma unroll
                for (int i = 0; i < OPV; ++i) f[i] = sc * acc[v][h * OPV + i];
                if (add) {
                    float old[OPV];
                    Elem<TOut>::unpack(*reinterpret_cast<const uint4*>(o + h * OPV), old);
#pragma unroll
                    for (int i = 0; i < OPV; ++i) f[i] += old[i];
                }
                if (g.bias) {
#pragma unroll
                    for (int i = 0; i < OPV; ++i) f[i] += g.bias[coff[v] + h * OPV + i];
                }
                if (g.relu) {
#pragma unroll
                    for (int i = 0; i < OPV; ++i) f[i] = f[i] > 0.f ? f[i] : 0.f;
                }
                *reinterpret_cast<uint4*>(o + h * OPV) = Elem<TOut>::pack(f);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Aggregation fused with the transform (aggregate-first layers, fp32, d_in <= 128, d_out <= 256).
//
// A workgroup owns 64 destination rows.  Phase 1: its four wavefronts aggregate those rows as
// the slot kernel above does (G lanes per row, rows taken from the degree-sorted list so that
// the slots of a wavefront finish together) and leave the sums Z in LDS instead of in memory;
// rows that were cut into segments arrive through `zlong` (their sums were combined by the
// long-row kernel) and are copied.  For GraphSAGE the rows' own input rows are staged beside
// them.  Phase 2: Y = act(Z W (+ X W_s) + b) on the fp32 matrix cores straight from that tile
// (v_mfma_f32_32x32x2f32: A fragments from LDS, B fragments - rows of W, shared by every
// workgroup and resident in L2 - from memory), stored to the rows' places in the output.
// Z is neither written nor read back, and the contraction runs in the shadow of the other
// workgroups' row fetches.
// ---------------------------------------------------------------------------------------------
typedef float floatx16 __attribute__((ext_vector_type(16)));

struct FusedArgs {
    SpmmArgs sp;            // operator rows and sources; sp.out is unused
    const float* zlong;     // [n_p, d_in]: valid in the rows listed in sp.it.long_row
    const float* xself;     // own input rows [n_p, d_in] (GraphSAGE), else null
    const float* w;         // [d_in, d_out]
    const float* ws;        // [d_in, d_out] or null
    const float* bias;      // [d_out] or null
    float* y;               // [n_p, d_out]
    int32_t dout, relu;
    int32_t kp;             // LDS row stride in floats (odd)
    int32_t seg_blocks;     // the first seg_blocks workgroups compute segment partial sums instead
    int32_t long_only;      // 1: the tiles cover the long rows only (second launch), 0: the short rows only
};

template <int G>
__global__ __launch_bounds__(kBlock) void k_agg_gemm(const FusedArgs g)
{
    constexpr int TM = 64;                      // rows per workgroup
    constexpr int S = kWave / G;                // row slots per wavefront
    constexpr int RPW = TM / (kBlock / kWave);  // rows per wavefront: 16
    constexpr int UNROLL = 8;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    float* Zs = lds;                            // [TM][kp]
    float* Xs = lds + TM * g.kp;                // [TM][kp], GraphSAGE only
    const SpmmArgs& sp = g.sp;
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int slot = lane / G, gl = lane % G;
    const int32_t din = sp.d;
    // list of rows this launch tiles: the short rows (degree-sorted), or the long rows
    const int64_t nrows = g.long_only ? sp.it.nlong : sp.it.nshort;
    const float* a_rows = static_cast<const float*>(sp.a_rows);
    const float* b_rows = static_cast<const float*>(sp.b_rows);
    const int coff = gl * 4;
    const bool live = coff < din;
    const int cload = live ? coff : 0;

    if ((int32_t)blockIdx.x < g.seg_blocks) {
        // segment role: one 512-entry segment of a long row per slot -> fp32 partial sum; the
        // long-row kernel combines them afterwards and a second launch transforms those rows
        const int64_t item = ((int64_t)blockIdx.x * (kBlock / kWave) + wave) * S + slot;
        int64_t e_begin = 0;
        int32_t len = 0;
        if (item < sp.it.nsegs) {
            e_begin = sp.it.seg_begin[item];
            len = sp.it.seg_len[item];
        }
        int32_t maxlen = len;
        int lead = slot;
#pragma unroll
        for (int m = G; m < kWave; m <<= 1) {
            const int32_t ol = __shfl_xor(maxlen, m, kWave);
            const int os = __shfl_xor(lead, m, kWave);
            if (ol > maxlen || (ol == maxlen && os < lead)) { maxlen = ol; lead = os; }
        }
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        for (int32_t e0 = 0; e0 < maxlen; e0 += G) {
            int32_t my_c = 0;
            float my_w = 0.f;
            if (e0 + gl < len) {
                my_c = sp.col[e_begin + e0 + gl];
                my_w = sp.w ? sp.w[e_begin + e0 + gl] : 1.f;
            }
            const int cnt = len - e0;
            const int lead_cnt = maxlen - e0 < G ? maxlen - e0 : G;
#pragma unroll
            for (int j0 = 0; j0 < G; j0 += UNROLL) {
                if (j0 >= lead_cnt) break;
                float4 x[UNROLL];
                float ww[UNROLL];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) {
                    const int j = j0 + u;
                    const bool on = j < cnt;
                    const int src_lane = on ? slot * G + j : lead * G + (j < lead_cnt ? j : lead_cnt - 1);
                    const int32_t c = __shfl(my_c, src_lane, kWave);
                    const float wt = __shfl(my_w, src_lane, kWave);
                    ww[u] = on ? wt : 0.f;
                    const float* src = (c < sp.n_a) ? a_rows + (int64_t)c * sp.ld : b_rows + ((int64_t)c - sp.n_a) * sp.ld;
                    x[u] = *reinterpret_cast<const float4*>(src + cload);
                }
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) {
                    const bool on = (j0 + u) < cnt;
                    acc[0] += on ? ww[u] * x[u].x : 0.f;
                    acc[1] += on ? ww[u] * x[u].y : 0.f;
                    acc[2] += on ? ww[u] * x[u].z : 0.f;
                    acc[3] += on ? ww[u] * x[u].w : 0.f;
                }
            }
        }
        if (live && item < sp.it.nsegs)
            *reinterpret_cast<float4*>(sp.partial + item * (int64_t)sp.ld + coff) = make_float4(acc[0], acc[1], acc[2], acc[3]);
        return;
    }
    const int64_t tile0 = ((int64_t)blockIdx.x - g.seg_blocks) * TM;

    // ---- phase 1: sums of this wavefront's 16 rows, S at a time
    for (int r0 = 0; r0 < RPW; r0 += S) {
        const int tr = wave * RPW + r0 + slot;          // row of the tile
        const int64_t li = tile0 + tr;                  // position in the sorted list
        int32_t row = -1;
        int64_t e_begin = 0;
        int32_t len = 0;
        bool is_long = false;
        if (li < nrows) {
            if (g.long_only) {
                row = sp.it.long_row[li];
                is_long = true;
            } else {
                row = sp.it.rows_sorted[li] & 0x7FFFFFFF;
                e_begin = sp.rp[row];
                len = (int32_t)(sp.rp[row + 1] - e_begin);
            }
        }
        int32_t maxlen = len;
        int lead = slot;
#pragma unroll
        for (int m = G; m < kWave; m <<= 1) {
            const int32_t ol = __shfl_xor(maxlen, m, kWave);
            const int os = __shfl_xor(lead, m, kWave);
            if (ol > maxlen || (ol == maxlen && os < lead)) { maxlen = ol; lead = os; }
        }
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        for (int32_t e0 = 0; e0 < maxlen; e0 += G) {
            int32_t my_c = 0;
            float my_w = 0.f;
            if (e0 + gl < len) {
                my_c = sp.col[e_begin + e0 + gl];
                my_w = sp.w ? sp.w[e_begin + e0 + gl] : 1.f;
            }
            const int cnt = len - e0;
            const int lead_cnt = maxlen - e0 < G ? maxlen - e0 : G;
#pragma unroll
            for (int j0 = 0; j0 < G; j0 += UNROLL) {
                if (j0 >= lead_cnt) break;
                float4 x[UNROLL];
                float ww[UNROLL];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) {
                    const int j = j0 + u;
                    const bool on = j < cnt;
                    const int src_lane = on ? slot * G + j : lead * G + (j < lead_cnt ? j : lead_cnt - 1);
                    const int32_t c = __shfl(my_c, src_lane, kWave);
                    const float wt = __shfl(my_w, src_lane, kWave);
                    ww[u] = on ? wt : 0.f;
                    const float* src = (c < sp.n_a) ? a_rows + (int64_t)c * sp.ld : b_rows + ((int64_t)c - sp.n_a) * sp.ld;
                    x[u] = *reinterpret_cast<const float4*>(src + cload);
                }
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) {
                    const bool on = (j0 + u) < cnt;
                    acc[0] += on ? ww[u] * x[u].x : 0.f;
                    acc[1] += on ? ww[u] * x[u].y : 0.f;
                    acc[2] += on ? ww[u] * x[u].z : 0.f;
                    acc[3] += on ? ww[u] * x[u].w : 0.f;
                }
            }
        }
        if (live) {
            float z[4] = {0.f, 0.f, 0.f, 0.f};
            if (is_long) {
                const float4 v = *reinterpret_cast<const float4*>(g.zlong + (int64_t)row * din + coff);
                z[0] = v.x; z[1] = v.y; z[2] = v.z; z[3] = v.w;
            } else if (row >= 0) {
                const float sc = sp.rowscale ? sp.rowscale[row] : 1.f;
#pragma unroll
                for (int i = 0; i < 4; ++i) z[i] = sc * acc[i];
            }
            float* zr = Zs + tr * g.kp + coff;
#pragma unroll
            for (int i = 0; i < 4; ++i) zr[i] = z[i];
            if (g.xself) {
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (row >= 0) v = *reinterpret_cast<const float4*>(g.xself + (int64_t)row * din + coff);
                float* xr = Xs + tr * g.kp + coff;
                xr[0] = v.x; xr[1] = v.y; xr[2] = v.z; xr[3] = v.w;
            }
        }
    }
    // the k loop below runs to an even bound: one more column when d_in is odd (never: d_in % 4 == 0)
    __syncthreads();

    // ---- phase 2: Y tile = Zs W (+ Xs W_s); wavefront w owns the 32-column tiles w, w + 4, ...
    const int half = lane >> 5, xl = lane & 31;
    const int nseg = g.xself ? 2 : 1;
    floatx16 acc2[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc2[i][j][r] = 0.f;
    const int32_t col0 = 32 * wave + xl, col1 = 32 * (wave + 4) + xl;
    const bool c0 = col0 < g.dout, c1 = col1 < g.dout;
    const bool any1 = 32 * (wave + 4) < g.dout;           // uniform over the wavefront
    for (int seg = 0; seg < nseg; ++seg) {
        const float* As = seg == 0 ? Zs : Xs;
        const float* W = seg == 0 ? g.w : g.ws;
        constexpr int KU = 16;                              // k-steps (of 2) per batch of loads
        for (int32_t k0 = 0; k0 < din; k0 += 2 * KU) {
            float b0[KU], b1[KU], a0[KU], a1[KU];
#pragma unroll
            for (int u = 0; u < KU; ++u) {
                const int32_t k = k0 + 2 * u + half;
                const bool kin = k < din;
                const float* wr = W + (int64_t)(kin ? k : 0) * g.dout;
                b0[u] = (kin && c0) ? wr[col0] : 0.f;
                b1[u] = (kin && c1) ? wr[col1] : 0.f;
                a0[u] = kin ? As[xl * g.kp + k] : 0.f;
                a1[u] = kin ? As[(32 + xl) * g.kp + k] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < KU; ++u) {
                acc2[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[u], b0[u], acc2[0][0], 0, 0, 0);
                acc2[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[u], b0[u], acc2[1][0], 0, 0, 0);
                if (any1) {
                    acc2[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[u], b1[u], acc2[0][1], 0, 0, 0);
                    acc2[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[u], b1[u], acc2[1][1], 0, 0, 0);
                }
            }
        }
    }
    // ---- epilogue: lane holds C[8 (r/4) + 4 (lane/32) + r%4][lane%32] of each 32x32 tile
    __shared__ int32_t tile_row[TM];
    if (threadIdx.x < TM) {
        const int64_t li = tile0 + threadIdx.x;
        int32_t row = -1;
        if (li < nrows) row = g.long_only ? sp.it.long_row[li] : (sp.it.rows_sorted[li] & 0x7FFFFFFF);
        tile_row[threadIdx.x] = row;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int32_t col = j == 0 ? col0 : col1;
        if (col >= g.dout) continue;
        const float bv = g.bias ? g.bias[col] : 0.f;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int tr = 32 * i + 8 * (r >> 2) + 4 * half + (r & 3);
                const int32_t row = tile_row[tr];
                if (row < 0) continue;
                float v = acc2[i][j][r] + bv;
                if (g.relu) v = v > 0.f ? v : 0.f;
                g.y[(int64_t)row * g.dout + col] = v;
            }
    }
}

// out[row,:] = rowscale[row] * (partial[first,:] + partial[first+1,:] + ...): one wavefront per
// long row and 256-column block, segments added in ascending order (eight loads in flight per
// lane).
template <typename TOut, bool VEC>
__global__ __launch_bounds__(kBlock) void k_spmm_long_reduce(const SpmmArgs g)
{
    constexpr int U = 8;
    const int lane = threadIdx.x % kWave;
    const int64_t i = (int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
    if (i >= g.it.nlong) return;
    const int32_t row = g.it.long_row[i];
    const int64_t first = g.it.long_first[i];
    const int32_t ns = g.it.long_nseg[i];
    const float sc = g.rowscale ? g.rowscale[row] : 1.f;
    const int32_t cb = blockIdx.y * 256;          // first column of this block
    TOut* out = static_cast<TOut*>(g.out) + g.out_row(row) * (int64_t)g.ld;
    const bool add = g.adds(row);
    if (VEC) {
        const int32_t c = cb + lane * 4;
        if (c >= g.d) return;
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int32_t t0 = 0; t0 < ns; t0 += U) {
            float4 x[U];
#pragma unroll
            for (int u = 0; u < U; ++u)
                x[u] = t0 + u < ns
                           ? *reinterpret_cast<const float4*>(g.partial + (first + t0 + u) * (int64_t)g.ld + c)
                           : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int u = 0; u < U; ++u) { s.x += x[u].x; s.y += x[u].y; s.z += x[u].z; s.w += x[u].w; }
        }
        float o4[4] = {sc * s.x, sc * s.y, sc * s.z, sc * s.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (add) o4[e] += Elem<TOut>::load(out + c + e);
            if (g.bias) o4[e] += g.bias[c + e];
            if (g.relu) o4[e] = o4[e] > 0.f ? o4[e] : 0.f;
            Elem<TOut>::store(out + c + e, o4[e]);
        }
    } else {
        for (int32_t c = cb + lane; c < g.d && c < cb + 256; c += kWave) {
            float s = 0.f;
            for (int32_t t = 0; t < ns; ++t) s += g.partial[(first + t) * (int64_t)g.ld + c];
            s *= sc;
            if (add) s += Elem<TOut>::load(out + c);
            if (g.bias) s += g.bias[c];
            if (g.relu) s = s > 0.f ? s : 0.f;
            Elem<TOut>::store(out + c, s);
        }
    }
}

// dst[map(i),:] += src[i,:]
template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_scatter_add(const float* __restrict__ src, int64_t nrows,
                                                        int64_t n_own, int64_t base_row,
                                                        const int32_t* __restrict__ idx,
                                                        float* __restrict__ dst, int32_t d,
                                                        int32_t vpr)
{
    const int64_t total = nrows * vpr;
    for (int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x; t < total;
         t += (int64_t)gridDim.x * kBlock) {
        int64_t i = t / vpr;
        int32_t j = (int32_t)(t - i * vpr);
        int64_t r = i < n_own ? base_row + i : (int64_t)idx[i - n_own];
        if (VEC) {
            float4 a = reinterpret_cast<const float4*>(src + i * d)[j];
            float4* p = reinterpret_cast<float4*>(dst + r * d) + j;
            float4 b = *p;
            b.x += a.x; b.y += a.y; b.z += a.z; b.w += a.w;
            *p = b;
        } else {
            dst[r * d + j] += src[i * d + j];
        }
    }
}

// gcol[e] = row of the whole-graph array that local column lcol[e] of partition p stands for:
// own rows follow each other from `base`, the others are listed in the boundary list
__global__ __launch_bounds__(kBlock) void k_global_columns(const int32_t* __restrict__ lcol,
                                                           int32_t* __restrict__ gcol, int64_t count,
                                                           int32_t n_own, int32_t base,
                                                           const int32_t* __restrict__ bnd)
{
    for (int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x; e < count; e += (int64_t)gridDim.x * kBlock) {
        const int32_t c = lcol[e];
        gcol[e] = c < n_own ? base + c : bnd[c - n_own];
    }
}

__global__ __launch_bounds__(kBlock) void k_fill_zero(uint4* __restrict__ p, int64_t n16,
                                                      uint8_t* __restrict__ tail, int ntail)
{
    for (int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x; t < n16;
         t += (int64_t)gridDim.x * kBlock)
        p[t] = make_uint4(0, 0, 0, 0);
    if (blockIdx.x == 0 && (int)threadIdx.x < ntail) tail[threadIdx.x] = 0;
}

}  // namespace

void launch_gather_rows(const void* src, const int32_t* idx, void* dst, int64_t rows,
                        int64_t row_bytes, hipStream_t s)
{
    move_rows<false>(src, idx, dst, rows, row_bytes, s);
}

void launch_scatter_rows(const void* src, const int32_t* idx, void* dst, int64_t rows,
                         int64_t row_bytes, hipStream_t s)
{
    move_rows<true>(src, idx, dst, rows, row_bytes, s);
}

namespace {

// Operators whose rows average fewer entries than this take k_spmm_short.  The choice looks at the
// operator only, never at where its source rows lie, so that one operator is summed by the same
// kernel (in the same order) whether its sources are one array or two.
inline float short_rows_max()
{
    static const float v = [] {
        const char* off = std::getenv("GNNMI_SPMM_SHORT");
        if (off && off[0] == '0') return 0.f;
        const char* e = std::getenv("GNNMI_SPMM_SHORT_MAX");
        return e ? (float)std::atof(e) : 32.f;
    }();
    return v;
}

template <typename TIn, typename TOut>
void spmm_typed(const int64_t* rp, const int32_t* col, const float* w, const float* rowscale,
                const void* a_rows, int64_t n_a, const void* b_rows, void* out, int32_t d,
                const SpmmItems& items, float* partial, bool slices, const SpmmScatter& sc,
                hipStream_t s, int32_t ld)
{
    constexpr int EPV = Elem<TIn>::EPV;
    const int wpb = kBlock / kWave;
    // Column slices across XCDs.  Measured on the 2.4 M-vertex workload (1 KB rows): eight
    // 128-byte slices raise the L2 hit rate from 33 % to 47 % but turn each row into eight
    // separate DRAM accesses, and the fetch rate drops from 6.7 to 5.0 TB/s - no gain; slices of
    // 256 bytes keep DRAM bursts long enough and make the forward aggregation 11 % faster.  The
    // transposed operator consists mostly of rows with one or two entries, whose cost is per
    // row and only grows with slicing (1.3x slower on 2 KB rows), so it is never sliced.
    // So: forward only, slices of 256 to 512 bytes, at most eight.
    static const bool use_slices = [] {
        const char* e = std::getenv("GNNMI_SPMM_SLICES");
        return !(e && e[0] == '0');
    }();
    const int64_t row_bytes = (int64_t)d * (int64_t)sizeof(TIn);
    if (slices && sc.n_own < 0 && use_slices && row_bytes % 512 == 0 && row_bytes <= 4096 && items.rows_sorted &&
        d % Elem<TOut>::EPV == 0) {
        int ns = 8;
        while (ns > 1 && (row_bytes / ns < 256 || row_bytes % (ns * 256) != 0)) ns >>= 1;
        const int G = (int)(row_bytes / ns / 16);   // 16-byte vectors per slice: 16 or 32
        const int S = kWave / (G > 0 ? G : 1);
        const int64_t n_items = items.nsegs + items.nshort;
        const int64_t blocks = (n_items + (int64_t)wpb * S - 1) / ((int64_t)wpb * S);
        if (ns > 1 && (G == 16 || G == 32) && blocks * ns < ((int64_t)1 << 31) && n_items > 0) {
            SpmmArgs g;
            g.rp = rp; g.col = col; g.w = w; g.rowscale = rowscale;
            g.a_rows = a_rows; g.n_a = n_a; g.b_rows = b_rows; g.out = out; g.d = d; g.ld = ld;
            g.it = items; g.partial = partial;
            g.map_n_own = -1; g.map_base = 0; g.map_idx = nullptr; g.map_first = nullptr;
            g.bias = sc.bias; g.relu = sc.relu;
            const dim3 grid((unsigned)(blocks * ns));
            const bool few2s = items.avg_len > 0.f && items.avg_len < short_rows_max();
            if (G == 16 && few2s) hipLaunchKernelGGL((k_spmm_short<TIn, TOut, 16, 4, 1, false>), grid, dim3(kBlock), 0, s, g, ns);
            else if (G == 16) hipLaunchKernelGGL((k_spmm_slots<TIn, TOut, 16>), grid, dim3(kBlock), 0, s, g, ns);
            else if (few2s) hipLaunchKernelGGL((k_spmm_short<TIn, TOut, 32, 4, 1, false>), grid, dim3(kBlock), 0, s, g, ns);
            else hipLaunchKernelGGL((k_spmm_slots<TIn, TOut, 32>), grid, dim3(kBlock), 0, s, g, ns);
            return;
        }
    }
    const bool vec = (d % EPV == 0) && (d % Elem<TOut>::EPV == 0) && (ld % EPV == 0) && (ld % Elem<TOut>::EPV == 0);
    // Narrow rows (at most 512 bytes): the cost is latency per row, not bytes, above all in the
    // transposed operator whose rows have a handful of entries.  The slot-per-item kernel without
    // slicing works on 64 / G rows per wavefront at once instead of one after the other.
    static const bool use_narrow = [] {
        const char* e = std::getenv("GNNMI_SPMM_NARROW");
        return !(e && e[0] == '0');
    }();
    const int nvec = (d + EPV - 1) / EPV;
    // Operators with short rows (the transposed operators R_p: 3 to 27 entries per row on the
    // bench workloads; the forward operators of sparse directed graphs: 17) take the variant with
    // four loads in flight per slot and a rolled loop: 51-57 registers, eight wavefronts per SIMD.
    // Measured: 315 -> 264 ms of transposed aggregation per epoch at 3.6 entries per row, 20.3 ->
    // 18.4 ms at 12; forward 3 % at 17 entries per row, nothing at 55.  `few`: one source array of
    // fewer than 2^32 elements, 32-bit offsets; `few2`: 64-bit addresses.
    const bool short_rows = items.avg_len > 0.f && items.avg_len < short_rows_max();
    const bool few = short_rows && b_rows == nullptr && n_a * (int64_t)ld < ((int64_t)1 << 32);
    const bool few2 = short_rows && !few;
    if (use_narrow && vec && (few || few2) && nvec > 32 && nvec <= 64 && items.rows_sorted && sizeof(TIn) == 4 &&
        (sc.n_own < 0 || sizeof(TOut) == 4) && items.nsegs + items.nshort > 0) {
        // rows of 33..64 vectors: two vectors per lane, two rows per wavefront
        const int64_t n_items = items.nsegs + items.nshort;
        const int64_t blocks = (n_items + (int64_t)wpb * 2 - 1) / ((int64_t)wpb * 2);
        SpmmArgs g;
        g.rp = rp; g.col = col; g.w = w; g.rowscale = rowscale;
        g.a_rows = a_rows; g.n_a = n_a; g.b_rows = b_rows; g.out = out; g.d = d; g.ld = ld;
        g.it = items; g.partial = partial;
        g.map_n_own = sc.n_own; g.map_base = sc.base_row; g.map_idx = sc.idx; g.map_first = sc.first;
        g.bias = sc.bias; g.relu = sc.relu;
        if (few) hipLaunchKernelGGL((k_spmm_short<TIn, TOut, 32, 4, 2>), dim3((unsigned)blocks), dim3(kBlock), 0, s, g, 1);
        else hipLaunchKernelGGL((k_spmm_short<TIn, TOut, 32, 4, 2, false>), dim3((unsigned)blocks), dim3(kBlock), 0, s, g, 1);
        return;
    }
    if (use_narrow && vec && nvec <= 32 && items.rows_sorted && (sc.n_own < 0 || sizeof(TOut) == 4) &&
        items.nsegs + items.nshort > 0) {
        const int G = nvec <= 4 ? 4 : nvec <= 8 ? 8 : nvec <= 16 ? 16 : 32;
        const int S = kWave / G;
        const int64_t n_items = items.nsegs + items.nshort;
        const int64_t blocks = (n_items + (int64_t)wpb * S - 1) / ((int64_t)wpb * S);
        SpmmArgs g;
        g.rp = rp; g.col = col; g.w = w; g.rowscale = rowscale;
        g.a_rows = a_rows; g.n_a = n_a; g.b_rows = b_rows; g.out = out; g.d = d; g.ld = ld;
        g.it = items; g.partial = partial;
        g.map_n_own = sc.n_own; g.map_base = sc.base_row; g.map_idx = sc.idx; g.map_first = sc.first;
        g.bias = sc.bias; g.relu = sc.relu;
        const dim3 grid1((unsigned)blocks);
        if (G == 4) hipLaunchKernelGGL((k_spmm_slots<TIn, TOut, 4>), grid1, dim3(kBlock), 0, s, g, 1);
        else if (G == 8 && few) hipLaunchKernelGGL((k_spmm_short<TIn, TOut, 8, 4, 1>), grid1, dim3(kBlock), 0, s, g, 1);
        else if (G == 8 && few2) hipLaunchKernelGGL((k_spmm_short<TIn, TOut, 8, 4, 1, false>), grid1, dim3(kBlock), 0, s, g, 1);
        else if (G == 8) hipLaunchKernelGGL((k_spmm_slots<TIn, TOut, 8>), grid1, dim3(kBlock), 0, s, g, 1);
        else if (G == 16 && few) hipLaunchKernelGGL((k_spmm_short<TIn, TOut, 16, 4, 1>), grid1, dim3(kBlock), 0, s, g, 1);
        else if (G == 16 && few2) hipLaunchKernelGGL((k_spmm_short<TIn, TOut, 16, 4, 1, false>), grid1, dim3(kBlock), 0, s, g, 1);
        else if (G == 32 && few2) hipLaunchKernelGGL((k_spmm_short<TIn, TOut, 32, 4, 1, false>), grid1, dim3(kBlock), 0, s, g, 1);
        else if (G == 16) hipLaunchKernelGGL((k_spmm_slots<TIn, TOut, 16>), grid1, dim3(kBlock), 0, s, g, 1);
        else if (few) hipLaunchKernelGGL((k_spmm_short<TIn, TOut, 32, 4, 1>), grid1, dim3(kBlock), 0, s, g, 1);
        else hipLaunchKernelGGL((k_spmm_slots<TIn, TOut, 32>), grid1, dim3(kBlock), 0, s, g, 1);
        return;
    }
    const int64_t nitems = items.nsegs + items.nranges;
    const dim3 grid((unsigned)((nitems + wpb - 1) / wpb));
    const dim3 block(kBlock);
    // rows wider than 256 vectors (1024 floats / 2048 bf16) are processed in column blocks
    constexpr int32_t kColBlock = 256 * EPV;
    for (int32_t c0 = 0; c0 < d; c0 += kColBlock) {
        const int32_t dc = d - c0 < kColBlock ? d - c0 : kColBlock;
        SpmmArgs g;
        g.rp = rp; g.col = col; g.w = w; g.rowscale = rowscale;
        g.a_rows = static_cast<const TIn*>(a_rows) + c0; g.n_a = n_a;
        g.b_rows = b_rows ? static_cast<const TIn*>(b_rows) + c0 : nullptr;
        g.out = static_cast<TOut*>(out) + c0; g.d = dc; g.ld = ld; g.it = items;
        g.partial = partial + c0;
        g.map_n_own = sc.n_own; g.map_base = sc.base_row; g.map_idx = sc.idx; g.map_first = sc.first;
        g.bias = sc.bias ? sc.bias + c0 : nullptr; g.relu = sc.relu;
        const int nv = (dc + EPV - 1) / EPV;  // 16-byte vectors per row in this block
#define GNN_SPMM(G, NV, VEC) \
    hipLaunchKernelGGL((k_spmm_items<TIn, TOut, G, NV, VEC>), grid, block, 0, s, g)
        if (vec) {
            if (nv <= 8) GNN_SPMM(8, 1, true);
            else if (nv <= 16) GNN_SPMM(16, 1, true);
            else if (nv <= 32) GNN_SPMM(32, 1, true);
            else if (nv <= 64) GNN_SPMM(64, 1, true);
            else if (nv <= 128) GNN_SPMM(64, 2, true);
            else GNN_SPMM(64, 4, true);
        } else {
            if (nv <= 8) GNN_SPMM(8, 1, false);
            else if (nv <= 16) GNN_SPMM(16, 1, false);
            else if (nv <= 32) GNN_SPMM(32, 1, false);
            else if (nv <= 64) GNN_SPMM(64, 1, false);
            else if (nv <= 128) GNN_SPMM(64, 2, false);
            else GNN_SPMM(64, 4, false);
        }
#undef GNN_SPMM
    }
}

template <typename TOut>
void spmm_reduce_typed(const float* rowscale, void* out, int32_t d, const SpmmItems& items,
                       float* partial, const SpmmScatter& sc, hipStream_t s, int32_t ld)
{
    const int wpb = kBlock / kWave;
    SpmmArgs g{};
    g.rowscale = rowscale; g.out = out; g.d = d; g.ld = ld; g.it = items; g.partial = partial;
    g.map_n_own = sc.n_own; g.map_base = sc.base_row; g.map_idx = sc.idx; g.map_first = sc.first;
    g.bias = sc.bias; g.relu = sc.relu;
    const dim3 rgrid((unsigned)((items.nlong + wpb - 1) / wpb), (unsigned)((d + 255) / 256));
    if (d % 4 == 0 && ld % 4 == 0) hipLaunchKernelGGL((k_spmm_long_reduce<TOut, true>), rgrid, dim3(kBlock), 0, s, g);
    else hipLaunchKernelGGL((k_spmm_long_reduce<TOut, false>), rgrid, dim3(kBlock), 0, s, g);
}

}  // namespace

void launch_spmm(const int64_t* rp, const int32_t* col, const float* w, const float* rowscale,
                 const void* a_rows, int64_t n_a, const void* b_rows, void* out, int64_t nrows,
                 int32_t d, int in_bf16, int out_bf16, const SpmmItems& items, float* partial,
                 int column_slices, const SpmmScatter& sc, hipStream_t s, int32_t ld)
{
    if (nrows <= 0 || d <= 0 || items.nsegs + items.nranges <= 0) return;
    if (ld <= 0) ld = d;
    // rows ld elements apart: the column-sliced kernel cuts whole rows, so only for ld = d
    const bool sl = column_slices != 0 && ld == d;
    if (!in_bf16)
        spmm_typed<float, float>(rp, col, w, rowscale, a_rows, n_a, b_rows, out, d, items, partial, sl, sc, s, ld);
    else if (out_bf16)
        spmm_typed<uint16_t, uint16_t>(rp, col, w, rowscale, a_rows, n_a, b_rows, out, d, items, partial, sl, sc, s, ld);
    else
        spmm_typed<uint16_t, float>(rp, col, w, rowscale, a_rows, n_a, b_rows, out, d, items, partial, sl, sc, s, ld);
}

void launch_spmm_reduce(const float* rowscale, void* out, int32_t d, int out_bf16,
                        const SpmmItems& items, float* partial, const SpmmScatter& sc, hipStream_t s, int32_t ld)
{
    if (items.nlong <= 0 || d <= 0) return;
    if (ld <= 0) ld = d;
    if (out_bf16) spmm_reduce_typed<uint16_t>(rowscale, out, d, items, partial, sc, s, ld);
    else spmm_reduce_typed<float>(rowscale, out, d, items, partial, sc, s, ld);
}

// One launch for the heads of a multi-head aggregation whose heads lie side by side in rows of
// `ld` floats: nh column slices of f floats, slice j weighted by w + j wss (fp32).  The slices of
// a work item go to consecutive workgroups and so to different XCDs, whose caches then hold
// different columns of the source rows.  False (nothing launched) when the slice width is not
// 4, 8, 16 or 32 vectors of 16 bytes or the plan has no list of short rows.
bool launch_spmm_heads(const int64_t* rp, const int32_t* col, const float* w, int64_t wss, int32_t nh, int32_t f,
                       const float* a_rows, int64_t n_a, const float* b_rows, float* out, int32_t ld,
                       const SpmmItems& items, float* partial, const SpmmScatter& sc, hipStream_t s)
{
    const int G = f / 4;
    if (f % 4 != 0 || !(G == 4 || G == 8 || G == 16 || G == 32) || nh * f != ld || !items.rows_sorted) return false;
    const int64_t n_items = items.nsegs + items.nshort;
    if (n_items <= 0) return true;
    const int wpb = kBlock / kWave, S = kWave / G;
    const int64_t blocks = (n_items + (int64_t)wpb * S - 1) / ((int64_t)wpb * S);
    if (blocks * nh >= ((int64_t)1 << 31)) return false;
    SpmmArgs g;
    g.rp = rp; g.col = col; g.w = w; g.wss = wss; g.rowscale = nullptr;
    g.a_rows = a_rows; g.n_a = n_a; g.b_rows = b_rows; g.out = out; g.d = ld; g.ld = ld;
    g.it = items; g.partial = partial;
    g.map_n_own = sc.n_own; g.map_base = sc.base_row; g.map_idx = sc.idx; g.map_first = sc.first;
    g.bias = sc.bias; g.relu = sc.relu;
    const dim3 grid((unsigned)(blocks * nh));
    // operators of short rows: the variant with four loads in flight per slot (64-bit addresses)
    const bool few2 = items.avg_len > 0.f && items.avg_len < short_rows_max();
    if (G == 4) hipLaunchKernelGGL((k_spmm_slots<float, float, 4>), grid, dim3(kBlock), 0, s, g, nh);
    else if (G == 8 && few2) hipLaunchKernelGGL((k_spmm_short<float, float, 8, 4, 1, false>), grid, dim3(kBlock), 0, s, g, nh);
    else if (G == 8) hipLaunchKernelGGL((k_spmm_slots<float, float, 8>), grid, dim3(kBlock), 0, s, g, nh);
    else if (G == 16 && few2) hipLaunchKernelGGL((k_spmm_short<float, float, 16, 4, 1, false>), grid, dim3(kBlock), 0, s, g, nh);
    else if (G == 16) hipLaunchKernelGGL((k_spmm_slots<float, float, 16>), grid, dim3(kBlock), 0, s, g, nh);
    else if (few2) hipLaunchKernelGGL((k_spmm_short<float, float, 32, 4, 1, false>), grid, dim3(kBlock), 0, s, g, nh);
    else hipLaunchKernelGGL((k_spmm_slots<float, float, 32>), grid, dim3(kBlock), 0, s, g, nh);
    return true;
}

bool spmm_gemm_fused_init();

bool spmm_gemm_fused_ok(int32_t din, int32_t dout, const SpmmItems& items)
{
    // Off unless GNNMI_FUSE_AGG=1 (read per call: tests flip it).  Measured on the 50 M-vertex
    // GCN workload the fused forward pass of layer 1 takes 0.63 ms more per partition than the
    // stand-alone aggregation and saves a 0.29 ms contraction (epoch 1051 against 1025 ms; on the
    // 2.4 M-vertex GraphSAGE workload 105 against 99.8 ms): its row fetches lose the column
    // slicing across XCDs, and the LDS tile limits a CU to three or four workgroups.
    const char* e = std::getenv("GNNMI_FUSE_AGG");
    const bool on = e && e[0] == '1';
    return on && din % 4 == 0 && din > 32 && din <= 128 && dout >= 1 && dout <= 256 && items.rows_sorted &&
           items.nshort + items.nlong > 0 && spmm_gemm_fused_init();
}

void launch_spmm_gemm_fused(const int64_t* rp, const int32_t* col, const float* w, const float* rowscale,
                            const float* a_rows, int64_t n_a, const float* b_rows, int32_t din,
                            const SpmmItems& items, float* partial, float* zlong, const float* xself,
                            const float* W, const float* Ws, const float* bias, int relu, float* y,
                            int32_t dout, int stage, hipStream_t s)
{
    FusedArgs g{};
    g.sp.rp = rp; g.sp.col = col; g.sp.w = w; g.sp.rowscale = rowscale;
    g.sp.a_rows = a_rows; g.sp.n_a = n_a; g.sp.b_rows = b_rows; g.sp.out = nullptr;
    g.sp.d = din; g.sp.ld = din; g.sp.it = items; g.sp.partial = partial;
    g.sp.map_n_own = -1; g.sp.map_base = 0; g.sp.map_idx = nullptr; g.sp.map_first = nullptr; g.sp.bias = nullptr; g.sp.relu = 0;
    g.zlong = zlong; g.xself = xself; g.w = W; g.ws = Ws; g.bias = bias; g.y = y; g.dout = dout; g.relu = relu;
    g.kp = din + 1;
    const size_t lds = (size_t)64 * (size_t)g.kp * sizeof(float) * (xself ? 2 : 1);
    const int G = din <= 64 ? 16 : 32;
    const int64_t per_block = (int64_t)(kBlock / kWave) * (kWave / G);      // segments per workgroup
    if (stage == 0) {
        // segments first in the grid (they are the longest items), then the short rows in tiles of 64
        g.seg_blocks = (int32_t)((items.nsegs + per_block - 1) / per_block);
        g.long_only = 0;
        const int64_t blocks = g.seg_blocks + (items.nshort + 63) / 64;
        if (blocks <= 0) return;
        if (G == 16) hipLaunchKernelGGL((k_agg_gemm<16>), dim3((unsigned)blocks), dim3(kBlock), lds, s, g);
        else hipLaunchKernelGGL((k_agg_gemm<32>), dim3((unsigned)blocks), dim3(kBlock), lds, s, g);
    } else if (stage == 1) {
        launch_spmm_reduce(rowscale, zlong, din, 0, items, partial, SpmmScatter{}, s);
    } else if (items.nlong > 0) {
        g.seg_blocks = 0;
        g.long_only = 1;
        const dim3 grid((unsigned)((items.nlong + 63) / 64));
        if (G == 16) hipLaunchKernelGGL((k_agg_gemm<16>), grid, dim3(kBlock), lds, s, g);
        else hipLaunchKernelGGL((k_agg_gemm<32>), grid, dim3(kBlock), lds, s, g);
    }
}

// largest dynamic LDS the fused kernel may ask for: 64 rows x 129 floats, twice (GraphSAGE)
bool spmm_gemm_fused_init()
{
    constexpr int kMaxLds = 2 * 64 * 129 * 4;
    static const bool ok =
        hipFuncSetAttribute((const void*)k_agg_gemm<16>, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds) == hipSuccess &&
        hipFuncSetAttribute((const void*)k_agg_gemm<32>, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds) == hipSuccess;
    if (!ok) (void)hipGetLastError();
    return ok;
}

void launch_scatter_add(const float* src, int64_t nrows, int64_t n_own, int64_t base_row,
                        const int32_t* idx, float* dst, int32_t d, hipStream_t s)
{
    if (nrows <= 0 || d <= 0) return;
    const bool vec = (d % 4 == 0);
    const int32_t vpr = vec ? d / 4 : d;
    int64_t blocks = (nrows * vpr + kBlock - 1) / kBlock;
    blocks = blocks > 65536 * 4 ? 65536 * 4 : blocks;
    if (vec)
        hipLaunchKernelGGL((k_scatter_add<true>), dim3((unsigned)blocks), dim3(kBlock), 0, s, src,
                           nrows, n_own, base_row, idx, dst, d, vpr);
    else
        hipLaunchKernelGGL((k_scatter_add<false>), dim3((unsigned)blocks), dim3(kBlock), 0, s, src,
                           nrows, n_own, base_row, idx, dst, d, vpr);
}

void launch_global_columns(const int32_t* lcol, int32_t* gcol, int64_t count, int64_t n_own, int64_t base,
                           const int32_t* bnd, hipStream_t s)
{
    if (count <= 0) return;
    const int64_t blocks = std::min<int64_t>((count + kBlock - 1) / kBlock, 8192);
    hipLaunchKernelGGL(k_global_columns, dim3((unsigned)blocks), dim3(kBlock), 0, s, lcol, gcol, count,
                       (int32_t)n_own, (int32_t)base, bnd);
}

void launch_fill_zero(void* p, int64_t bytes, hipStream_t s)
{
    if (bytes <= 0) return;
    int64_t n16 = bytes / 16;
    int ntail = (int)(bytes - n16 * 16);
    int64_t blocks = (n16 + kBlock - 1) / kBlock;
    blocks = blocks < 1 ? 1 : (blocks > 16384 ? 16384 : blocks);
    hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)blocks), dim3(kBlock), 0, s, (uint4*)p, n16,
                       (uint8_t*)p + n16 * 16, ntail);
}

}  // namespace gnnmi
