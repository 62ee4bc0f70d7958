// HBM-bound kernels of the path: boundary gather, CSR aggregation (forward, recompute and
// transposed), scatter-add.  gfx950, wave64.
//
//   gather      staging[i,:] = A^{l-1}[B_p[i],:]                       (Gather / regather step)
//   spmm        Z_p[v,:] = scale_v * sum_{e in row v} w_e * src(col_e)  (aggregation along T_p)
//   scatter-add grad A^{l-1}[owner(i),:] += grad GA_p[i,:]              (scatter-accumulate step)
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
    if (row_bytes % 16 == 0)
        move_rows_typed<float4, SCATTER>(src, idx, dst, rows, (int32_t)(row_bytes / 16), s);
    else if (row_bytes % 4 == 0)
        move_rows_typed<uint32_t, SCATTER>(src, idx, dst, rows, (int32_t)(row_bytes / 4), s);
    else if (row_bytes % 2 == 0)
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
    const float* rowscale;
    const float* a_rows;
    int64_t n_a;
    const float* b_rows;
    float* out;
    int32_t d, ld;          // d: columns handled by this launch; ld: row stride
    SpmmItems it;
    float* partial;
};

template <int G, int NV, bool VEC>
__device__ inline void spmm_accumulate(const SpmmArgs& g, int64_t e_begin, int64_t e_end, int lane,
                                       float (&acc)[NV][4])
{
    constexpr int S = kWave / G;
    constexpr int UNROLL = (NV == 1) ? 8 : 4;   // source rows in flight per slot
    const int slot = lane / G;
    const int gl = lane % G;
    // column offsets of this lane's float4s; lanes past the row end read column 0 (their sums
    // are never stored), so that every load below is unconditional and the compiler can keep
    // all of them in flight
    int c4[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int c = (v * G + gl) * 4;
        c4[v] = c < g.d ? c : 0;
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
            const float* src[UNROLL];
            float ww[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int j = j0 + u * S + slot;
                const int jj = j < cnt ? j : cnt - 1;     // stay on a valid entry
                const int32_t c = __shfl(cur_c, jj, kWave);
                const float wt = __shfl(cur_w, jj, kWave);
                ww[u] = j < cnt ? wt : 0.f;
                src[u] = (c < g.n_a) ? g.a_rows + (int64_t)c * g.ld
                                     : g.b_rows + ((int64_t)c - g.n_a) * g.ld;
            }
            if (VEC) {
                float4 x[UNROLL][NV];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u)
#pragma unroll
                    for (int v = 0; v < NV; ++v)
                        x[u][v] = *reinterpret_cast<const float4*>(src[u] + c4[v]);
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) {
                    const bool on = (j0 + u * S + slot) < cnt;
#pragma unroll
                    for (int v = 0; v < NV; ++v) {
                        acc[v][0] += on ? ww[u] * x[u][v].x : 0.f;
                        acc[v][1] += on ? ww[u] * x[u][v].y : 0.f;
                        acc[v][2] += on ? ww[u] * x[u][v].z : 0.f;
                        acc[v][3] += on ? ww[u] * x[u][v].w : 0.f;
                    }
                }
            } else {
#pragma unroll
                for (int u = 0; u < UNROLL; ++u)
#pragma unroll
                    for (int v = 0; v < NV; ++v)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            int c = (v * G + gl) * 4 + i;
                            if (c < g.d && ww[u] != 0.f) acc[v][i] += ww[u] * src[u][c];
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
            for (int i = 0; i < 4; ++i) acc[v][i] += __shfl_xor(acc[v][i], m, kWave);
}

template <int G, int NV, bool VEC>
__device__ inline void spmm_store(float* o, int32_t d, int lane, float sc, const float (&acc)[NV][4])
{
    if (lane >= G) return;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        int c4 = (v * G + lane) * 4;
        if (VEC) {
            if (c4 < d)
                *reinterpret_cast<float4*>(o + c4) =
                    make_float4(sc * acc[v][0], sc * acc[v][1], sc * acc[v][2], sc * acc[v][3]);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (c4 + i < d) o[c4 + i] = sc * acc[v][i];
        }
    }
}

template <int G, int NV, bool VEC>
__global__ __launch_bounds__(kBlock) void k_spmm_items(const SpmmArgs g)
{
    const int lane = threadIdx.x % kWave;
    // the item index is the same for the whole wavefront; tell the compiler so that row
    // pointers and item descriptors travel through scalar registers
    const int64_t item = __builtin_amdgcn_readfirstlane(
        (int)(blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave));
    float acc[NV][4];
    if (item < g.it.nsegs) {
        // one segment of a long row -> partial sum
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[v][i] = 0.f;
        const int64_t e0 = g.it.seg_begin[item];
        spmm_accumulate<G, NV, VEC>(g, e0, e0 + g.it.seg_len[item], lane, acc);
        spmm_store<G, NV, VEC>(g.partial + item * (int64_t)g.ld, g.d, lane, 1.f, acc);
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
            for (int i = 0; i < 4; ++i) acc[v][i] = 0.f;
        spmm_accumulate<G, NV, VEC>(g, e_begin, e_end, lane, acc);
        spmm_store<G, NV, VEC>(g.out + row * (int64_t)g.ld, g.d, lane,
                               g.rowscale ? g.rowscale[row] : 1.f, acc);
    }
}

// out[row,:] = rowscale[row] * (partial[first,:] + partial[first+1,:] + ...): one wavefront per
// long row and 256-float column block, segments added in ascending order (eight loads in
// flight per lane).
template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_spmm_long_reduce(const SpmmArgs g, int32_t c0,
                                                             int32_t dc)
{
    constexpr int U = 8;
    const int lane = threadIdx.x % kWave;
    const int64_t i = (int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
    if (i >= g.it.nlong) return;
    const int32_t row = g.it.long_row[i];
    const int64_t first = g.it.long_first[i];
    const int32_t ns = g.it.long_nseg[i];
    const float sc = g.rowscale ? g.rowscale[row] : 1.f;
    const int32_t cb = c0 + blockIdx.y * 256;          // first column of this block
    const int32_t cend = c0 + dc;
    if (VEC) {
        const int32_t c = cb + lane * 4;
        if (c >= cend) return;
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
        *reinterpret_cast<float4*>(g.out + row * (int64_t)g.ld + c) =
            make_float4(sc * s.x, sc * s.y, sc * s.z, sc * s.w);
    } else {
        for (int32_t c = cb + lane; c < cend && c < cb + 256; c += kWave) {
            float s = 0.f;
            for (int32_t t = 0; t < ns; ++t) s += g.partial[(first + t) * (int64_t)g.ld + c];
            g.out[row * (int64_t)g.ld + c] = sc * s;
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
SpmmArgs spmm_args(const int64_t* rp, const int32_t* col, const float* w, const float* rowscale,
                   const float* a_rows, int64_t n_a, const float* b_rows, float* out, int32_t c0,
                   int32_t dc, int32_t d, const SpmmItems& items, float* partial)
{
    SpmmArgs g;
    g.rp = rp; g.col = col; g.w = w; g.rowscale = rowscale;
    g.a_rows = a_rows + c0; g.n_a = n_a; g.b_rows = b_rows ? b_rows + c0 : nullptr;
    g.out = out + c0; g.d = dc; g.ld = d; g.it = items; g.partial = partial + c0;
    return g;
}
}  // namespace

void launch_spmm(const int64_t* rp, const int32_t* col, const float* w, const float* rowscale,
                 const float* a_rows, int64_t n_a, const float* b_rows, float* out,
                 int64_t nrows, int32_t d, const SpmmItems& items, float* partial, hipStream_t s)
{
    if (nrows <= 0 || d <= 0) return;
    const int64_t nitems = items.nsegs + items.nranges;
    if (nitems <= 0) return;
    const int wpb = kBlock / kWave;
    const dim3 grid((unsigned)((nitems + wpb - 1) / wpb));
    const dim3 block(kBlock);
    const bool vec = (d % 4 == 0);
    // rows wider than 1024 floats are processed in column blocks of 1024, one launch each
    for (int32_t c0 = 0; c0 < d; c0 += 1024) {
        const int32_t dc = d - c0 < 1024 ? d - c0 : 1024;
        const SpmmArgs g = spmm_args(rp, col, w, rowscale, a_rows, n_a, b_rows, out, c0, dc, d, items,
                                     partial);
        const int nv4 = (dc + 3) / 4;  // float4 columns of this block
#define GNN_SPMM(G, NV, VEC) \
    hipLaunchKernelGGL((k_spmm_items<G, NV, VEC>), grid, block, 0, s, g)
        if (vec) {
            if (nv4 <= 8) GNN_SPMM(8, 1, true);
            else if (nv4 <= 16) GNN_SPMM(16, 1, true);
            else if (nv4 <= 32) GNN_SPMM(32, 1, true);
            else if (nv4 <= 64) GNN_SPMM(64, 1, true);
            else if (nv4 <= 128) GNN_SPMM(64, 2, true);
            else GNN_SPMM(64, 4, true);
        } else {
            if (nv4 <= 8) GNN_SPMM(8, 1, false);
            else if (nv4 <= 16) GNN_SPMM(16, 1, false);
            else if (nv4 <= 32) GNN_SPMM(32, 1, false);
            else if (nv4 <= 64) GNN_SPMM(64, 1, false);
            else if (nv4 <= 128) GNN_SPMM(64, 2, false);
            else GNN_SPMM(64, 4, false);
        }
#undef GNN_SPMM
    }
}

void launch_spmm_reduce(const float* rowscale, float* out, int32_t d, const SpmmItems& items,
                        float* partial, hipStream_t s)
{
    if (items.nlong <= 0 || d <= 0) return;
    const int wpb = kBlock / kWave;
    const bool vec = (d % 4 == 0);
    SpmmArgs g = spmm_args(nullptr, nullptr, nullptr, rowscale, nullptr, 0, nullptr, out, 0, d, d, items,
                           partial);
    const dim3 rgrid((unsigned)((items.nlong + wpb - 1) / wpb), (unsigned)((d + 255) / 256));
    if (vec) hipLaunchKernelGGL(k_spmm_long_reduce<true>, rgrid, dim3(kBlock), 0, s, g, 0, d);
    else hipLaunchKernelGGL(k_spmm_long_reduce<false>, rgrid, dim3(kBlock), 0, s, g, 0, d);
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
