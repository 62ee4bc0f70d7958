// C ABI of libgnnmi: context, validation, device mirrors of the partition metadata, and the
// per-(layer, partition) schedule of the paper's overall procedure (forward: gather, FW;
// backward: regather, BW, scatter-accumulate).
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

#include "gnn_ctx.h"

using namespace gnnmi;

namespace {

thread_local std::string g_create_error;

constexpr int64_t kAlign = 256;
int64_t align_up(int64_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

}  // namespace

namespace {

void free_plan(DevMeta::Plan& P)
{
    if (P.range_rows) (void)hipFree(P.range_rows);
    if (P.seg_row) (void)hipFree(P.seg_row);
    if (P.seg_begin) (void)hipFree(P.seg_begin);
    if (P.seg_len) (void)hipFree(P.seg_len);
    if (P.long_row) (void)hipFree(P.long_row);
    if (P.long_first) (void)hipFree(P.long_first);
    if (P.long_nseg) (void)hipFree(P.long_nseg);
    if (P.rows_sorted) (void)hipFree(P.rows_sorted);
    P = DevMeta::Plan{};
}

void free_masked(DevMeta::Masked& T)
{
    if (T.trp) (void)hipFree(T.trp);
    if (T.tcol) (void)hipFree(T.tcol);
    if (T.tw) (void)hipFree(T.tw);
    if (T.out_row) (void)hipFree(T.out_row);
    free_plan(T.plan);
    T = DevMeta::Masked{};
}

void free_device(DevMeta& D)
{
    free_masked(D.masked_t);
    if (D.rp) (void)hipFree(D.rp);
    if (D.lcol) (void)hipFree(D.lcol);
    if (D.gcol) (void)hipFree(D.gcol);
    if (D.ew) (void)hipFree(D.ew);
    if (D.rscale) (void)hipFree(D.rscale);
    if (D.bnd) (void)hipFree(D.bnd);
    if (D.bnd_local) (void)hipFree(D.bnd_local);
    if (D.bnd_flat) (void)hipFree(D.bnd_flat);
    if (D.trp) (void)hipFree(D.trp);
    if (D.tcol) (void)hipFree(D.tcol);
    if (D.tw) (void)hipFree(D.tw);
    if (D.order) (void)hipFree(D.order);
    if (D.tperm) (void)hipFree(D.tperm);
    if (D.first) (void)hipFree(D.first);
    free_plan(D.fwd);
    free_plan(D.bwd);
    D = DevMeta{};
}

template <typename T>
hipError_t upload(T*& dst, const std::vector<T>& src)
{
    dst = nullptr;
    if (src.empty()) return hipSuccess;
    hipError_t e = hipMalloc((void**)&dst, src.size() * sizeof(T));
    if (e != hipSuccess) return e;
    return hipMemcpy(dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice);
}

hipError_t upload_plan(DevMeta::Plan& P, const HostMeta::Plan& H)
{
    hipError_t e = hipSuccess;
    auto step = [&](hipError_t r) { if (e == hipSuccess) e = r; };
    step(upload(P.range_rows, H.range_rows));
    step(upload(P.seg_row, H.seg_row));
    step(upload(P.seg_begin, H.seg_begin));
    step(upload(P.seg_len, H.seg_len));
    step(upload(P.long_row, H.long_row));
    step(upload(P.long_first, H.long_first));
    step(upload(P.long_nseg, H.long_nseg));
    step(upload(P.rows_sorted, H.rows_sorted));
    return e;
}

// Reads the bound train mask and builds the output layer's transposed operator over train
// vertices, on the host, then uploads it.
gnn_status build_masked(gnn_ctx* c)
{
    free_masked(c->D.masked_t);
    c->M.masked_t = HostMeta::MaskedTranspose{};
    std::vector<uint8_t> mask((size_t)c->M.n);
    hipError_t e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipMemcpy(mask.data(), c->mask, mask.size(), hipMemcpyDeviceToHost);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return c->fail(GNN_EHIP, std::string("reading the train mask: ") + hipGetErrorString(e));
    }
    try {
        build_masked_transpose(c->M, mask.data());
    } catch (const std::bad_alloc&) {
        c->M.masked_t = HostMeta::MaskedTranspose{};
        return c->fail(GNN_ENOMEM, "out of host memory while building the train-vertex operator");
    }
    const HostMeta::MaskedTranspose& H = c->M.masked_t;
    DevMeta::Masked& T = c->D.masked_t;
    auto step = [&](hipError_t r) { if (e == hipSuccess) e = r; };
    step(upload(T.trp, H.trp));
    step(upload(T.tcol, H.tcol));
    step(upload(T.tw, H.tw));
    step(upload(T.out_row, H.out_row));
    step(upload_plan(T.plan, H.plan));
    if (e != hipSuccess) {
        free_masked(T);
        (void)hipGetLastError();
        return c->fail(e == hipErrorOutOfMemory ? GNN_ENOMEM : GNN_EHIP,
                       std::string("uploading the train-vertex operator: ") + hipGetErrorString(e));
    }
    T.ready = true;
    // the host copy of the entries is not needed again (the plan offsets are)
    std::vector<int32_t>().swap(c->M.masked_t.tcol);
    std::vector<float>().swap(c->M.masked_t.tw);
    std::vector<int32_t>().swap(c->M.masked_t.out_row);
    return GNN_OK;
}

// HostMeta::first_bits: the partitions in schedule order, each one's rows (own, then B_p) marked
// when nobody before them named the same row of the whole-graph array.
void build_first_touch(HostMeta& M)
{
    M.first_off.assign((size_t)M.k + 1, 0);
    for (int32_t p = 0; p < M.k; ++p) {
        const int64_t rows = (M.off[(size_t)p + 1] - M.off[(size_t)p]) + (M.boff[(size_t)p + 1] - M.boff[(size_t)p]);
        M.first_off[(size_t)p + 1] = M.first_off[(size_t)p] + (rows + 31) / 32;
    }
    M.first_bits.assign((size_t)M.first_off[(size_t)M.k], 0u);
    std::vector<uint8_t> seen((size_t)M.n, 0);
    for (int32_t t = 0; t < M.k; ++t) {
        const int32_t p = M.sched[(size_t)t];
        uint32_t* bits = M.first_bits.data() + M.first_off[(size_t)p];
        const int64_t r0 = M.off[(size_t)p], np = M.off[(size_t)p + 1] - r0;
        const int64_t b0 = M.boff[(size_t)p], nb = M.boff[(size_t)p + 1] - b0;
        for (int64_t r = 0; r < np + nb; ++r) {
            const int64_t row = r < np ? r0 + r : (int64_t)M.bnd[(size_t)(b0 + r - np)];
            if (!seen[(size_t)row]) {
                seen[(size_t)row] = 1;
                bits[r >> 5] |= 1u << (r & 31);
            }
        }
    }
    // the short rows of the transposed plan carry the same mark in the top bit of their list
    // entry, where the kernels that walk that list find it without another load
    HostMeta::Plan& B = M.plan_bwd;
    for (int32_t p = 0; p < M.k && !B.rows_off.empty(); ++p) {
        const uint32_t* bits = M.first_bits.data() + M.first_off[(size_t)p];
        for (int64_t i = B.rows_off[(size_t)p]; i < B.rows_off[(size_t)p + 1]; ++i) {
            const int32_t r = B.rows_sorted[(size_t)i] & 0x7FFFFFFF;
            const bool first = (bits[r >> 5] >> (r & 31)) & 1u;
            B.rows_sorted[(size_t)i] = first ? (int32_t)((uint32_t)r | 0x80000000u) : r;
        }
    }
}

gnn_status ensure_device(gnn_ctx* c)
{
    if (c->D.ready) return GNN_OK;
    DevMeta& D = c->D;
    try {
        build_first_touch(c->M);
    } catch (const std::bad_alloc&) {
        return c->fail(GNN_ENOMEM, "out of host memory while marking first-touch rows");
    }
    const HostMeta& M = c->M;
    hipError_t e = hipSuccess;
    auto step = [&](hipError_t r) { if (e == hipSuccess) e = r; };
    step(upload(D.rp, M.rp));
    step(upload(D.lcol, M.lcol));
    step(upload(D.ew, M.ew));
    step(upload(D.rscale, M.rscale));
    step(upload(D.bnd, M.bnd));
    step(upload(D.bnd_local, M.bnd_local));
    step(upload(D.bnd_flat, M.bnd_flat));
    step(upload(D.trp, M.trp));
    step(upload(D.tcol, M.tcol));
    step(upload(D.tw, M.tw));
    step(upload(D.order, M.order));
    step(upload(D.tperm, M.tperm));
    step(upload(D.first, M.first_bits));
    step(upload_plan(D.fwd, M.plan_fwd));
    step(upload_plan(D.bwd, M.plan_bwd));
    if (e != hipSuccess) {
        free_device(D);
        (void)hipGetLastError();
        return c->fail(e == hipErrorOutOfMemory ? GNN_ENOMEM : GNN_EHIP,
                       std::string("uploading partition metadata: ") + hipGetErrorString(e));
    }
    D.ready = true;
    return GNN_OK;
}

// Column indices of every partition's operator as rows of the whole-graph arrays.
gnn_status ensure_global_columns(gnn_ctx* c)
{
    if (c->D.gcol || c->M.lcol.empty()) return GNN_OK;
    const HostMeta& M = c->M;
    hipError_t e = hipMalloc((void**)&c->D.gcol, M.lcol.size() * sizeof(int32_t));
    if (e != hipSuccess) {
        c->D.gcol = nullptr;
        (void)hipGetLastError();
        return c->fail(e == hipErrorOutOfMemory ? GNN_ENOMEM : GNN_EHIP,
                       std::string("global column indices: ") + hipGetErrorString(e));
    }
    for (int32_t p = 0; p < M.k; ++p) {
        const int64_t r0 = M.off[(size_t)p], r1 = M.off[(size_t)p + 1];
        const int64_t e0 = M.rp[(size_t)r0], e1 = M.rp[(size_t)r1];
        launch_global_columns(c->D.lcol + e0, c->D.gcol + e0, e1 - e0, r1 - r0, r0, c->D.bnd + M.boff[(size_t)p], nullptr);
    }
    e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipGetLastError();
    if (e != hipSuccess) {
        (void)hipFree(c->D.gcol);
        c->D.gcol = nullptr;
        return c->fail(GNN_EHIP, std::string("global column indices: ") + hipGetErrorString(e));
    }
    return GNN_OK;
}

// Streaming schedule: may layers transform first?  Their whole-graph buffer must leave room in
// the HBM budget for two whole per-layer arrays of the widest layer (a layer's input and output,
// or its input and the gradient it produces) beside the smallest block cache.  With less, the
// arrays a transform-first layer reads and writes would each cross the host link several times
// and the schedule that aggregates first, keeping whole arrays in the pool, moves fewer bytes
// over the link (measured on the beyond-HBM recipe at 56 % of its working set: 1.43 s per epoch
// against 1.99 s, both bound by the link).
void update_stream_xf(gnn_ctx* c)
{
    c->stream_xf_ok = false;
    if (!c->streaming() || !c->built || c->model == GNN_GAT) return;
    int64_t dmax = 0;
    for (int32_t d : c->dims) dmax = std::max<int64_t>(dmax, d);
    const int64_t blk = (std::max<int64_t>(1, c->M.stats.max_own) * dmax * 4 + 255) / 256 * 256;
    const int64_t array = (int64_t)c->M.k * blk;
    c->stream_xf_ok = c->xf_buffer_bytes(c->M.n) + 2 * array + 4 * blk <= c->hbm_budget / 256 * 256;
}

void compute_workspace(gnn_ctx* c)
{
    update_stream_xf(c);
    const HostMeta& M = c->M;
    const int32_t L = c->L;
    int64_t max_np = M.stats.max_own, max_b = M.stats.max_boundary, max_r = 0;
    for (int32_t p = 0; p < M.k; ++p)
        max_r = std::max(max_r, M.toff[(size_t)p + 1] - M.toff[(size_t)p]);
    int64_t din = 0, dout = 0, part = 0;
    for (int32_t l = 0; l < L; ++l) {
        din = std::max<int64_t>(din, c->dims[(size_t)l]);
        dout = std::max<int64_t>(dout, c->dims[(size_t)l + 1]);
        int sp = gemm_tn_splits(max_np, c->dims[(size_t)l], c->dims[(size_t)l + 1]);
        part = std::max(part, (int64_t)sp * c->dims[(size_t)l] * c->dims[(size_t)l + 1]);
        if (c->nheads(l + 1) > 1) {   // the weight gradient is taken head by head
            sp = gemm_tn_splits(max_np, c->dims[(size_t)l], c->head_cols(l + 1));
            part = std::max(part, (int64_t)sp * c->dims[(size_t)l] * c->head_cols(l + 1));
        }
        if (c->bf16())
            part = std::max(part, gemm_bf16_tn_partial_floats(max_np, c->dims[(size_t)l], c->dims[(size_t)l + 1]));
    }
    // rows that pass through staging, Z, the padded dY copy and the segment partial sums are as
    // wide as the widest aggregated row: an input width, or the padded output width of a layer
    // that transforms first
    for (int32_t l = 1; l <= L; ++l)
        if (c->transform_first(l)) din = std::max<int64_t>(din, c->hrow(l));
    Workspace& w = c->ws;
    w.staging_bytes = align_up(std::max<int64_t>(1, max_b * din * 4));
    int64_t o = 0;
    auto take = [&](int64_t floats) { int64_t at = o; o += align_up(std::max<int64_t>(1, floats) * 4); return at; };
    w.z = take(max_np * din);
    w.z2 = take(max_np * din);
    w.zkeep.assign((size_t)L, -1);
    if (c->keep_forward && c->model != GNN_GAT && !c->streaming())
        for (int32_t l = 1; l <= L; ++l)
            if (!c->transform_first(l))      // n rows of the layer's input width, storage type
                w.zkeep[(size_t)l - 1] = take((M.n * (int64_t)c->dims[(size_t)l - 1] * c->es() + 3) / 4);
    w.dy = take(max_np * dout);
    w.dz = take(max_np * din);
    w.dga = take(max_r * din);
    w.partial = take(part);
    w.partial2 = take(part);
    w.colpart = take(std::max(act_bwd_partial_floats(max_np, (int32_t)dout),
                              gat_rank1_partial_floats(max_np, (int32_t)dout)));
    w.losspart = take(loss_partial_floats(M.n, M.k));
    w.scalars = take(64);
    w.segpart = take(std::max(M.plan_fwd.max_segs, M.plan_bwd.max_segs) * din);
    if (c->bf16()) {
        int64_t wmax = 0;
        for (int32_t l = 0; l < L; ++l)
            wmax = std::max<int64_t>(wmax, (int64_t)c->dims[(size_t)l] * c->dims[(size_t)l + 1]);
        w.wt = take((wmax + 1) / 2);
    }
    int64_t hp = 0;
    for (int32_t l = 1; l <= L; ++l)
        if (c->transform_first(l)) hp = std::max<int64_t>(hp, c->hrow(l));
    w.h = w.gh = 0;
    w.h_floats = w.dyall_floats = 0;
    if (hp > 0) {
        // H is read by the forward pass only and its gradient exists in the backward pass only:
        // one buffer serves both, except for attention, whose backward pass reads H again.
        // (Streaming schedule: these whole-graph buffers come out of the HBM budget instead, see
        // stream_engine_create.)
        w.h_floats = M.n * hp;
        w.gat_h_off.clear();
        if (!c->streaming()) {
            if (c->model == GNN_GAT && c->keep_forward) {
                // one H per layer, one after the other
                int64_t total = 0;
                for (int32_t l = 1; l <= L; ++l) {
                    w.gat_h_off.push_back(total);
                    total += M.n * (int64_t)c->hrow(l);
                }
                w.h = take(total);
            } else {
                w.h = take(M.n * hp);
            }
            w.gh = c->model == GNN_GAT ? take(M.n * hp) : w.h;
        }
        w.wpad = take(2 * din * hp);
    }
    w.dyall = -1;
    if (c->model == GNN_SAGE_MEAN && !c->bf16()) {
        int64_t dyw = 0;
        for (int32_t l = 2; l < L; ++l)
            if (c->transform_first(l)) dyw = std::max<int64_t>(dyw, c->padded(l));
        if (dyw > 0 && !c->streaming()) {
            w.dyall_floats = M.n * dyw;
            w.dyall = take(M.n * dyw);
        }
    }
    if (c->model == GNN_GAT) {
        const int64_t mh = c->max_heads();      // per-vertex scores: the heads' values side by side
        // (kept forward results: the scores of every layer, the attention weights of every layer
        // and partition)
        const int64_t keepl = c->keep_forward ? L : 1;
        w.ssrc = take(M.n * mh * keepl);
        w.sdst = take(M.n * mh * keepl);
        w.gssrc = take(M.n * mh);
        w.gsdst = take(M.n * mh);
        w.bs = take(max_b * mh);
        w.att = take(M.stats.max_nnz * mh * (c->keep_forward ? (int64_t)L * M.k : 1));   // per-entry arrays: one per head
        w.dal = take(M.stats.max_nnz * mh);
        w.twatt = take(M.stats.max_nnz * mh);
        w.pair = take(M.stats.max_nnz * mh * 2);
    }
    w.scratch_bytes = o;
}

gnn_status check_lp(gnn_ctx* c, int32_t layer, int32_t p)
{
    if (!c->bound) return c->fail(GNN_ESTATE, "buffers are not bound (call gnn_bind)");
    if (layer < 1 || layer > c->L) return c->fail(GNN_EINVAL, "layer outside 1..L");
    if (p < 0 || p >= c->M.k) return c->fail(GNN_EINVAL, "partition outside 0..k-1");
    if (c->streaming())
        return c->fail(GNN_EUNSUPPORTED,
                       "with a streaming budget only gnn_epoch drives the schedule; the per-partition "
                       "entry points need resident buffers");
    return GNN_OK;
}


// Z_p = S_p [in_own ; staging]
void run_spmm_fwd(gnn_ctx* c, int32_t layer, int32_t p, const char* in_own, hipStream_t s)
{
    const HostMeta& M = c->M;
    const int64_t r0 = M.off[(size_t)p], np = M.off[(size_t)p + 1] - r0;
    const int32_t din = c->dims[(size_t)layer - 1];
    SpmmItems items = plan_items(M.plan_fwd, c->D.fwd, p);
    items.avg_len = (float)(M.rp[(size_t)M.off[(size_t)p + 1]] - M.rp[(size_t)r0]) / (float)std::max<int64_t>(1, np);
    const float* rscale = c->D.rscale ? c->D.rscale + r0 : nullptr;
    void* Z = c->z_region(layer, p);
    float* segpart = (float*)(c->scratch + c->ws.segpart);
    const int b16 = c->bf16() ? 1 : 0;
    {
        Timed t(c, s, GNN_K_SPMM);
        if (c->gather_fused())
            launch_spmm(c->D.rp + r0, c->D.gcol, c->D.ew, rscale, c->layer_input(layer), M.n, nullptr, Z, np, din,
                        b16, b16, items, segpart, 1, SpmmScatter{}, s);
        else
            launch_spmm(c->D.rp + r0, c->D.lcol, c->D.ew, rscale, in_own, np, c->staging, Z, np, din, b16,
                        b16, items, segpart, 1, SpmmScatter{}, s);
    }
    if (items.nlong > 0) {
        Timed t(c, s, GNN_K_SPMM_REDUCE);
        launch_spmm_reduce(rscale, Z, din, b16, items, segpart, SpmmScatter{}, s);
    }
}

}  // namespace

namespace gnnmi {

SpmmItems plan_items(const HostMeta::Plan& H, const DevMeta::Plan& P, int32_t p)
{
    SpmmItems it;
    const int64_t r0 = H.range_off[(size_t)p], s0 = H.seg_off[(size_t)p], l0 = H.long_off[(size_t)p];
    it.nranges = H.range_off[(size_t)p + 1] - r0 - 1;
    if (it.nranges < 0) it.nranges = 0;
    it.range_rows = P.range_rows ? P.range_rows + r0 : nullptr;
    it.nsegs = H.seg_off[(size_t)p + 1] - s0;
    it.seg_row = P.seg_row ? P.seg_row + s0 : nullptr;
    it.seg_begin = P.seg_begin ? P.seg_begin + s0 : nullptr;
    it.seg_len = P.seg_len ? P.seg_len + s0 : nullptr;
    it.nlong = H.long_off[(size_t)p + 1] - l0;
    it.long_row = P.long_row ? P.long_row + l0 : nullptr;
    it.long_first = P.long_first ? P.long_first + l0 : nullptr;
    it.long_nseg = P.long_nseg ? P.long_nseg + l0 : nullptr;
    it.nshort = H.rows_off[(size_t)p + 1] - H.rows_off[(size_t)p];
    it.rows_sorted = P.rows_sorted ? P.rows_sorted + H.rows_off[(size_t)p] : nullptr;
    return it;
}

void collect_profile(gnn_ctx* c)
{
    for (int i = 0; i < GNN_K_COUNT; ++i) { c->prof_ms[i] = 0; c->prof_launches[i] = 0; }
    for (size_t i = 0; i + 1 < c->events_used; i += 2) {
        int cls = c->event_class[i];
        float ms = 0.f;
        if (cls >= 0 && cls < GNN_K_COUNT &&
            hipEventElapsedTime(&ms, c->events[i], c->events[i + 1]) == hipSuccess) {
            c->prof_ms[cls] += ms;
            c->prof_launches[cls] += 1;
        }
    }
    c->events_used = 0;
}

void zero_weight_grads(gnn_ctx* c, hipStream_t s)
{
    Timed t(c, s, GNN_K_OTHER);
    for (int32_t l = 0; l < c->L; ++l) {
        const int64_t wsz = (int64_t)c->dims[(size_t)l] * c->dims[(size_t)l + 1] * 4;
        launch_fill_zero(c->gw[(size_t)3 * l], wsz, s);
        if (c->model == GNN_SAGE_MEAN) launch_fill_zero(c->gw[(size_t)3 * l + 1], wsz, s);
        if (c->model == GNN_GAT) launch_fill_zero(c->gw[(size_t)3 * l + 1], (int64_t)2 * c->dims[(size_t)l + 1] * 4, s);
        if (c->has_bias) launch_fill_zero(c->gw[(size_t)3 * l + 2], (int64_t)c->dims[(size_t)l + 1] * 4, s);
    }
}

static inline uint64_t splitmix64(uint64_t x)
{
    uint64_t z = x + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Dropout after the activation of hidden layer `layer` on `rows` output rows starting at library
// row r0 (nothing when the rate is zero or the layer is the output layer).
void apply_dropout(gnn_ctx* c, int32_t layer, int64_t r0, int64_t rows, void* out_own, int is_bf16, hipStream_t s)
{
    if (!(c->dropout_p > 0.f) || layer >= c->L) return;
    const uint64_t key = splitmix64(c->dropout_seed ^ splitmix64((uint64_t)(64 * c->dropout_epoch + layer)));
    const uint32_t threshold = (uint32_t)std::floor((double)c->dropout_p * 4294967296.0);
    launch_dropout(out_own, is_bf16, c->D.order + r0, rows, c->dims[(size_t)layer], key, threshold,
                   1.f / (1.f - c->dropout_p), s);
}

void compute_fwd(gnn_ctx* c, int32_t layer, int32_t p, const char* in_own, char* out_own, hipStream_t s)
{
    const HostMeta& M = c->M;
    const int64_t np = M.off[(size_t)p + 1] - M.off[(size_t)p];
    const int32_t din = c->dims[(size_t)layer - 1], dout = c->dims[(size_t)layer];
    if (!c->bf16()) {
        // aggregate and transform in one kernel, the aggregated rows staying in LDS
        const SpmmItems items = plan_items(M.plan_fwd, c->D.fwd, p);
        if (!c->gather_fused() && spmm_gemm_fused_ok(din, dout, items)) {
            const int64_t r0 = M.off[(size_t)p];
            const bool sage = c->model == GNN_SAGE_MEAN;
            const float* rscale = c->D.rscale ? c->D.rscale + r0 : nullptr;
            float* zlong = (float*)(c->scratch + c->z_off());
            auto stage = [&](int st) {
                launch_spmm_gemm_fused(c->D.rp + r0, c->D.lcol, c->D.ew, rscale,
                                       (const float*)in_own, np, (const float*)c->staging, din, items,
                                       (float*)(c->scratch + c->ws.segpart), zlong,
                                       sage ? (const float*)in_own : nullptr, (const float*)c->w[(size_t)3 * (layer - 1)],
                                       sage ? (const float*)c->w[(size_t)3 * (layer - 1) + 1] : nullptr,
                                       c->has_bias ? (const float*)c->w[(size_t)3 * (layer - 1) + 2] : nullptr,
                                       layer < c->L ? 1 : 0, (float*)out_own, dout, st, s);
            };
            {
                Timed t(c, s, GNN_K_SPMM);
                stage(0);
            }
            if (items.nlong > 0) {
                Timed t(c, s, GNN_K_SPMM_REDUCE);
                stage(1);
                stage(2);
            }
            if (c->fwd_side)      // this region of Z is free again once the kernels above have run
                if (hipEventRecord(c->side_events[c->side_events.size() - 2 + (size_t)c->z_slot], s) != hipSuccess)
                    c->deferred = hipErrorUnknown;
            if (c->dropout_p > 0.f && layer < c->L) {
                const uint64_t key = splitmix64(c->dropout_seed ^ splitmix64((uint64_t)(64 * c->dropout_epoch + layer)));
                const uint32_t threshold = (uint32_t)std::floor((double)c->dropout_p * 4294967296.0);
                launch_dropout(out_own, 0, c->D.order + r0, np, dout, key, threshold, 1.f / (1.f - c->dropout_p), s);
            }
            return;
        }
    }
    run_spmm_fwd(c, layer, p, in_own, s);
    if (c->keeps_z(layer)) c->z_done[(size_t)(layer - 1) * (size_t)c->M.k + (size_t)p] = 1;
    if (c->fwd_side) {
        // gnn_epoch, resident: the contraction (and the dropout behind it) goes to the side stream
        // once Z is complete, and the caller's stream moves on to the next partition's gather
        hipEvent_t ready = c->side_events[c->side_events.size() - 3];
        hipError_t e = hipEventRecord(ready, s);
        if (e == hipSuccess) e = hipStreamWaitEvent(c->fwd_side, ready, 0);
        if (e != hipSuccess) {
            // without the dependency the contraction must not leave this stream: report the
            // failure (check_launch picks it up) and stay on the caller's stream
            c->deferred = e;
        } else {
            s = c->fwd_side;
        }
    }
    struct Release {        // the Z region is free again when everything launched below has run
        gnn_ctx* c; hipStream_t s;
        ~Release()
        {
            if (c->fwd_side) {
                hipError_t e = hipEventRecord(c->side_events[c->side_events.size() - 2 + (size_t)c->z_slot], s);
                if (e != hipSuccess && c->deferred == hipSuccess) c->deferred = e;
            }
        }
    } release{c, s};
    Timed t(c, s, GNN_K_GEMM_FWD);
    GemmEpilogue ep;
    ep.bias = c->has_bias ? (const float*)c->w[(size_t)3 * (layer - 1) + 2] : nullptr;
    ep.relu = layer < c->L ? 1 : 0;
    const bool sage = c->model == GNN_SAGE_MEAN;
    if (!c->bf16()) {
        GemmSeg seg[2];
        seg[0].a = (const float*)c->z_region(layer, p); seg[0].lda = din;
        seg[0].b = (const float*)c->w[(size_t)3 * (layer - 1)]; seg[0].ldb = dout; seg[0].k = din;
        if (sage) {
            seg[1].a = (const float*)in_own; seg[1].lda = din;
            seg[1].b = (const float*)c->w[(size_t)3 * (layer - 1) + 1]; seg[1].ldb = dout; seg[1].k = din;
        }
        launch_gemm_nn(seg, sage ? 2 : 1, (float*)out_own, dout, np, dout, ep, s);
    } else {
        GemmSegBf16 seg[2];
        seg[0].a = c->z_region(layer, p); seg[0].lda = din;
        seg[0].b = c->w[(size_t)3 * (layer - 1)]; seg[0].ldb = dout; seg[0].k = din;
        if (sage) {
            seg[1].a = in_own; seg[1].lda = din;
            seg[1].b = c->w[(size_t)3 * (layer - 1) + 1]; seg[1].ldb = dout; seg[1].k = din;
        }
        launch_gemm_bf16_nn(seg, sage ? 2 : 1, out_own, layer < c->L ? 1 : 0 /* logits stay fp32 */, dout,
                            np, dout, ep, s, c->scratch + c->ws.wt);
    }
    if (c->dropout_p > 0.f && layer < c->L) {
        const uint64_t key = splitmix64(c->dropout_seed ^ splitmix64((uint64_t)(64 * c->dropout_epoch + layer)));
        const uint32_t threshold = (uint32_t)std::floor((double)c->dropout_p * 4294967296.0);
        launch_dropout(out_own, c->bf16() ? 1 : 0, c->D.order + M.off[(size_t)p], np, dout, key, threshold,
                       1.f / (1.f - c->dropout_p), s);
    }
}

// The transposed operator of partition p as the aggregation kernels take it, with every result
// row added onto its owner's row of a whole-graph array: the full operator (rows = R_p), or, for
// the output layer with gnn_set_masked_backward, its entries at train vertices only.
struct TransposedOp {
    const int64_t* rp;
    const int32_t* col;
    const float* w;
    int64_t nrows;
    SpmmItems items;
    SpmmScatter sc;
};
static TransposedOp transposed_op(gnn_ctx* c, int32_t layer, int32_t p)
{
    const HostMeta& M = c->M;
    TransposedOp op;
    if (layer == c->L && c->masked_transpose()) {
        const HostMeta::MaskedTranspose& T = M.masked_t;
        const int64_t t0 = T.toff[(size_t)p];
        op.rp = c->D.masked_t.trp + t0;
        op.col = c->D.masked_t.tcol;
        op.w = c->D.masked_t.tw;
        op.nrows = T.toff[(size_t)p + 1] - t0;
        op.items = plan_items(T.plan, c->D.masked_t.plan, p);
        op.items.avg_len = (float)(T.trp[(size_t)(t0 + op.nrows)] - T.trp[(size_t)t0]) / (float)std::max<int64_t>(1, op.nrows);
        op.sc.n_own = 0;                       // every kept row names its owner
        op.sc.base_row = 0;
        op.sc.idx = c->D.masked_t.out_row + t0;
        return op;
    }
    const int64_t r0 = M.off[(size_t)p], np = M.off[(size_t)p + 1] - r0;
    const int64_t nb = M.boff[(size_t)p + 1] - M.boff[(size_t)p];
    const int64_t t0 = M.toff[(size_t)p];
    op.rp = c->D.trp + t0;
    op.col = c->D.tcol;
    op.w = c->D.tw;
    op.nrows = np + nb;
    op.items = plan_items(M.plan_bwd, c->D.bwd, p);
    op.items.avg_len = (float)(M.trp[(size_t)M.toff[(size_t)p + 1]] - M.trp[(size_t)t0]) / (float)std::max<int64_t>(1, np + nb);
    op.sc.n_own = np;
    op.sc.base_row = r0;
    op.sc.idx = c->D.bnd + M.boff[(size_t)p];
    if (c->first_touch && c->D.first) op.sc.first = c->D.first + M.first_off[(size_t)p];
    return op;
}

const char* compute_bwd(gnn_ctx* c, int32_t layer, int32_t p, const char* in_own, const float* g_own,
                        const char* act_own, float* fused_gprev, const SpmmScatter* fused_map, hipStream_t s)
{
    const HostMeta& M = c->M;
    const int32_t L = c->L;
    const int64_t np = M.off[(size_t)p + 1] - M.off[(size_t)p];
    const int64_t nb = M.boff[(size_t)p + 1] - M.boff[(size_t)p];
    const int32_t din = c->dims[(size_t)layer - 1], dout = c->dims[(size_t)layer];
    const char* W = c->w[(size_t)3 * (layer - 1)];
    float* gW = c->gw[(size_t)3 * (layer - 1)];
    float* gWs = c->gw[(size_t)3 * (layer - 1) + 1];
    float* gb = c->has_bias ? c->gw[(size_t)3 * (layer - 1) + 2] : nullptr;
    char* Z = c->z_region(layer, p);
    char* dYbuf = c->scratch + c->ws.dy;
    char* dZ = c->scratch + c->ws.dz;
    float* dGA = (float*)(c->scratch + c->ws.dga);
    float* partial = (float*)(c->scratch + c->ws.partial);
    float* colpart = (float*)(c->scratch + c->ws.colpart);
    const bool b16 = c->bf16();
    const bool sage = c->model == GNN_SAGE_MEAN;

    // activation backward: dY = grad A ⊙ [A > 0] on hidden layers, grad A itself on the last
    const char* dY = (const char*)g_own;
    const float drop_scale = c->dropout_p > 0.f ? 1.f / (1.f - c->dropout_p) : 1.f;
    {
        Timed t(c, s, GNN_K_ACT_BWD);
        if (b16) {
            launch_act_bwd_bf16(g_own, layer < L ? act_own : nullptr, dYbuf, np, dout, gb, colpart,
                                drop_scale, s);
            dY = dYbuf;
        } else if (layer < L) {
            launch_act_bwd(g_own, (const float*)act_own, (float*)dYbuf, np, dout, gb, colpart, drop_scale, s);
            dY = dYbuf;
        } else {
            // output layer: grad A^L is the loss kernel's, zero outside the train mask
            launch_act_bwd(g_own, nullptr, nullptr, np, dout, gb, colpart, 1.f, s,
                           c->streaming() ? nullptr : c->mask + M.off[(size_t)p]);
        }
    }
    // recompute the aggregate from the regathered rows (unless the forward pass's is kept)
    if (!(c->keeps_z(layer) && c->z_done[(size_t)(layer - 1) * (size_t)M.k + (size_t)p]))
        run_spmm_fwd(c, layer, p, in_own, s);
    // weight gradients, summed over partitions
    {
        Timed t(c, s, GNN_K_GEMM_DW);
        if (b16) {
            launch_gemm_bf16_tn(Z, din, dY, dout, gW, dout, din, dout, np, partial, s);
            if (sage) launch_gemm_bf16_tn(in_own, din, dY, dout, gWs, dout, din, dout, np, partial, s);
        } else {
            launch_gemm_tn((const float*)Z, din, (const float*)dY, dout, gW, dout, din, dout, np, partial, s);
            if (sage)
                launch_gemm_tn((const float*)in_own, din, (const float*)dY, dout, gWs, dout, din, dout, np,
                               partial, s);
        }
    }
    if (layer >= 2) {
        {
            Timed t(c, s, GNN_K_GEMM_DZ);
            GemmEpilogue ep;
            if (b16) launch_gemm_bf16_nt(dY, dout, W, dout, dZ, 1, din, np, din, dout, ep, s);
            else launch_gemm_nt((const float*)dY, dout, (const float*)W, dout, (float*)dZ, din, np, din, dout, ep, s);
        }
        float* segpart = (float*)(c->scratch + c->ws.segpart);
        // With fused_gprev the transposed aggregation adds each row of the gathered-row gradient
        // straight onto its owner row of grad A^{l-1} (own rows in place, boundary rows through
        // B_p) instead of writing it to scratch for a separate scatter-add pass.
        TransposedOp op = transposed_op(c, fused_gprev && !fused_map ? layer : 0, p);
        float* out = fused_gprev;
        if (!fused_gprev) {
            op.sc = SpmmScatter{};
            out = dGA;
        } else if (fused_map) {
            op.sc = *fused_map;                  // another row numbering of the same owners
        }
        {
            Timed t(c, s, GNN_K_SPMM_T);
            launch_spmm(op.rp, op.col, op.w, nullptr, dZ, np, nullptr, out, op.nrows, din,
                        b16 ? 1 : 0, 0, op.items, segpart, 0, op.sc, s);
        }
        if (op.items.nlong > 0) {
            Timed t(c, s, GNN_K_SPMM_REDUCE);
            launch_spmm_reduce(nullptr, out, din, 0, op.items, segpart, op.sc, s);
        }
    }
    return dY;
}

void compute_bwd_self(gnn_ctx* c, int32_t layer, int32_t p, const char* dY, float* gprev_own,
                      hipStream_t s, int accumulate)
{
    if (c->model != GNN_SAGE_MEAN || layer < 2) return;
    const int64_t np = c->M.off[(size_t)p + 1] - c->M.off[(size_t)p];
    const int32_t din = c->dims[(size_t)layer - 1], dout = c->dims[(size_t)layer];
    const char* Ws = c->w[(size_t)3 * (layer - 1) + 1];
    Timed t(c, s, GNN_K_GEMM_DZ);
    GemmEpilogue ep;
    ep.accumulate = accumulate;
    if (c->bf16()) launch_gemm_bf16_nt(dY, dout, Ws, dout, gprev_own, 0, din, np, din, dout, ep, s);
    else launch_gemm_nt((const float*)dY, dout, (const float*)Ws, dout, gprev_own, din, np, din, dout, ep, s);
}


static int32_t all_done(const std::vector<uint8_t>& flags, int32_t layer, int32_t k)
{
    int32_t cnt = 0;
    for (int32_t q = 0; q < k; ++q) cnt += flags[(size_t)(layer - 1) * (size_t)k + (size_t)q] ? 1 : 0;
    return cnt;
}

// Rows of W (which = 0) or W_s (which = 1) of a transform-first layer padded to the layer's
// padded width, so that every operand of its contractions has 16-byte rows; the weights
// themselves when no padding is needed.
struct PaddedW {
    const float* p;
    int32_t ld;
};
static PaddedW padded_weight(gnn_ctx* c, int32_t layer, int which)
{
    const int32_t din = c->dims[(size_t)layer - 1], dout = c->dims[(size_t)layer], dp = c->padded(layer);
    const float* w = (const float*)c->w[(size_t)3 * (layer - 1) + which];
    if (dp == dout) return {w, dout};
    return {(const float*)(c->scratch + c->ws.wpad) + (int64_t)which * din * dp, dp};
}
static void refresh_padded_weights(gnn_ctx* c, int32_t layer, hipStream_t s)
{
    const int32_t din = c->dims[(size_t)layer - 1], dout = c->dims[(size_t)layer], dp = c->padded(layer);
    if (dp == dout) return;
    Timed t(c, s, GNN_K_OTHER);
    float* base = (float*)(c->scratch + c->ws.wpad);
    launch_pad_rows(base, (const float*)c->w[(size_t)3 * (layer - 1)], din, dout, dp, s);
    if (c->model == GNN_SAGE_MEAN)
        launch_pad_rows(base + (int64_t)din * dp, (const float*)c->w[(size_t)3 * (layer - 1) + 1], din, dout, dp, s);
}

// Transform-first layer, forward of partition p after H = A^{l-1} W exists for every vertex:
// Z = S_p [H_own ; staging], A_p^l = act(Z (+ A_p^{l-1} W_s) + b).
void xf_aggregate_fwd(gnn_ctx* c, int32_t layer, int32_t p, const char* in_own, char* out_own, hipStream_t s)
{
    const HostMeta& M = c->M;
    const int64_t r0 = M.off[(size_t)p], np = M.off[(size_t)p + 1] - r0;
    const int32_t din = c->dims[(size_t)layer - 1], dout = c->dims[(size_t)layer], dp = c->padded(layer);
    SpmmItems items = plan_items(M.plan_fwd, c->D.fwd, p);
    items.avg_len = (float)(M.rp[(size_t)M.off[(size_t)p + 1]] - M.rp[(size_t)r0]) / (float)std::max<int64_t>(1, np);
    const float* rscale = c->D.rscale ? c->D.rscale + r0 : nullptr;
    float* Z = (float*)(c->scratch + c->ws.z);
    float* segpart = (float*)(c->scratch + c->ws.segpart);
    const bool b16 = c->bf16();        // H and staging hold bfloat16 rows then; Z is fp32 either way
    const char* H = c->hbuf + r0 * dp * c->es();
    float* out = (float*)out_own;
    const float* bias = c->has_bias ? (const float*)c->w[(size_t)3 * (layer - 1) + 2] : nullptr;
    const int relu = layer < c->L ? 1 : 0;
    // Without a self term and without padding the aggregation finishes the layer itself: bias and
    // activation are applied where a row's sum is stored, in the storage type of the output rows
    const bool direct = c->model != GNN_SAGE_MEAN && dp == dout;
    SpmmScatter fin;
    if (direct) {
        fin.bias = bias;
        fin.relu = relu;
    }
    void* agg_out = direct ? (void*)out_own : (void*)Z;
    const int agg_out_bf16 = direct && b16 && layer < c->L ? 1 : 0;
    {
        Timed t(c, s, GNN_K_SPMM);
        if (c->gather_fused())
            launch_spmm(c->D.rp + r0, c->D.gcol, c->D.ew, rscale, c->hbuf, M.n, nullptr, agg_out, np, dp,
                        b16 ? 1 : 0, agg_out_bf16, items, segpart, 1, fin, s);
        else
            launch_spmm(c->D.rp + r0, c->D.lcol, c->D.ew, rscale, H, np, c->staging, agg_out, np, dp, b16 ? 1 : 0,
                        agg_out_bf16, items, segpart, 1, fin, s);
    }
    if (items.nlong > 0) {
        Timed t(c, s, GNN_K_SPMM_REDUCE);
        launch_spmm_reduce(rscale, agg_out, dp, agg_out_bf16, items, segpart, fin, s);
    }
    if (direct) {
        // nothing left to do
    } else if (c->model == GNN_SAGE_MEAN) {
        {
            Timed t(c, s, GNN_K_GEMM_FWD);
            GemmEpilogue ep;
            ep.bias = bias;
            if (b16) {
                GemmSegBf16 seg;
                seg.a = in_own; seg.lda = din;
                seg.b = c->w[(size_t)3 * (layer - 1) + 1]; seg.ldb = dout; seg.k = din;
                launch_gemm_bf16_nn(&seg, 1, out, 0, dout, np, dout, ep, s);
            } else {
                const PaddedW ws = padded_weight(c, layer, 1);
                GemmSeg seg;
                seg.a = (const float*)in_own; seg.lda = din;
                seg.b = ws.p; seg.ldb = ws.ld; seg.k = din;
                launch_gemm_nn(&seg, 1, out, dout, np, dout, ep, s);
            }
        }
        Timed t(c, s, GNN_K_OTHER);
        launch_add_padded(out, Z, np, dout, dp, nullptr, 1, relu, s);
    } else if (b16 && layer < c->L) {
        // hidden layer with bfloat16 storage: the output rows are rounded once, here
        Timed t(c, s, GNN_K_OTHER);
        launch_bias_act_bf16(out_own, Z, np, dout, dp, bias, relu, s);
    } else {
        Timed t(c, s, GNN_K_OTHER);
        launch_add_padded(out, Z, np, dout, dp, bias, 0, relu, s);
    }
    if (c->dropout_p > 0.f && layer < c->L) {
        const uint64_t key = splitmix64(c->dropout_seed ^ splitmix64((uint64_t)(64 * c->dropout_epoch + layer)));
        const uint32_t threshold = (uint32_t)std::floor((double)c->dropout_p * 4294967296.0);
        launch_dropout(out_own, b16 ? 1 : 0,
                       c->D.order + r0, np, dout, key, threshold, 1.f / (1.f - c->dropout_p), s);
    }
}

// Transform-first layer, backward of partition p: dY_p, bias and self-weight gradients, and
// grad H [R_p] += S_p^T dY_p (the scatter-accumulate happens at the layer's output width).
// in_own: A_p^{l-1} (GraphSAGE only), g_own: grad A_p^l, act_own: A_p^l (hidden layers),
// gprev_own: grad A_p^{l-1} (only where the self term is written in this sweep).
void xf_aggregate_bwd(gnn_ctx* c, int32_t layer, int32_t p, const char* in_own_c, const float* g_own,
                      const char* act_own, float* gprev_own, hipStream_t s)
{
    const HostMeta& M = c->M;
    const int32_t L = c->L;
    const int64_t r0 = M.off[(size_t)p], np = M.off[(size_t)p + 1] - r0;
    const int64_t nb = M.boff[(size_t)p + 1] - M.boff[(size_t)p];
    const int32_t din = c->dims[(size_t)layer - 1], dout = c->dims[(size_t)layer], dp = c->padded(layer);
    float* gb = c->has_bias ? c->gw[(size_t)3 * (layer - 1) + 2] : nullptr;
    float* dYbuf = (float*)(c->scratch + c->ws.dy);
    float* colpart = (float*)(c->scratch + c->ws.colpart);
    const float drop_scale = c->dropout_p > 0.f ? 1.f / (1.f - c->dropout_p) : 1.f;
    if (c->bf16()) {
        // output layer with bfloat16 storage (dp == dout): dY as bfloat16, the rest as below
        {
            Timed t(c, s, GNN_K_ACT_BWD);
            launch_act_bwd_bf16(g_own, layer < L ? act_own : nullptr, dYbuf, np, dout, gb, colpart,
                                layer < L ? drop_scale : 1.f, s);
        }
        if (c->model == GNN_SAGE_MEAN) {
            {
                Timed t(c, s, GNN_K_GEMM_DW);
                launch_gemm_bf16_tn(in_own_c, din, dYbuf, dout, c->gw[(size_t)3 * (layer - 1) + 1],
                                    dout, din, dout, np, (float*)(c->scratch + c->ws.partial), s);
            }
            if (layer >= 2)
                // (the first thing written to these rows of grad A^{l-1})
                compute_bwd_self(c, layer, p, (const char*)dYbuf, gprev_own, s, 0);
        }
        const TransposedOp opb = transposed_op(c, layer, p);
        float* segb = (float*)(c->scratch + c->ws.segpart);
        float* gHb = (float*)c->ghbuf;
        {
            Timed t(c, s, GNN_K_SPMM_T);
            launch_spmm(opb.rp, opb.col, opb.w, nullptr, dYbuf, np, nullptr, gHb, opb.nrows, dp, 1, 0, opb.items,
                        segb, 0, opb.sc, s);
        }
        if (opb.items.nlong > 0) {
            Timed t(c, s, GNN_K_SPMM_REDUCE);
            launch_spmm_reduce(nullptr, gHb, dp, 0, opb.items, segb, opb.sc, s);
        }
        return;
    }
    // a hidden GraphSAGE layer keeps its (padded) dY rows for the second sweep
    float* keep = c->model == GNN_SAGE_MEAN && layer >= 2 && layer < L && c->dyall_buf
                      ? c->dyall_buf + r0 * dp : nullptr;
    if (keep && dp == dout) dYbuf = keep;
    const float* dY = g_own;
    {
        Timed t(c, s, GNN_K_ACT_BWD);
        if (layer < L) {
            launch_act_bwd(g_own, (const float*)act_own, dYbuf, np, dout, gb,
                           colpart, drop_scale, s);
            dY = dYbuf;
        } else {
            // output layer: grad A^L is the loss kernel's, zero outside the train mask
            launch_act_bwd(g_own, nullptr, nullptr, np, dout, gb, colpart, 1.f, s,
                           c->streaming() ? nullptr : c->mask + r0);
        }
    }
    const float* in_own = (const float*)in_own_c;
    // dY with rows padded to whole vectors (zeros in the padding): the operand of everything below
    const float* dYp = dY;
    if (dp != dout) {
        Timed t(c, s, GNN_K_OTHER);
        float* pad = keep ? keep : (float*)(c->scratch + c->ws.dz);
        launch_pad_rows(pad, dY, np, dout, dp, s);
        dYp = pad;
    }
    if (c->model == GNN_SAGE_MEAN) {
        {
            Timed t(c, s, GNN_K_GEMM_DW);
            launch_gemm_tn(in_own, din, dYp, dp, c->gw[(size_t)3 * (layer - 1) + 1], dout, din, dout, np,
                           (float*)(c->scratch + c->ws.partial), s);
        }
        if (layer >= 2 && layer < L && !keep && gprev_own) {
            // self term: grad A^{l-1}_own = dY W_s^T (the first thing written to these rows),
            // contracted over the padded width.  (Not reached while the workspace keeps dY of every
            // partition: then the second sweep takes both terms of grad A^{l-1} in one contraction,
            // as the output layer does with dY = grad A^L.)
            const PaddedW ws = padded_weight(c, layer, 1);
            Timed t(c, s, GNN_K_GEMM_DZ);
            GemmEpilogue ep;
            launch_gemm_nt(dYp, dp, ws.p, ws.ld, gprev_own, din, np, din, dp, ep, s);
        }
    }
    const TransposedOp op = transposed_op(c, layer, p);
    float* segpart = (float*)(c->scratch + c->ws.segpart);
    float* gH = (float*)c->ghbuf;
    {
        Timed t(c, s, GNN_K_SPMM_T);
        launch_spmm(op.rp, op.col, op.w, nullptr, dYp, np, nullptr, gH, op.nrows, dp, 0, 0, op.items,
                    segpart, 0, op.sc, s);
    }
    if (op.items.nlong > 0) {
        Timed t(c, s, GNN_K_SPMM_REDUCE);
        launch_spmm_reduce(nullptr, gH, dp, 0, op.items, segpart, op.sc, s);
    }
}

// Transform-first layer, first sweep of the forward pass: H_p = A_p^{l-1} W (rows of partition p
// of the whole-graph buffer H).
void xf_transform_fwd(gnn_ctx* c, int32_t layer, int32_t p, const char* in_own, hipStream_t s)
{
    const HostMeta& M = c->M;
    const int64_t r0 = M.off[(size_t)p], np = M.off[(size_t)p + 1] - r0;
    const int32_t din = c->dims[(size_t)layer - 1], dout = c->dims[(size_t)layer], dp = c->padded(layer);
    if (c->bf16()) {
        // bfloat16 storage (dp == dout): H in bfloat16
        Timed t(c, s, GNN_K_GEMM_FWD);
        GemmSegBf16 seg;
        seg.a = in_own; seg.lda = din;
        seg.b = c->w[(size_t)3 * (layer - 1)]; seg.ldb = dout; seg.k = din;
        launch_gemm_bf16_nn(&seg, 1, c->hbuf + r0 * dp * 2, 1, dp, np, dout, GemmEpilogue{}, s,
                            c->scratch + c->ws.wt);
        return;
    }
    float* H = (float*)c->hbuf + r0 * dp;
    refresh_padded_weights(c, layer, s);
    // all dp columns are computed: the padding columns of W are zero, so are those of H
    const PaddedW w = padded_weight(c, layer, 0);
    Timed t(c, s, GNN_K_GEMM_FWD);
    GemmSeg seg;
    seg.a = (const float*)in_own; seg.lda = din;
    seg.b = w.p; seg.ldb = w.ld; seg.k = din;
    launch_gemm_nn(&seg, 1, H, dp, np, w.ld == dp ? dp : dout, GemmEpilogue{}, s);
}

// Transform-first layer, second sweep of the backward pass, once grad H is complete:
// grad W += A_p^{l-1 T} grad H_p, grad A_p^{l-1} = grad H_p W^T (+ dY_p W_s^T).  g_own = grad A_p^l
// (read by a GraphSAGE output layer, whose dY is grad A^L itself).  act_own = A_p^l: given for a
// hidden GraphSAGE layer when the first sweep kept no dY rows (streaming schedule); dY_p is then
// taken again from g_own and act_own, the same values, and enters the same contraction.
void xf_transform_bwd(gnn_ctx* c, int32_t layer, int32_t p, const char* in_own_c, const float* g_own,
                      const char* act_own, float* gprev_own, hipStream_t s)
{
    const HostMeta& M = c->M;
    const int64_t r0 = M.off[(size_t)p], np = M.off[(size_t)p + 1] - r0;
    const int32_t din = c->dims[(size_t)layer - 1], dout = c->dims[(size_t)layer], dp = c->padded(layer);
    const float* gH = (const float*)c->ghbuf + r0 * dp;
    if (c->bf16()) {
        // the contractions take bfloat16 operands: grad H of this partition is rounded once
        char* gHb = c->scratch + c->ws.dz;
        {
            Timed t(c, s, GNN_K_OTHER);
            launch_to_bf16(gH, gHb, np * (int64_t)dp, s);
        }
        {
            Timed t(c, s, GNN_K_GEMM_DW);
            launch_gemm_bf16_tn(in_own_c, din, gHb, dp, c->gw[(size_t)3 * (layer - 1)], dout, din,
                                dout, np, (float*)(c->scratch + c->ws.partial), s);
        }
        if (layer >= 2) {
            Timed t(c, s, GNN_K_GEMM_DZ);
            GemmEpilogue ep;
            ep.accumulate = c->model == GNN_SAGE_MEAN ? 1 : 0;    // SAGE: the self term is there already
            launch_gemm_bf16_nt(gHb, dp, c->w[(size_t)3 * (layer - 1)], dout, gprev_own, 0,
                                din, np, din, dout, ep, s);
        }
        return;
    }
    const float* in_own = (const float*)in_own_c;
    {
        Timed t(c, s, GNN_K_GEMM_DW);
        launch_gemm_tn(in_own, din, gH, dp, c->gw[(size_t)3 * (layer - 1)], dout, din, dout, np,
                       (float*)(c->scratch + (c->on_side ? c->ws.partial2 : c->ws.partial)), s);
    }
    const float* dYk = nullptr;          // padded dY_p of a hidden GraphSAGE layer
    if (c->model == GNN_SAGE_MEAN && layer >= 2 && layer < c->L) {
        if (c->dyall_buf) {
            dYk = c->dyall_buf + r0 * dp;
        } else if (act_own) {
            float* dyb = (float*)(c->scratch + c->ws.dy);
            {
                Timed t(c, s, GNN_K_ACT_BWD);
                launch_act_bwd(g_own, (const float*)act_own, dyb, np, dout, nullptr, (float*)(c->scratch + c->ws.colpart),
                               c->dropout_p > 0.f ? 1.f / (1.f - c->dropout_p) : 1.f, s);
            }
            dYk = dyb;
            if (dp != dout) {
                Timed t(c, s, GNN_K_OTHER);
                float* pad = (float*)(c->scratch + c->ws.dz);
                launch_pad_rows(pad, dyb, np, dout, dp, s);
                dYk = pad;
            }
        }
    }
    const bool kept = dYk != nullptr;
    if (layer >= 2 && (layer == c->L || kept) && c->model == GNN_SAGE_MEAN) {
        // grad A^{l-1}_own = grad H_p W^T + dY_p W_s^T in one pass over the result: the output
        // layer's dY_p is grad A^L_p, a hidden layer's padded dY_p was kept by the first sweep
        const float* dY = kept ? dYk : g_own;
        if (!kept && dp != dout) {
            Timed t(c, s, GNN_K_OTHER);
            float* pad = (float*)(c->scratch + c->ws.dz);
            launch_pad_rows(pad, dY, np, dout, dp, s);
            dY = pad;
        }
        const PaddedW w = padded_weight(c, layer, 0), ws = padded_weight(c, layer, 1);
        Timed t(c, s, GNN_K_GEMM_DZ);
        GemmSeg seg[2];
        seg[0].a = gH; seg[0].lda = dp; seg[0].b = w.p; seg[0].ldb = w.ld; seg[0].k = dp;
        seg[1].a = dY; seg[1].lda = dp; seg[1].b = ws.p; seg[1].ldb = ws.ld; seg[1].k = dp;
        launch_gemm_nt2(seg, 2, gprev_own, din, np, din, GemmEpilogue{}, s);
    } else if (layer >= 2) {
        const PaddedW w = padded_weight(c, layer, 0);
        Timed t(c, s, GNN_K_GEMM_DZ);
        GemmEpilogue ep;
        ep.accumulate = c->model == GNN_SAGE_MEAN ? 1 : 0;    // SAGE: the self term is there already
        launch_gemm_nt(gH, dp, w.p, w.ld, gprev_own, din, np, din, dp, ep, s);
    }
}

// Start of a transform-first layer's backward pass: grad H := 0 (it takes the buffer H was in).
void xf_begin_bwd(gnn_ctx* c, int32_t layer, hipStream_t s)
{
    // (an epoch that lets first-touch rows store has nothing to zero, unless the operator is the
    // output layer's over train vertices, which does not reach every row)
    if (!(c->first_touch && c->D.first && !(layer == c->L && c->masked_transpose()))) {
        Timed t(c, s, GNN_K_OTHER);
        launch_fill_zero(c->ghbuf, c->M.n * (int64_t)c->padded(layer) * 4, s);
        // grad A^{l-1} needs no initialisation here: each of its rows is written once (by
        // the self term, else by grad H W^T) before anything is added to it
    }
    refresh_padded_weights(c, layer, s);
}

}  // namespace gnnmi

// =================================================================================================
extern "C" {

gnn_status gnn_create(const gnn_config* cfg, gnn_ctx** out)
{
    auto bad = [&](gnn_status st, const char* m) { g_create_error = m; return st; };
    if (!cfg || !out) return bad(GNN_EINVAL, "cfg and out must be non-null");
    *out = nullptr;
    if (cfg->model != GNN_GCN && cfg->model != GNN_SAGE_MEAN && cfg->model != GNN_GAT)
        return bad(GNN_EINVAL, "unknown model");
    if (cfg->model == GNN_GAT && (cfg->dtype != GNN_F32 || cfg->hbm_budget_bytes != 0))
        return bad(GNN_EUNSUPPORTED, "graph-attention layers are built for GNN_F32 and the resident schedule");
    if (cfg->dtype != GNN_F32 && cfg->dtype != GNN_BF16) return bad(GNN_EINVAL, "unknown dtype");
    if (cfg->n_layers < 1 || cfg->n_layers > 64) return bad(GNN_EINVAL, "n_layers must be in 1..64");
    if (!cfg->dims) return bad(GNN_EINVAL, "dims is null");
    for (int32_t l = 0; l <= cfg->n_layers; ++l)
        if (cfg->dims[l] < 1 || cfg->dims[l] > (1 << 20)) return bad(GNN_EINVAL, "layer width out of range");
    if (cfg->has_bias != 0 && cfg->has_bias != 1) return bad(GNN_EINVAL, "has_bias must be 0 or 1");
    if (cfg->hbm_budget_bytes < 0) return bad(GNN_EINVAL, "hbm_budget_bytes must be >= 0");
    gnn_ctx* c = new (std::nothrow) gnn_ctx();
    if (!c) return bad(GNN_ENOMEM, "out of host memory");
    c->model = cfg->model;
    c->dtype = cfg->dtype;
    c->L = cfg->n_layers;
    c->has_bias = cfg->has_bias;
    c->hbm_budget = cfg->hbm_budget_bytes;
    c->dims.assign(cfg->dims, cfg->dims + cfg->n_layers + 1);
    *out = c;
    return GNN_OK;
}

void gnn_destroy(gnn_ctx* c)
{
    if (!c) return;
    stream_engine_destroy(c);
    tier_close(c);
    if (c->D.ready) free_device(c->D);
    for (hipEvent_t e : c->events) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->side_events) (void)hipEventDestroy(e);
    if (c->side) (void)hipStreamDestroy(c->side);
    delete c;
}

const char* gnn_last_error(const gnn_ctx* c) { return c ? c->err.c_str() : g_create_error.c_str(); }

gnn_status gnn_build_partitions(gnn_ctx* c, int64_t n, const int64_t* rowptr, const int32_t* colidx,
                                int32_t k, int32_t mode, uint64_t seed, const int32_t* user_part)
{
    if (!c) return GNN_EINVAL;
    if (c->streaming() && k > 4096)
        return c->fail(GNN_EINVAL, "the streaming schedule supports at most 4096 partitions");
    gnn_status st;
    try {
        HostMeta M;
        std::string err;
        st = build_host_meta(c->model, n, rowptr, colidx, k, mode, seed, user_part, c->streaming(), M, err);
        if (st != GNN_OK) return c->fail(st, err);
        stream_engine_destroy(c);
        tier_close(c);                 // its arrays were sized for the graph before
        if (c->D.ready) free_device(c->D);
        c->M = std::move(M);
    } catch (const std::bad_alloc&) {
        return c->fail(GNN_ENOMEM, "out of host memory while building partitions");
    } catch (...) {
        return c->fail(GNN_ENOMEM, "failed to build partitions (could not start worker threads?)");
    }
    c->built = true;
    c->bound = false;
    c->staged_layer = c->staged_p = -1;
    c->loss_done = false;
    c->fwd_done.assign((size_t)c->L * (size_t)k, 0);
    c->xf_fwd_done.assign((size_t)c->L * (size_t)k, 0);
    c->att_done.assign((size_t)c->L * (size_t)k, 0);
    c->z_done.assign((size_t)c->L * (size_t)k, 0);
    c->xf_bwd_done.assign((size_t)c->L * (size_t)k, 0);
    c->bwd_done.assign((size_t)c->L + 2, 0);
    compute_workspace(c);
    return GNN_OK;
}

gnn_status gnn_get_partition(const gnn_ctx* c, const int32_t** part, int32_t* k)
{
    if (!c || !part || !k) return GNN_EINVAL;
    if (!c->built) return c->fail(GNN_ESTATE, "no partitions built");
    *part = c->M.part.data();
    *k = c->M.k;
    return GNN_OK;
}

gnn_status gnn_get_order(const gnn_ctx* c, const int32_t** order, const int64_t** part_offset)
{
    if (!c || !order || !part_offset) return GNN_EINVAL;
    if (!c->built) return c->fail(GNN_ESTATE, "no partitions built");
    *order = c->M.order.data();
    *part_offset = c->M.off.data();
    return GNN_OK;
}

gnn_status gnn_get_boundary(const gnn_ctx* c, int32_t p, const int32_t** idx, int64_t* count)
{
    if (!c || !idx || !count) return GNN_EINVAL;
    if (!c->built) return c->fail(GNN_ESTATE, "no partitions built");
    if (p < 0 || p >= c->M.k) return c->fail(GNN_EINVAL, "partition outside 0..k-1");
    *idx = c->M.bnd_orig.data() + c->M.boff[(size_t)p];
    *count = c->M.boff[(size_t)p + 1] - c->M.boff[(size_t)p];
    return GNN_OK;
}

gnn_status gnn_get_stats(const gnn_ctx* c, gnn_stats* out)
{
    if (!c || !out) return GNN_EINVAL;
    if (!c->built) return c->fail(GNN_ESTATE, "no partitions built");
    *out = c->M.stats;
    return GNN_OK;
}

gnn_status gnn_get_schedule(const gnn_ctx* c, const int32_t** order)
{
    if (!c || !order) return GNN_EINVAL;
    if (!c->built) return c->fail(GNN_ESTATE, "no partitions built");
    *order = c->M.sched.data();
    return GNN_OK;
}

gnn_status gnn_get_partitioner_history(const gnn_ctx* c, int32_t* iterations, double* objective,
                                       int32_t capacity)
{
    if (!c || !iterations || (capacity > 0 && !objective)) return GNN_EINVAL;
    if (!c->built) return c->fail(GNN_ESTATE, "no partitions built");
    *iterations = c->M.part_iterations;
    const int64_t m = std::min<int64_t>(capacity, (int64_t)c->M.part_objective.size());
    for (int64_t i = 0; i < m; ++i) objective[i] = c->M.part_objective[(size_t)i];
    return GNN_OK;
}

gnn_status gnn_workspace_bytes(const gnn_ctx* c, int64_t* staging, int64_t* scratch)
{
    if (!c || !staging || !scratch) return GNN_EINVAL;
    if (!c->built) return c->fail(GNN_ESTATE, "no partitions built");
    *staging = c->ws.staging_bytes;
    *scratch = c->ws.scratch_bytes;
    return GNN_OK;
}

gnn_status gnn_bind(gnn_ctx* c, const void* feat, void* const* act, void* const* grad_act,
                    const void* const* weights, void* const* grad_w, const int32_t* labels,
                    const uint8_t* train_mask, void* staging, void* scratch)
{
    if (!c) return GNN_EINVAL;
    if (!c->built) return c->fail(GNN_ESTATE, "gnn_bind before gnn_build_partitions");
    // with a storage tier the per-vertex arrays are the tier's: feat, act and grad_act are ignored
    const bool tiered = c->tier != nullptr;
    if ((!tiered && (!feat || !act || !grad_act)) || !weights || !grad_w || !labels || !train_mask || !staging ||
        !scratch)
        return c->fail(GNN_EINVAL, "null buffer passed to gnn_bind");
    const int32_t L = c->L;
    for (int32_t l = 0; l < L; ++l) {
        if (!tiered && (!act[l] || !grad_act[l])) return c->fail(GNN_EINVAL, "null activation or gradient buffer");
        if (!weights[3 * l] || !grad_w[3 * l]) return c->fail(GNN_EINVAL, "null weight or weight-gradient buffer");
        if ((c->model == GNN_SAGE_MEAN || c->model == GNN_GAT) && (!weights[3 * l + 1] || !grad_w[3 * l + 1]))
            return c->fail(GNN_EINVAL, "null self-weight (SAGE) or attention-vector (GAT) buffer");
        if (c->has_bias && (!weights[3 * l + 2] || !grad_w[3 * l + 2]))
            return c->fail(GNN_EINVAL, "null bias buffer although has_bias is set");
    }
    // every per-vertex array and every weight matrix is read and written in 16-byte vectors
    uintptr_t bits = reinterpret_cast<uintptr_t>(staging) | reinterpret_cast<uintptr_t>(scratch) |
                     (tiered ? 0 : reinterpret_cast<uintptr_t>(feat));
    for (int32_t l = 0; l < L; ++l) {
        if (!tiered) bits |= reinterpret_cast<uintptr_t>(act[l]) | reinterpret_cast<uintptr_t>(grad_act[l]);
        for (int j = 0; j < 2; ++j)
            bits |= reinterpret_cast<uintptr_t>(weights[3 * l + j]) | reinterpret_cast<uintptr_t>(grad_w[3 * l + j]);
    }
    if (bits & 15)
        return c->fail(GNN_EINVAL, "feat, act[], grad_act[], the weight matrices and their gradients, staging and "
                                   "scratch must be 16-byte aligned");
    gnn_status st = ensure_device(c);
    if (st != GNN_OK) return st;
    if (c->fuse_gather && !c->streaming() && (st = ensure_global_columns(c)) != GNN_OK) return st;
    c->feat = tiered ? nullptr : (const char*)feat;
    c->act.assign((size_t)L, nullptr);
    c->gact.assign((size_t)L, nullptr);
    c->w.assign((size_t)3 * L, nullptr);
    c->gw.assign((size_t)3 * L, nullptr);
    for (int32_t l = 0; l < L; ++l) {
        if (!tiered) {
            c->act[(size_t)l] = (char*)act[l];
            c->gact[(size_t)l] = (float*)grad_act[l];
        }
        for (int j = 0; j < 3; ++j) {
            c->w[(size_t)(3 * l + j)] = (const char*)weights[3 * l + j];
            c->gw[(size_t)(3 * l + j)] = (float*)grad_w[3 * l + j];
        }
    }
    c->labels = labels;
    c->mask = train_mask;
    free_masked(c->D.masked_t);           // belongs to the mask bound before
    if (c->masked_bwd && !c->streaming() && c->model != GNN_GAT && (st = build_masked(c)) != GNN_OK) return st;
    c->staging = (char*)staging;
    c->scratch = (char*)scratch;
    // whole-graph buffers of transform-first layers: in scratch (resident schedule) or given out
    // of the HBM budget by the streaming engine below
    c->hbuf = c->ghbuf = nullptr;
    c->dyall_buf = nullptr;
    if (!c->streaming() && c->ws.h_floats > 0) {
        c->hbuf = c->scratch + c->ws.h;
        c->ghbuf = c->scratch + c->ws.gh;
        if (c->ws.dyall >= 0) c->dyall_buf = (float*)(c->scratch + c->ws.dyall);
    }
    c->staged_layer = c->staged_p = -1;
    c->loss_done = false;
    std::fill(c->fwd_done.begin(), c->fwd_done.end(), 0);
    std::fill(c->xf_fwd_done.begin(), c->xf_fwd_done.end(), 0);
    std::fill(c->att_done.begin(), c->att_done.end(), 0);
    std::fill(c->z_done.begin(), c->z_done.end(), 0);
    std::fill(c->xf_bwd_done.begin(), c->xf_bwd_done.end(), 0);
    std::fill(c->bwd_done.begin(), c->bwd_done.end(), 0);
    c->h_layer = 0;
    if (c->streaming()) {
        st = stream_engine_create(c);
        if (st != GNN_OK) return st;
    }
    c->bound = true;
    return GNN_OK;
}

gnn_status gnn_permute_rows(gnn_ctx* c, const void* src, void* dst, int64_t row_bytes,
                            int32_t to_library_order, void* stream)
{
    if (!c) return GNN_EINVAL;
    if (!c->built) return c->fail(GNN_ESTATE, "no partitions built");
    if (!src || !dst || row_bytes < 1 || src == dst) return c->fail(GNN_EINVAL, "bad permute arguments");
    gnn_status st = ensure_device(c);
    if (st != GNN_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    if (to_library_order) launch_gather_rows(src, c->D.order, dst, c->M.n, row_bytes, s);
    else launch_scatter_rows(src, c->D.order, dst, c->M.n, row_bytes, s);
    return check_launch(c, "gnn_permute_rows");
}

gnn_status gnn_to_bf16(gnn_ctx* c, const float* src, void* dst, int64_t count, void* stream)
{
    if (!c) return GNN_EINVAL;
    if (!src || !dst || count < 0) return c->fail(GNN_EINVAL, "bad gnn_to_bf16 arguments");
    if ((reinterpret_cast<uintptr_t>(src) & 3) || (reinterpret_cast<uintptr_t>(dst) & 1))
        return c->fail(GNN_EINVAL, "gnn_to_bf16: src must be 4-byte and dst 2-byte aligned");
    if (count == 0) return GNN_OK;
    launch_to_bf16(src, dst, count, (hipStream_t)stream);
    return check_launch(c, "gnn_to_bf16");
}

gnn_status gnn_gather_boundary(gnn_ctx* c, int32_t layer, int32_t p, void* stream)
{
    if (!c) return GNN_EINVAL;
    gnn_status st = check_lp(c, layer, p);
    if (st != GNN_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    const HostMeta& M = c->M;
    const int64_t b0 = M.boff[(size_t)p], nb = M.boff[(size_t)p + 1] - b0;
    if (c->transform_first(layer)) {
        // the layer aggregates H = A^{l-1} W: every partition's rows of H must exist
        if (all_done(c->xf_fwd_done, layer, M.k) < M.k)
            return c->fail(GNN_ESTATE, "transform-first layer: gnn_layer_transform_fwd has not covered every partition");
        if (c->model == GNN_GAT) {
            gat_gather(c, layer, p, s);
            c->staged_layer = layer;
            c->staged_p = p;
            return check_launch(c, "gnn_gather_boundary");
        }
        if (!c->gather_fused()) {
            Timed t(c, s, GNN_K_GATHER);
            launch_gather_rows(c->hbuf, c->D.bnd + b0, c->staging, nb, (int64_t)c->padded(layer) * c->es(), s);
        }
    } else if (!c->gather_fused()) {
        const int64_t row_bytes = (int64_t)c->dims[(size_t)layer - 1] * c->es();
        Timed t(c, s, GNN_K_GATHER);
        launch_gather_rows(c->layer_input(layer), c->D.bnd + b0, c->staging, nb, row_bytes, s);
    }
    c->staged_layer = layer;
    c->staged_p = p;
    return check_launch(c, "gnn_gather_boundary");
}

gnn_status gnn_set_gather_fusion(gnn_ctx* c, int32_t on)
{
    if (!c) return GNN_EINVAL;
    if (on != 0 && on != 1) return c->fail(GNN_EINVAL, "gnn_set_gather_fusion takes 0 or 1");
    c->fuse_gather = on == 1;
    c->staged_layer = c->staged_p = -1;       // staging holds nothing the other mode could use
    if (c->fuse_gather && c->D.ready && !c->streaming()) return ensure_global_columns(c);
    return GNN_OK;
}

gnn_status gnn_set_masked_backward(gnn_ctx* c, int32_t on)
{
    if (!c) return GNN_EINVAL;
    if (on != 0 && on != 1) return c->fail(GNN_EINVAL, "gnn_set_masked_backward takes 0 or 1");
    c->masked_bwd = on == 1;
    if (!c->masked_bwd) {
        free_masked(c->D.masked_t);
        return GNN_OK;
    }
    if (c->bound && !c->streaming() && c->model != GNN_GAT && !c->D.masked_t.ready) return build_masked(c);
    return GNN_OK;
}

gnn_status gnn_get_masked_backward_size(const gnn_ctx* c, int64_t* entries, int64_t* rows)
{
    if (!c || !entries || !rows) return GNN_EINVAL;
    *entries = *rows = 0;
    if (c->masked_transpose()) {
        const HostMeta::MaskedTranspose& T = c->M.masked_t;
        *rows = T.toff.back();
        *entries = T.trp.back();
    }
    return GNN_OK;
}

gnn_status gnn_gather_is_fused(const gnn_ctx* c, int32_t* out)
{
    if (!c || !out) return GNN_EINVAL;
    // the index array is set up by gnn_bind at the latest
    *out = c->fuse_gather && !c->streaming() ? 1 : 0;
    return GNN_OK;
}

gnn_status gnn_layer_fwd(gnn_ctx* c, int32_t layer, int32_t p, void* stream)
{
    if (!c) return GNN_EINVAL;
    gnn_status st = check_lp(c, layer, p);
    if (st != GNN_OK) return st;
    if (c->staged_layer != layer || c->staged_p != p)
        return c->fail(GNN_ESTATE, "staging does not hold this (layer, partition); call gnn_gather_boundary first");
    hipStream_t s = (hipStream_t)stream;
    const int64_t r0 = c->M.off[(size_t)p];
    const int32_t dout = c->dims[(size_t)layer];
    if (c->model == GNN_GAT)
        gat_layer_fwd(c, layer, p, s);
    else if (c->transform_first(layer))
        xf_aggregate_fwd(c, layer, p, c->layer_input(layer, r0),
                         c->act[(size_t)layer - 1] + r0 * (int64_t)dout * c->act_es(layer), s);
    else
        compute_fwd(c, layer, p, c->layer_input(layer, r0),
                    c->act[(size_t)layer - 1] + r0 * (int64_t)dout * c->act_es(layer), s);
    c->fwd_done[(size_t)(layer - 1) * (size_t)c->M.k + (size_t)p] = 1;
    return check_launch(c, "gnn_layer_fwd");
}

gnn_status gnn_set_layer_order(gnn_ctx* c, int32_t mode)
{
    if (!c) return GNN_EINVAL;
    if (mode != GNN_ORDER_AGGREGATE_FIRST && mode != GNN_ORDER_AUTO)
        return c->fail(GNN_EINVAL, "unknown layer order");
    c->order_mode = mode;
    c->bound = false;              // workspace sizes depend on the order
    if (c->built) compute_workspace(c);
    return GNN_OK;
}

gnn_status gnn_set_gat_heads(gnn_ctx* c, int32_t layer, int32_t heads)
{
    if (!c) return GNN_EINVAL;
    if (c->model != GNN_GAT) return c->fail(GNN_EINVAL, "attention heads exist for GNN_GAT only");
    if (layer < 1 || layer > c->L) return c->fail(GNN_EINVAL, "layer outside 1..L");
    if (heads < 1 || heads > 64 || c->dims[(size_t)layer] % heads != 0)
        return c->fail(GNN_EINVAL, "the head count must be in 1..64 and divide the layer's output width");
    if (c->heads.empty()) c->heads.assign((size_t)c->L, 1);
    c->heads[(size_t)layer - 1] = heads;
    c->bound = false;              // workspace sizes depend on the head counts
    c->h_layer = 0;
    if (c->built) compute_workspace(c);
    return GNN_OK;
}

gnn_status gnn_set_keep_forward(gnn_ctx* c, int32_t on)
{
    if (!c) return GNN_EINVAL;
    if (on != 0 && on != 1) return c->fail(GNN_EINVAL, "gnn_set_keep_forward takes 0 or 1");
    if (c->keep_forward == (on == 1)) return GNN_OK;
    c->keep_forward = on == 1;
    if (!c->streaming()) {
        c->bound = false;          // workspace sizes depend on it
        c->h_layer = 0;
        if (c->built) compute_workspace(c);
    }
    return GNN_OK;
}

gnn_status gnn_layer_is_transform_first(const gnn_ctx* c, int32_t layer, int32_t* out)
{
    if (!c || !out) return GNN_EINVAL;
    if (layer < 1 || layer > c->L) return c->fail(GNN_EINVAL, "layer outside 1..L");
    *out = c->transform_first(layer) ? 1 : 0;
    return GNN_OK;
}

gnn_status gnn_layer_transform_fwd(gnn_ctx* c, int32_t layer, int32_t p, void* stream)
{
    if (!c) return GNN_EINVAL;
    gnn_status st = check_lp(c, layer, p);
    if (st != GNN_OK) return st;
    if (!c->transform_first(layer)) return c->fail(GNN_ESTATE, "this layer aggregates first");
    hipStream_t s = (hipStream_t)stream;
    const HostMeta& M = c->M;
    const bool kept = c->model == GNN_GAT && c->keep_forward;
    if (c->h_layer != layer) {
        // one buffer holds H for whichever layer is being worked on (attention that keeps its
        // forward results: one per layer)
        if (!kept) std::fill(c->xf_fwd_done.begin(), c->xf_fwd_done.end(), 0);
        c->h_layer = layer;
    }
    if (c->model == GNN_GAT)      // attention weights taken from the old rows of H are void
        std::fill(c->att_done.begin() + (size_t)(layer - 1) * (size_t)M.k,
                  c->att_done.begin() + (size_t)layer * (size_t)M.k, 0);
    if (c->model == GNN_GAT) gat_transform_fwd(c, layer, p, s);
    else xf_transform_fwd(c, layer, p, c->layer_input(layer, M.off[(size_t)p]), s);
    c->xf_fwd_done[(size_t)(layer - 1) * (size_t)M.k + (size_t)p] = 1;
    return check_launch(c, "gnn_layer_transform_fwd");
}

gnn_status gnn_layer_transform_bwd(gnn_ctx* c, int32_t layer, int32_t p, void* stream)
{
    if (!c) return GNN_EINVAL;
    gnn_status st = check_lp(c, layer, p);
    if (st != GNN_OK) return st;
    if (!c->transform_first(layer)) return c->fail(GNN_ESTATE, "this layer aggregates first");
    if (!c->loss_done || c->bwd_done[(size_t)layer] < c->M.k)
        return c->fail(GNN_ESTATE, "gnn_layer_bwd of this layer has not covered every partition");
    hipStream_t s = (hipStream_t)stream;
    const HostMeta& M = c->M;
    if (c->model == GNN_GAT) {
        gat_transform_bwd(c, layer, p, s);
    } else {
        const int64_t r0 = M.off[(size_t)p];
        xf_transform_bwd(c, layer, p, c->layer_input(layer, r0),
                         c->gact[(size_t)layer - 1] + r0 * c->dims[(size_t)layer], nullptr,
                         layer >= 2 ? c->gact[(size_t)layer - 2] + r0 * c->dims[(size_t)layer - 1] : nullptr, s);
    }
    c->xf_bwd_done[(size_t)(layer - 1) * (size_t)M.k + (size_t)p] = 1;
    return check_launch(c, "gnn_layer_transform_bwd");
}

gnn_status gnn_loss(gnn_ctx* c, void* stream)
{
    if (!c) return GNN_EINVAL;
    if (!c->bound) return c->fail(GNN_ESTATE, "buffers are not bound (call gnn_bind)");
    if (c->streaming()) return c->fail(GNN_EUNSUPPORTED, "with a streaming budget only gnn_epoch drives the schedule");
    for (uint8_t f : c->fwd_done)
        if (!f) return c->fail(GNN_ESTATE, "gnn_loss before the forward pass has covered every (layer, partition)");
    hipStream_t s = (hipStream_t)stream;
    float* scal = (float*)(c->scratch + c->ws.scalars);
    {
        Timed t(c, s, GNN_K_LOSS);
        launch_loss((const float*)c->act[(size_t)c->L - 1], c->labels, c->mask, c->gact[(size_t)c->L - 1],
                    c->M.n, c->dims[(size_t)c->L], c->M.off.data(), c->M.k, (unsigned long long*)(scal + 16),
                    (float*)(c->scratch + c->ws.losspart), scal, s);
    }
    c->loss_done = true;
    std::fill(c->bwd_done.begin(), c->bwd_done.end(), 0);
    return check_launch(c, "gnn_loss");
}

gnn_status gnn_loss_static(gnn_ctx* c, void* stream, float* loss_dev)
{
    if (!c || !loss_dev) return GNN_EINVAL;
    if (!c->bound) return c->fail(GNN_ESTATE, "buffers are not bound (call gnn_bind)");
    if (c->streaming()) return c->fail(GNN_EUNSUPPORTED, "with a streaming budget only gnn_epoch drives the schedule");
    for (uint8_t f : c->fwd_done)
        if (!f) return c->fail(GNN_ESTATE, "gnn_loss_static before the forward pass has covered every (layer, partition)");
    if (loss_partial_floats(c->M.n, c->M.k) > loss_static_max_partials())
        return c->fail(GNN_EINVAL, "gnn_loss_static: " + std::to_string(c->M.n) + " vertices in " + std::to_string(c->M.k) +
                                       " partitions need more block partial sums (one per 64 rows of a partition) than "
                                       "the static scratch array holds (" + std::to_string(loss_static_max_partials()) + ")");
    hipStream_t s = (hipStream_t)stream;
    hipError_t e;
    {
        Timed t(c, s, GNN_K_LOSS);
        e = launch_loss_static((const float*)c->act[(size_t)c->L - 1], c->labels, c->mask, c->gact[(size_t)c->L - 1],
                               c->M.n, c->dims[(size_t)c->L], c->M.off.data(), c->M.k, loss_dev, s);
    }
    if (e != hipSuccess) return c->fail(GNN_EHIP, std::string("gnn_loss_static: ") + hipGetErrorString(e));
    c->loss_done = true;
    std::fill(c->bwd_done.begin(), c->bwd_done.end(), 0);
    return GNN_OK;
}

gnn_status gnn_read_loss(gnn_ctx* c, void* stream, float* loss_out)
{
    if (!c || !loss_out) return GNN_EINVAL;
    if (!c->bound || !c->loss_done) return c->fail(GNN_ESTATE, "no loss has been computed");
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = hipStreamSynchronize(s);
    if (e == hipSuccess)
        e = hipMemcpy(loss_out, c->scratch + c->ws.scalars, sizeof(float), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return c->fail(GNN_EHIP, std::string("gnn_read_loss: ") + hipGetErrorString(e));
    return GNN_OK;
}

gnn_status gnn_layer_bwd(gnn_ctx* c, int32_t layer, int32_t p, void* stream)
{
    if (!c) return GNN_EINVAL;
    gnn_status st = check_lp(c, layer, p);
    if (st != GNN_OK) return st;
    if (!c->loss_done) return c->fail(GNN_ESTATE, "gnn_layer_bwd before the forward pass and gnn_loss");
    if (layer < c->L && c->bwd_done[(size_t)layer + 1] < c->M.k)
        return c->fail(GNN_ESTATE, "the backward pass of layer+1 has not covered every partition");
    if (layer < c->L && c->transform_first(layer + 1) && all_done(c->xf_bwd_done, layer + 1, c->M.k) < c->M.k)
        return c->fail(GNN_ESTATE, "gnn_layer_transform_bwd of layer+1 has not covered every partition");
    hipStream_t s = (hipStream_t)stream;
    if (c->model == GNN_GAT) {
        // attention needs the gathered rows of H again (regather), and recomputes its weights
        if (c->staged_layer != layer || c->staged_p != p)
            return c->fail(GNN_ESTATE, "staging does not hold this (layer, partition); call gnn_gather_boundary first");
        if (c->bwd_done[(size_t)layer] == 0) {
            gat_bwd_begin(c, layer, s);
            for (int32_t q = 0; q < c->M.k; ++q) c->xf_bwd_done[(size_t)(layer - 1) * (size_t)c->M.k + (size_t)q] = 0;
        }
        gat_layer_bwd(c, layer, p, s);
        c->bwd_done[(size_t)layer] += 1;
        return check_launch(c, "gnn_layer_bwd");
    }
    if (c->transform_first(layer)) {
        // no regather and no recompute: the layer aggregated H, whose gradient is accumulated here
        if (c->bwd_done[(size_t)layer] == 0) {
            xf_begin_bwd(c, layer, s);
            // grad H takes the buffer H was in
            c->h_layer = 0;
            std::fill(c->xf_fwd_done.begin(), c->xf_fwd_done.end(), 0);
            for (int32_t q = 0; q < c->M.k; ++q) c->xf_bwd_done[(size_t)(layer - 1) * (size_t)c->M.k + (size_t)q] = 0;
        }
        {
            const int64_t r0x = c->M.off[(size_t)p];
            const int32_t dl = c->dims[(size_t)layer], dprev = c->dims[(size_t)layer - 1];
            xf_aggregate_bwd(c, layer, p, c->layer_input(layer, r0x), c->gact[(size_t)layer - 1] + r0x * dl,
                             c->act[(size_t)layer - 1] + r0x * (int64_t)dl * c->act_es(layer),
                             layer >= 2 ? c->gact[(size_t)layer - 2] + r0x * dprev : nullptr, s);
        }
        c->bwd_done[(size_t)layer] += 1;
        return check_launch(c, "gnn_layer_bwd");
    }
    // (a kept aggregate needs no regathered rows)
    const bool kept_z = c->keeps_z(layer) && c->z_done[(size_t)(layer - 1) * (size_t)c->M.k + (size_t)p];
    if (!kept_z && (c->staged_layer != layer || c->staged_p != p))
        return c->fail(GNN_ESTATE, "staging does not hold this (layer, partition); call gnn_gather_boundary first");
    const HostMeta& M = c->M;
    const int64_t r0 = M.off[(size_t)p], np = M.off[(size_t)p + 1] - r0;
    const int64_t nb = M.boff[(size_t)p + 1] - M.boff[(size_t)p];
    const int32_t din = c->dims[(size_t)layer - 1], dout = c->dims[(size_t)layer];

    // scatter-accumulate of the gathered-row gradient: fused into the transposed aggregation
    // (GNNMI_FUSE_SCATTER=0 keeps it a separate pass over a scratch copy)
    static const bool fuse = [] {
        const char* e = std::getenv("GNNMI_FUSE_SCATTER");
        return !(e && e[0] == '0');
    }();
    // write-back buffer initialisation: first partition of this layer since gnn_loss (not when
    // the epoch lets first-touch rows store; the operator over train vertices does not reach
    // every row)
    const bool stores_first = fuse && c->first_touch && c->D.first && !(layer == c->L && c->masked_transpose());
    if (layer >= 2 && c->bwd_done[(size_t)layer] == 0 && !stores_first) {
        Timed t(c, s, GNN_K_OTHER);
        launch_fill_zero(c->gact[(size_t)layer - 2], M.n * (int64_t)din * 4, s);
    }
    const char* act_own = c->act[(size_t)layer - 1] + r0 * (int64_t)dout * c->act_es(layer);
    float* gprev = layer >= 2 ? c->gact[(size_t)layer - 2] : nullptr;
    const char* dY = compute_bwd(c, layer, p, c->layer_input(layer, r0),
                                 c->gact[(size_t)layer - 1] + r0 * dout, act_own, fuse ? gprev : nullptr, nullptr, s);
    if (layer >= 2) {
        if (!fuse) {
            Timed t(c, s, GNN_K_SCATTER);
            launch_scatter_add((const float*)(c->scratch + c->ws.dga), np + nb, np, r0,
                               c->D.bnd + M.boff[(size_t)p], gprev, din, s);
        }
        compute_bwd_self(c, layer, p, dY, gprev + r0 * din, s);
    }
    c->bwd_done[(size_t)layer] += 1;
    return check_launch(c, "gnn_layer_bwd");
}

static gnn_status epoch_resident(gnn_ctx* c, void* stream, float* loss_out);

gnn_status gnn_epoch(gnn_ctx* c, void* stream, float* loss_out)
{
    if (!c || !loss_out) return GNN_EINVAL;
    if (!c->bound) return c->fail(GNN_ESTATE, "buffers are not bound (call gnn_bind)");
    c->events_used = 0;
    if (c->streaming()) {
        gnn_status st = epoch_streaming(c, (hipStream_t)stream, loss_out);
        if (st == GNN_OK && c->prof) collect_profile(c);
        return st;
    }
    const gnn_status st = epoch_resident(c, stream, loss_out);
    if (st != GNN_OK) {
        // an error exit may leave work queued on the context's side stream: the caller's stream
        // waits for it, so that whatever the caller does next on `stream` is ordered behind it
        c->fwd_side = nullptr;
        c->z_slot = 0;
        c->on_side = false;
        if (c->side) {
            const std::string keep = c->err;
            if (hipStreamSynchronize(c->side) != hipSuccess) (void)hipGetLastError();
            c->err = keep;
        }
    }
    return st;
}

static gnn_status epoch_resident(gnn_ctx* c, void* stream, float* loss_out)
{
    hipStream_t s = (hipStream_t)stream;
    const int32_t L = c->L, k = c->M.k;
    gnn_status st = GNN_OK;
    // Overlap (fp32 GCN / GraphSAGE): where an aggregate-first layer l sits below a transform-first
    // layer l + 1, the contractions of layer l + 1's own sweep (H_p = A_p^l W forward; grad W,
    // grad A_p^l backward) run on a side stream, partition by partition, beside layer l's gather /
    // aggregation kernels of the other partitions.  Those contractions touch only rows of
    // partition p, H / grad H, the padded weight copies, their own weight gradient and a split-K
    // region of their own; every dependency is an event, and each buffer sees its kernels in the
    // order of the one-stream schedule, so the results are the same bits.  GNNMI_OVERLAP=0: off.
    const char* overlap_env = std::getenv("GNNMI_OVERLAP");          // read per epoch: tests flip it
    bool overlap = !(overlap_env && overlap_env[0] == '0') && !c->bf16() && c->model != GNN_GAT;
    if (overlap) {
        bool any = false;                 // an aggregate-first layer: its forward contraction moves too
        for (int32_t l = 1; l <= L; ++l) any = any || !c->transform_first(l);
        overlap = any;
    }
    if (overlap && !c->side) {
        if (hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking) != hipSuccess) {
            (void)hipGetLastError();
            c->side = nullptr;
            overlap = false;
        }
    }
    if (overlap)
        while (c->side_events.size() < (size_t)k + 5) {   // k steps, two fences, Z ready, two Z regions free
            hipEvent_t e;
            if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) {
                (void)hipGetLastError();
                overlap = false;
                break;
            }
            c->side_events.push_back(e);
        }
    // layer l aggregates first and layer l + 1 transforms first
    auto paired = [&](int32_t l) {
        return overlap && l >= 1 && l < L && !c->transform_first(l) && c->transform_first(l + 1);
    };
    // backward: a GraphSAGE output layer with padded rows pads its dY into scratch that layer l's
    // partitions use as well, so that pair stays on one stream
    auto paired_bwd = [&](int32_t l) {
        return paired(l) && !(c->model == GNN_SAGE_MEAN && l + 1 == L && c->padded(L) != c->dims[(size_t)L]);
    };
    auto hip_ok = [&](hipError_t e, const char* what) {
        if (e == hipSuccess) return GNN_OK;
        return c->fail(GNN_EHIP, std::string(what) + ": " + hipGetErrorString(e));
    };
    hipEvent_t* step_event = c->side_events.data();                          // [k]
    const hipEvent_t fence_main = overlap ? c->side_events[(size_t)k] : nullptr;
    const hipEvent_t fence_side = overlap ? c->side_events[(size_t)k + 1] : nullptr;

    zero_weight_grads(c, s);
    for (int32_t l = 1; l <= L; ++l) {
        if (c->transform_first(l) && !paired(l - 1))
            for (int32_t t = 0; t < k; ++t)
                if ((st = gnn_layer_transform_fwd(c, l, c->M.sched[(size_t)t], stream)) != GNN_OK) return st;
        // an aggregate-first layer: Z_p is aggregated on the caller's stream into one of two
        // regions and its contraction follows on the side stream while the caller's stream
        // gathers and aggregates the next partition
        // (not when layer l + 1 keeps the side stream busy already: measured neutral in wall time
        // there, and it only stretches the aggregation kernels further)
        const bool side_fwd = overlap && !c->transform_first(l) && !paired(l);
        for (int32_t t = 0; t < k; ++t) {
            const int32_t p = c->M.sched[(size_t)t];
            if (side_fwd) {
                c->z_slot = t & 1;
                // the contraction that read this region two steps ago
                const hipEvent_t z_free = c->side_events[c->side_events.size() - 2 + (size_t)c->z_slot];
                if ((st = hip_ok(hipStreamWaitEvent(s, z_free, 0), "hipStreamWaitEvent")) != GNN_OK) break;
                c->fwd_side = c->side;
            }
            if ((st = gnn_gather_boundary(c, l, p, stream)) != GNN_OK) break;
            if ((st = gnn_layer_fwd(c, l, p, stream)) != GNN_OK) break;
            if (paired(l)) {
                // A_p^l is complete on the caller's stream: layer l + 1 transforms it on the side
                if ((st = hip_ok(hipEventRecord(step_event[t], s), "hipEventRecord")) != GNN_OK) break;
                if ((st = hip_ok(hipStreamWaitEvent(c->side, step_event[t], 0), "hipStreamWaitEvent")) != GNN_OK) break;
                if ((st = gnn_layer_transform_fwd(c, l + 1, p, (void*)c->side)) != GNN_OK) break;
            }
        }
        c->fwd_side = nullptr;
        c->z_slot = 0;
        if (st != GNN_OK) return st;
        if (side_fwd || paired(l)) {
            if ((st = hip_ok(hipEventRecord(fence_side, c->side), "hipEventRecord")) != GNN_OK) return st;
            if ((st = hip_ok(hipStreamWaitEvent(s, fence_side, 0), "hipStreamWaitEvent")) != GNN_OK) return st;
        }
    }
    if ((st = gnn_loss(c, stream)) != GNN_OK) return st;
    // the partitions of a backward layer are walked in schedule order from here on: rows that are
    // first to reach their row of a gradient array store, the others add
    static const bool first_touch_on = [] {
        const char* e = std::getenv("GNNMI_FIRST_TOUCH");
        return !(e && e[0] == '0');
    }();
    struct FirstTouch {
        gnn_ctx* c;
        ~FirstTouch() { c->first_touch = false; }
    } first_touch_scope{c};
    c->first_touch = first_touch_on && c->model != GNN_GAT;
    bool wait_steps = false;          // the partitions of this layer wait for the side stream, step by step
    for (int32_t l = L; l >= 1; --l) {
        const bool xf = c->transform_first(l);
        const bool regather = !xf || c->model == GNN_GAT;
        if (c->model == GNN_GAT && c->h_layer != l &&
            !(c->keep_forward && all_done(c->xf_fwd_done, l, k) == k))
            // attention needs H and the scores of this layer again: recompute them
            for (int32_t t = 0; t < k; ++t)
                if ((st = gnn_layer_transform_fwd(c, l, c->M.sched[(size_t)t], stream)) != GNN_OK) return st;
        for (int32_t t = 0; t < k; ++t) {
            const int32_t p = c->M.sched[(size_t)t];
            if (wait_steps &&
                (st = hip_ok(hipStreamWaitEvent(s, step_event[t], 0), "hipStreamWaitEvent")) != GNN_OK)
                return st;
            const bool kept = c->keeps_z(l) && c->z_done[(size_t)(l - 1) * (size_t)k + (size_t)p];
            if (regather && !kept && (st = gnn_gather_boundary(c, l, p, stream)) != GNN_OK) return st;
            if ((st = gnn_layer_bwd(c, l, p, stream)) != GNN_OK) return st;
        }
        wait_steps = false;
        if (xf && paired_bwd(l - 1)) {
            // grad H of this layer is complete on the caller's stream: its contractions go to the
            // side stream, and partition p of layer l - 1 starts when grad A_p^{l-1} is there
            if ((st = hip_ok(hipEventRecord(fence_main, s), "hipEventRecord")) != GNN_OK) return st;
            if ((st = hip_ok(hipStreamWaitEvent(c->side, fence_main, 0), "hipStreamWaitEvent")) != GNN_OK) return st;
            c->on_side = true;
            for (int32_t t = 0; t < k; ++t) {
                st = gnn_layer_transform_bwd(c, l, c->M.sched[(size_t)t], (void*)c->side);
                if (st == GNN_OK) st = hip_ok(hipEventRecord(step_event[t], c->side), "hipEventRecord");
                if (st != GNN_OK) break;
            }
            c->on_side = false;
            if (st != GNN_OK) return st;
            wait_steps = true;
        } else if (xf) {
            for (int32_t t = 0; t < k; ++t)
                if ((st = gnn_layer_transform_bwd(c, l, c->M.sched[(size_t)t], stream)) != GNN_OK) return st;
        }
    }
    if ((st = gnn_read_loss(c, stream, loss_out)) != GNN_OK) return st;
    if (c->prof) collect_profile(c);
    return GNN_OK;
}

gnn_status gnn_set_dropout(gnn_ctx* c, float p, uint64_t seed, int64_t epoch_index)
{
    if (!c) return GNN_EINVAL;
    if (!(p >= 0.f && p < 1.f)) return c->fail(GNN_EINVAL, "dropout rate must lie in [0, 1)");
    c->dropout_p = p;
    c->dropout_seed = seed;
    c->dropout_epoch = epoch_index;
    return GNN_OK;
}

gnn_status gnn_bind_optimizer(gnn_ctx* c, void* const* m, void* const* v)
{
    if (!c || !m || !v) return GNN_EINVAL;
    const int32_t L = c->L;
    c->opt_m.assign((size_t)3 * L, nullptr);
    c->opt_v.assign((size_t)3 * L, nullptr);
    for (int32_t l = 0; l < L; ++l)
        for (int j = 0; j < 3; ++j) {
            const bool needed = j == 0 || (j == 1 && c->model != GNN_GCN) || (j == 2 && c->has_bias);
            if (needed && (!m[3 * l + j] || !v[3 * l + j])) {
                c->opt_m.clear();
                c->opt_v.clear();
                return c->fail(GNN_EINVAL, "gnn_bind_optimizer: a moment buffer of an existing tensor is null");
            }
            c->opt_m[(size_t)(3 * l + j)] = (float*)m[3 * l + j];
            c->opt_v[(size_t)(3 * l + j)] = (float*)v[3 * l + j];
        }
    return GNN_OK;
}

gnn_status gnn_bind_master_weights(gnn_ctx* c, void* const* master)
{
    if (!c || !master) return GNN_EINVAL;
    if (!c->bf16())
        return c->fail(GNN_EUNSUPPORTED, "fp32 weights are updated in place: master copies belong to GNN_BF16");
    const int32_t L = c->L;
    std::vector<float*> mw((size_t)3 * L, nullptr);
    for (int32_t l = 0; l < L; ++l)
        for (int j = 0; j < 2; ++j) {
            const bool needed = j == 0 || c->model != GNN_GCN;
            if (!needed) continue;
            if (!master[3 * l + j] || (reinterpret_cast<uintptr_t>(master[3 * l + j]) & 3) != 0)
                return c->fail(GNN_EINVAL, "gnn_bind_master_weights: a master copy of an existing matrix is null or unaligned");
            mw[(size_t)(3 * l + j)] = (float*)master[3 * l + j];
        }
    c->master.swap(mw);
    return GNN_OK;
}

gnn_status gnn_optimizer_step(gnn_ctx* c, const gnn_optimizer* opt, int64_t step, void* stream)
{
    if (!c || !opt) return GNN_EINVAL;
    if (!c->bound) return c->fail(GNN_ESTATE, "gnn_optimizer_step before gnn_bind");
    if (c->bf16() && c->master.empty())
        return c->fail(GNN_ESTATE, "bfloat16 weights are stepped through fp32 master copies: call gnn_bind_master_weights");
    if (opt->kind != GNN_OPT_SGD && opt->kind != GNN_OPT_ADAM) return c->fail(GNN_EINVAL, "unknown optimizer");
    if (step < 1) return c->fail(GNN_EINVAL, "step numbers start at 1");
    if (opt->kind == GNN_OPT_ADAM && c->opt_m.empty())
        return c->fail(GNN_ESTATE, "Adam needs gnn_bind_optimizer");
    hipStream_t s = (hipStream_t)stream;
    const float corr1 = (float)(1.0 / (1.0 - std::pow((double)opt->beta1, (double)step)));
    const float corr2 = (float)(1.0 / (1.0 - std::pow((double)opt->beta2, (double)step)));
    Timed t(c, s, GNN_K_OTHER);
    for (int32_t l = 0; l < c->L; ++l)
        for (int j = 0; j < 3; ++j) {
            float* w = (float*)const_cast<char*>(c->w[(size_t)(3 * l + j)]);
            float* g = c->gw[(size_t)(3 * l + j)];
            if (!w || !g) continue;
            if (j == 1 && c->model == GNN_GCN) continue;
            if (j == 2 && !c->has_bias) continue;
            // bfloat16 storage: the step is taken on the fp32 master copy of a matrix, and the
            // bound matrix receives its rounding (biases are fp32 and stepped in place)
            void* w16 = nullptr;
            if (c->bf16() && j < 2) {
                w16 = w;
                w = c->master[(size_t)(3 * l + j)];
            }
            int64_t cnt = j == 2 ? (int64_t)c->dims[(size_t)l + 1]
                                 : (int64_t)c->dims[(size_t)l] * c->dims[(size_t)l + 1];
            if (j == 1 && c->model == GNN_GAT) cnt = (int64_t)2 * c->dims[(size_t)l + 1];
            if (opt->kind == GNN_OPT_ADAM)
                launch_adam(w, g, c->opt_m[(size_t)(3 * l + j)], c->opt_v[(size_t)(3 * l + j)], cnt, opt->lr,
                            opt->beta1, opt->beta2, opt->eps, opt->weight_decay, corr1, corr2, s, w16);
            else
                launch_sgd(w, g, cnt, opt->lr, opt->weight_decay, s, w16);
        }
    return check_launch(c, "gnn_optimizer_step");
}

gnn_status gnn_train(gnn_ctx* c, const gnn_optimizer* opt, int32_t epochs, int64_t first_epoch,
                     float dropout_p, uint64_t dropout_seed, void* stream, float* losses)
{
    if (!c || !opt || !losses || epochs < 0 || first_epoch < 0) return GNN_EINVAL;
    gnn_status st;
    for (int32_t e = 0; e < epochs; ++e) {
        if ((st = gnn_set_dropout(c, dropout_p, dropout_seed, first_epoch + e)) != GNN_OK) return st;
        if ((st = gnn_epoch(c, stream, &losses[e])) != GNN_OK) return st;
        if ((st = gnn_optimizer_step(c, opt, first_epoch + e + 1, stream)) != GNN_OK) return st;
    }
    return GNN_OK;
}

gnn_status gnn_set_profiling(gnn_ctx* c, int32_t enabled)
{
    if (!c || enabled < 0 || enabled > 2) return GNN_EINVAL;
    c->prof = enabled;
    c->events_used = 0;
    return GNN_OK;
}

gnn_status gnn_get_profile(const gnn_ctx* c, double* ms, int64_t* launches)
{
    if (!c || !ms || !launches) return GNN_EINVAL;
    for (int i = 0; i < GNN_K_COUNT; ++i) {
        ms[i] = c->prof_ms[i];
        launches[i] = c->prof_launches[i];
    }
    return GNN_OK;
}

gnn_status gnn_storage_open(gnn_ctx* c, const char* dir, int64_t host_budget_bytes)
{
    if (!c || !dir) return GNN_EINVAL;
    if (!c->built) return c->fail(GNN_ESTATE, "gnn_storage_open before gnn_build_partitions");
    if (!c->streaming())
        return c->fail(GNN_ESTATE, "the storage tier belongs to the streaming schedule: create the context with hbm_budget_bytes > 0");
    c->bound = false;                  // feat / act / grad_act of an earlier gnn_bind are no longer used
    return tier_open(c, dir, host_budget_bytes);
}

gnn_status gnn_storage_close(gnn_ctx* c)
{
    if (!c) return GNN_EINVAL;
    if (c->tier) {
        (void)hipDeviceSynchronize();
        tier_close(c);
        c->bound = false;
    }
    return GNN_OK;
}

gnn_status gnn_storage_keep_results(gnn_ctx* c, int32_t on)
{
    if (!c) return GNN_EINVAL;
    if (!c->tier) return c->fail(GNN_ESTATE, "no storage tier is open (gnn_storage_open)");
    if (on != 0 && on != 1) return c->fail(GNN_EINVAL, "gnn_storage_keep_results takes 0 or 1");
    tier_keep_results(c, on == 1);
    return GNN_OK;
}

static gnn_status storage_array(gnn_ctx* c, int32_t kind, int32_t layer, int* id)
{
    if (!c->tier) return c->fail(GNN_ESTATE, "no storage tier is open (gnn_storage_open)");
    *id = (kind == 0 || kind == 1) ? tier_array_id(c, kind, layer) : -1;
    if (*id < 0) return c->fail(GNN_EINVAL, "no such array: kind 0 takes layers 0..L, kind 1 layers 1..L");
    return GNN_OK;
}

gnn_status gnn_storage_write(gnn_ctx* c, int32_t kind, int32_t layer, const void* src_host)
{
    if (!c || !src_host) return GNN_EINVAL;
    int id;
    gnn_status st = storage_array(c, kind, layer, &id);
    if (st != GNN_OK) return st;
    if (hipDeviceSynchronize() != hipSuccess) (void)hipGetLastError();
    return tier_write(c, id, src_host);
}

gnn_status gnn_storage_read(gnn_ctx* c, int32_t kind, int32_t layer, void* dst_host)
{
    if (!c || !dst_host) return GNN_EINVAL;
    int id;
    gnn_status st = storage_array(c, kind, layer, &id);
    if (st != GNN_OK) return st;
    if (hipDeviceSynchronize() != hipSuccess) (void)hipGetLastError();
    return tier_read(c, id, dst_host);
}

gnn_status gnn_get_storage_stats(const gnn_ctx* c, gnn_storage_stats* out)
{
    if (!c || !out) return GNN_EINVAL;
    if (!c->tier) return c->fail(GNN_ESTATE, "no storage tier is open (gnn_storage_open)");
    tier_get_stats(c, out);
    return GNN_OK;
}

gnn_status gnn_get_stream_stats(const gnn_ctx* c, gnn_stream_stats* out)
{
    if (!c || !out) return GNN_EINVAL;
    *out = c->stream_stats;
    return GNN_OK;
}

}  // extern "C"
