// Graph-attention layers on partitions (one or several heads, the heads' outputs side by side;
// the layer definition is Velickovic et al.'s,
// the model family the paper evaluates next to GCN and GraphSAGE; its section on activation
// regathering notes that attention needs the gathered inputs themselves in the backward pass).
//
// A layer always transforms first.  (With the gather fused into the kernels, see GatView, the
// gathers below move nothing and the kernels read the same rows and scores where they lie.)
// Forward: sweep 1 computes H_p = A_p^{l-1} W and the scores
// s_src = H a_src, s_dst = H a_dst for every partition; sweep 2, per partition, gathers the rows
// of H and the scores s_src of the boundary vertices, turns the scores into attention weights
// (softmax over each destination's sources of LeakyReLU(s_src + s_dst)) and aggregates H with
// them.  Backward: sweep 1, per partition, regathers, recomputes the attention weights (nothing
// is kept from the forward pass), takes the edge-wise products dY[v] . H[u], pushes them through
// softmax and LeakyReLU, and scatter-accumulates both grad H (rows of R_p) and the gradients of
// the scores onto their owners; sweep 2 adds the rank-one terms of the scores to grad H, and
// takes the gradients of the attention vectors, of W and of A^{l-1}.
#include "gnn_ctx.h"

namespace gnnmi {

namespace {

// One head of a layer on one partition.  With one head: f = d_l, fp = the padded row width, and
// every offset below is zero.  With several, head j is a layer of its own on columns
// [j f, (j + 1) f) of W, of the attention vectors, of the bias and of the output, with its own
// attention weights and edge-wise products (`hs` floats per head).  H, grad H and the staged rows
// of the heads lie
//   side by side  (f a multiple of 4: rows of d_l floats, head j at column j f; the layer's
//                  contractions, its gather and its row-wise kernels then run once, on whole
//                  rows, and only the aggregations and the edge-wise products go head by head, on
//                  a column block each), or
//   head after head  (otherwise: an array of fp = f rounded up to 4 floats per vertex for
//                  every head, every step head by head).
// Either way a head's rows are `ldh` floats apart.  The scores of a vertex lie side by side, nh
// floats per vertex, so that the row-wise passes fetch a neighbour's scores once for all heads
// (they run all heads in one launch; the score pointers below then are head 0's).
struct GatView {
    int64_t r0, np, nb, e0, n, hs;
    int32_t din, dout, nh, f, fp, ldh;
    bool side;                  // heads side by side
    // Gather fused into the kernels (gnn_set_gather_fusion): rows of H and scores of boundary
    // vertices are read where they lie, through column indices that name rows of the whole-graph
    // arrays, and nothing is staged.  `col`, `src` / `n_src` / `bsrc` describe the sources either
    // way: columns below n_src are rows of src, the others rows of bsrc.
    bool fused;
    const int32_t* col;
    const float *src, *bsrc;
    int64_t n_src;
    float *H, *gH, *ssrc, *sdst, *gssrc, *gsdst, *bs, *att, *dal, *twatt, *pair, *stg;
    const float *W, *a_src, *a_dst;
    int64_t own() const { return r0 * ldh; }     // offset of the partition's first row in H / grad H
};

GatView view(gnn_ctx* c, int32_t layer, int32_t p, int32_t h)
{
    const HostMeta& M = c->M;
    GatView v;
    v.n = M.n;
    v.r0 = M.off[(size_t)p];
    v.np = M.off[(size_t)p + 1] - v.r0;
    v.nb = M.boff[(size_t)p + 1] - M.boff[(size_t)p];
    v.e0 = M.rp[(size_t)v.r0];
    v.din = c->dims[(size_t)layer - 1];
    v.dout = c->dims[(size_t)layer];
    v.nh = c->nheads(layer);
    v.f = c->head_cols(layer);
    v.fp = c->head_padded(layer);
    v.side = v.nh > 1 && v.fp == v.f;
    v.ldh = v.side ? v.dout : v.fp;
    char* sc = c->scratch;
    const int64_t hoff = v.side ? (int64_t)h * v.f : (int64_t)h * v.n * v.fp;
    // forward results kept for the backward pass (gnn_set_keep_forward): H, the scores and the
    // attention weights of every layer (and partition) have places of their own
    const bool keep = c->keep_forward && !c->ws.gat_h_off.empty();
    const int64_t mh = c->max_heads();
    v.H = (float*)c->hbuf + (keep ? c->ws.gat_h_off[(size_t)layer - 1] : 0) + hoff;
    v.gH = (float*)c->ghbuf + hoff;
    // scores: element (vertex r, head h) at [r nh + h]
    const int64_t so = keep ? (int64_t)(layer - 1) * v.n * mh : 0;
    v.ssrc = (float*)(sc + c->ws.ssrc) + so + h;
    v.sdst = (float*)(sc + c->ws.sdst) + so + h;
    v.gssrc = (float*)(sc + c->ws.gssrc) + h;
    v.gsdst = (float*)(sc + c->ws.gsdst) + h;
    v.bs = (float*)(sc + c->ws.bs) + h;
    v.stg = (float*)c->staging + (v.side ? (int64_t)h * v.f : (int64_t)h * v.nb * v.fp);
    v.hs = M.stats.max_nnz;
    v.att = (float*)(sc + c->ws.att) + (keep ? ((int64_t)(layer - 1) * M.k + p) * mh * v.hs : 0) + (int64_t)h * v.hs;
    v.dal = (float*)(sc + c->ws.dal) + (int64_t)h * v.hs;
    v.twatt = (float*)(sc + c->ws.twatt) + (int64_t)h * v.hs;
    v.pair = (float*)(sc + c->ws.pair);       // (att, dpre) of every entry and head, entry-major
    v.W = (const float*)c->w[(size_t)3 * (layer - 1)] + (int64_t)h * v.f;
    v.a_src = (const float*)c->w[(size_t)3 * (layer - 1) + 1] + (int64_t)h * v.f;
    v.a_dst = v.a_src + v.dout;
    v.fused = c->gather_fused();
    v.col = v.fused ? c->D.gcol : c->D.lcol;
    v.src = v.fused ? v.H : v.H + v.own();
    v.bsrc = v.fused ? nullptr : v.stg;
    v.n_src = v.fused ? v.n : v.np;
    return v;
}

GatRowsHost rows_of(gnn_ctx* c, const GatView& v, int32_t p)
{
    GatRowsHost h;
    h.rp = c->D.rp + v.r0;
    h.col = v.col;
    h.e0 = v.e0;
    h.n_own = v.n_src;
    h.ssrc_own = v.fused ? v.ssrc : v.ssrc + v.r0 * v.nh;
    h.ssrc_bnd = v.bs;
    h.sdst_own = v.sdst + v.r0 * v.nh;
    h.nh = v.nh;
    h.hs = v.hs;
    h.items = plan_items(c->M.plan_fwd, c->D.fwd, p);
    // entries per row: the aggregation launchers pick their short-row kernels by it
    h.items.avg_len = (float)(c->M.rp[(size_t)(v.r0 + v.np)] - v.e0) / (float)std::max<int64_t>(1, v.np);
    return h;
}

}  // namespace

void gat_transform_fwd(gnn_ctx* c, int32_t layer, int32_t p, hipStream_t s)
{
    const int32_t nh = c->nheads(layer);
    const GatView v0 = view(c, layer, p, 0);
    const float* in_own = (const float*)c->layer_input(layer, v0.r0);
    // H_p = A_p^{l-1} W: one contraction for whole rows, or one per head
    const int32_t steps = v0.side ? 1 : nh;
    for (int32_t h = 0; h < steps; ++h) {
        const GatView v = view(c, layer, p, h);
        float* Hp = v.H + v.own();
        if (v.fp != v.f) {
            Timed t(c, s, GNN_K_OTHER);
            launch_fill_zero(Hp, v.np * (int64_t)v.fp * 4, s);
        }
        Timed t(c, s, GNN_K_GEMM_FWD);
        GemmSeg seg;
        seg.a = in_own; seg.lda = v.din;
        seg.b = v.W; seg.ldb = v.dout; seg.k = v.din;
        launch_gemm_nn(&seg, 1, Hp, v.ldh, v.np, v.side ? v.dout : v.f, GemmEpilogue{}, s);
    }
    Timed t(c, s, GNN_K_OTHER);
    launch_gat_scores(v0.H + v0.own(), v0.ldh, v0.f, v0.np, v0.a_src, v0.a_dst, v0.ssrc + v0.r0 * nh,
                      v0.sdst + v0.r0 * nh, nh, v0.side ? (int64_t)v0.f : v0.n * (int64_t)v0.fp, s);
}

// rows of H and scores s_src of the boundary vertices of p
void gat_gather(gnn_ctx* c, int32_t layer, int32_t p, hipStream_t s)
{
    const int32_t nh = c->nheads(layer);
    const int32_t* bnd = c->D.bnd + c->M.boff[(size_t)p];
    const GatView v0 = view(c, layer, p, 0);
    if (v0.fused) return;            // the kernels read the boundary rows and scores themselves
    Timed t(c, s, GNN_K_GATHER);
    const int32_t steps = v0.side ? 1 : nh;
    for (int32_t h = 0; h < steps; ++h) {
        const GatView v = view(c, layer, p, h);
        launch_gather_rows(v.H, bnd, v.stg, v.nb, (int64_t)v.ldh * 4, s);
    }
    launch_gather_rows(v0.ssrc, bnd, v0.bs, v0.nb, (int64_t)nh * 4, s);   // all heads' scores
}

void gat_layer_fwd(gnn_ctx* c, int32_t layer, int32_t p, hipStream_t s)
{
    const int32_t nh = c->nheads(layer);
    float* Z = (float*)(c->scratch + c->ws.z);
    float* segpart = (float*)(c->scratch + c->ws.segpart);
    const GatView v0 = view(c, layer, p, 0);
    const GatRowsHost rows = rows_of(c, v0, p);
    {
        // attention weights of every head
        Timed t(c, s, GNN_K_OTHER);
        launch_gat_attention(rows, v0.att, segpart, s);
        c->att_done[(size_t)(layer - 1) * (size_t)c->M.k + (size_t)p] = 1;
    }
    const float* bias = c->has_bias ? (const float*)c->w[(size_t)3 * (layer - 1) + 2] : nullptr;
    float* out = (float*)c->act[(size_t)layer - 1] + v0.r0 * v0.dout;
    const int relu = layer < c->L ? 1 : 0;
    // Rows of H as wide as the output rows (heads side by side, or one head of unpadded width): the
    // aggregation stores the layer's output itself, bias and activation where it stores a row.
    // Otherwise it fills Z and the head's columns are copied out.
    const bool direct = v0.ldh == v0.dout;
    float* agg = direct ? out : Z;
    SpmmScatter fin;                 // no scatter; what is applied to a stored row
    if (direct) {
        fin.bias = bias;
        fin.relu = relu;
    }
    // heads side by side: every head in one launch, a column slice of the rows each (when the
    // head width suits the slot kernels), else head by head
    bool all_heads = false;
    if (v0.side) {
        Timed t(c, s, GNN_K_SPMM);
        all_heads = launch_spmm_heads(rows.rp, rows.col, v0.att - v0.e0, v0.hs, nh, v0.f, v0.src, v0.n_src,
                                      v0.bsrc, agg, v0.ldh, rows.items, segpart, fin, s);
    }
    if (all_heads && rows.items.nlong > 0) {
        Timed t(c, s, GNN_K_SPMM_REDUCE);
        launch_spmm_reduce(nullptr, agg, v0.ldh, 0, rows.items, segpart, fin, s);
    }
    for (int32_t h = 0; h < nh && !all_heads; ++h) {
        const GatView v = view(c, layer, p, h);
        // the head's column block of the output rows (or of Z), or Z as an array of its own
        float* Zh = agg + (v.side ? (int64_t)h * v.f : 0);
        SpmmScatter finh = fin;
        if (finh.bias) finh.bias += (int64_t)h * v.f;
        {
            Timed t(c, s, GNN_K_SPMM);
            launch_spmm(rows.rp, rows.col, v.att - v.e0, nullptr, v.src, v.n_src, v.bsrc, Zh, v.np, v.fp,
                        0, 0, rows.items, segpart, 1, finh, s, v.ldh);
        }
        if (rows.items.nlong > 0) {
            Timed t(c, s, GNN_K_SPMM_REDUCE);
            launch_spmm_reduce(nullptr, Zh, v.fp, 0, rows.items, segpart, finh, s, v.ldh);
        }
        if (!direct) {
            // the head's columns of the output rows
            Timed t(c, s, GNN_K_GEMM_FWD);
            launch_add_padded(out + (int64_t)h * v.f, Z, v.np, v.f, v.fp, bias ? bias + (int64_t)h * v.f : nullptr, 0,
                              relu, s, v.dout);
        }
    }
    Timed t(c, s, GNN_K_OTHER);
    apply_dropout(c, layer, v0.r0, v0.np, out, 0, s);       // after the activation of a hidden layer
}

// first partition of a layer's backward pass: the accumulators start from zero
void gat_bwd_begin(gnn_ctx* c, int32_t layer, hipStream_t s)
{
    const int64_t n = c->M.n;
    const int64_t nh = c->nheads(layer);
    Timed t(c, s, GNN_K_OTHER);
    launch_fill_zero(c->ghbuf, n * (int64_t)c->hrow(layer) * 4, s);
    launch_fill_zero(c->scratch + c->ws.gssrc, n * nh * 4, s);
    launch_fill_zero(c->scratch + c->ws.gsdst, n * nh * 4, s);
    // grad A^{l-1} needs no initialisation: each of its rows is written once, by grad H_p W^T
}

void gat_layer_bwd(gnn_ctx* c, int32_t layer, int32_t p, hipStream_t s)
{
    const HostMeta& M = c->M;
    const int32_t nh = c->nheads(layer);
    const GatView v0 = view(c, layer, p, 0);
    float* gb = c->has_bias ? c->gw[(size_t)3 * (layer - 1) + 2] : nullptr;
    float* dYbuf = (float*)(c->scratch + c->ws.dy);
    float* colpart = (float*)(c->scratch + c->ws.colpart);
    const float* g_own = c->gact[(size_t)layer - 1] + v0.r0 * v0.dout;
    const float* dY = g_own;
    {
        Timed t(c, s, GNN_K_ACT_BWD);
        if (layer < c->L) {
            // (dropout followed the activation: its dropped elements are the zeros of the stored
            // rows, the others carry the factor 1 / (1 - p))
            launch_act_bwd(g_own, (const float*)c->act[(size_t)layer - 1] + v0.r0 * v0.dout, dYbuf, v0.np, v0.dout, gb,
                           colpart, c->dropout_p > 0.f ? 1.f / (1.f - c->dropout_p) : 1.f, s);
            dY = dYbuf;
        } else {
            launch_act_bwd(g_own, nullptr, nullptr, v0.np, v0.dout, gb, colpart, 1.f, s);
        }
    }
    const int64_t t0 = M.toff[(size_t)p];
    SpmmItems titems = plan_items(M.plan_bwd, c->D.bwd, p);
    titems.avg_len = (float)(M.trp[(size_t)M.toff[(size_t)p + 1]] - M.trp[(size_t)t0]) /
                     (float)std::max<int64_t>(1, v0.np + v0.nb);
    const int32_t* bnd = c->D.bnd + M.boff[(size_t)p];
    float* segpart = (float*)(c->scratch + c->ws.segpart);
    const GatRowsHost rows = rows_of(c, v0, p);
    if (!(c->keep_forward && c->att_done[(size_t)(layer - 1) * (size_t)M.k + (size_t)p])) {
        // recompute the attention weights of every head from the regathered scores (unless the
        // forward pass's are kept)
        Timed t(c, s, GNN_K_OTHER);
        launch_gat_attention(rows, v0.att, segpart, s);
    }
    // The head's columns of dY with rows ldh floats apart: dY itself when the heads lie side by
    // side (or there is one head of unpadded width), else copies of fp floats per row, head after
    // head (np fp floats each).
    float* pad = (float*)(c->scratch + c->ws.dz);
    const bool copy = !v0.side && (nh > 1 || v0.fp != v0.f);
    auto dy_of = [&](const GatView& v, int32_t h) -> const float* {
        if (copy) return pad + (int64_t)h * v.np * v.fp;
        return dY + (v.side ? (int64_t)h * v.f : 0);
    };
    const bool sliced = v0.side;      // every head in one launch, a column slice of the rows each
    if (sliced) {
        Timed t(c, s, GNN_K_SPMM);      // edge-wise products of every head: one source row read per entry and head
        launch_gat_dots(rows.rp, rows.col, v0.e0, v0.n_src, v0.src, v0.bsrc, dY, v0.f, v0.ldh, v0.dal, rows.items,
                        s, nh, v0.hs);
    }
    for (int32_t h = 0; h < nh && !sliced; ++h) {
        const GatView v = view(c, layer, p, h);
        if (copy) {
            Timed t(c, s, GNN_K_OTHER);
            launch_pad_rows(pad + (int64_t)h * v.np * v.fp, dY + (int64_t)h * v.f, v.np, v.f, v.fp, s, v.dout);
        }
        Timed t(c, s, GNN_K_SPMM);      // edge-wise products: one source row read per entry
        launch_gat_dots(rows.rp, rows.col, v.e0, v.n_src, v.src, v.bsrc, dy_of(v, h), v.fp, v.ldh, v.dal,
                        rows.items, s);
    }
    {
        Timed t(c, s, GNN_K_OTHER);     // every head
        launch_gat_bwd_scalars(rows, v0.att, v0.dal, v0.pair, v0.gsdst + v0.r0 * nh, segpart, s);
        launch_gat_transposed(c->D.trp + t0, c->D.tperm, v0.e0, v0.np, v0.r0, bnd, titems, v0.pair, v0.twatt,
                              v0.gssrc, nh, v0.hs, segpart, s);
    }
    SpmmScatter sc;
    sc.n_own = v0.np;
    sc.base_row = v0.r0;
    sc.idx = bnd;
    bool all_heads = false;
    if (v0.side) {
        Timed t(c, s, GNN_K_SPMM_T);
        all_heads = launch_spmm_heads(c->D.trp + t0, c->D.tcol, v0.twatt - v0.e0, v0.hs, nh, v0.f, dY, v0.np, nullptr,
                                      v0.gH, v0.ldh, titems, segpart, sc, s);
    }
    if (all_heads && titems.nlong > 0) {
        Timed t(c, s, GNN_K_SPMM_REDUCE);
        launch_spmm_reduce(nullptr, v0.gH, v0.ldh, 0, titems, segpart, sc, s);
    }
    for (int32_t h = 0; h < nh && !all_heads; ++h) {
        const GatView v = view(c, layer, p, h);
        {
            Timed t(c, s, GNN_K_SPMM_T);
            launch_spmm(c->D.trp + t0, c->D.tcol, v.twatt - v.e0, nullptr, dy_of(v, h), v.np, nullptr, v.gH,
                        v.np + v.nb, v.fp, 0, 0, titems, segpart, 0, sc, s, v.ldh);
        }
        if (titems.nlong > 0) {
            Timed t(c, s, GNN_K_SPMM_REDUCE);
            launch_spmm_reduce(nullptr, v.gH, v.fp, 0, titems, segpart, sc, s, v.ldh);
        }
    }
}

void gat_transform_bwd(gnn_ctx* c, int32_t layer, int32_t p, hipStream_t s)
{
    const int32_t nh = c->nheads(layer);
    float* part = (float*)(c->scratch + c->ws.colpart);
    float* ga = c->gw[(size_t)3 * (layer - 1) + 1];       // grad a_src (d_l floats), then grad a_dst
    float* gW = c->gw[(size_t)3 * (layer - 1)];
    float* splitk = (float*)(c->scratch + c->ws.partial);
    const GatView v0 = view(c, layer, p, 0);
    const float* in_own = (const float*)c->layer_input(layer, v0.r0);
    float* gprev = layer >= 2 ? c->gact[(size_t)layer - 2] + v0.r0 * v0.din : nullptr;
    if (nh == 1 || v0.side) {
        // whole rows: one rank-one update, one weight gradient, one input gradient
        float* gHp = v0.gH + v0.own();
        {
            Timed t(c, s, GNN_K_OTHER);
            launch_gat_rank1(gHp, v0.H + v0.own(), v0.ldh, v0.dout, v0.np, v0.gssrc + v0.r0 * nh, v0.gsdst + v0.r0 * nh,
                             nh, v0.f, v0.a_src, v0.a_dst, part, s);
            launch_colsum_finish(part, (v0.np + 255) / 256, 2 * v0.dout, ga, s);
        }
        {
            Timed t(c, s, GNN_K_GEMM_DW);
            launch_gemm_tn(in_own, v0.din, gHp, v0.ldh, gW, v0.dout, v0.din, v0.dout, v0.np, splitk, s);
        }
        if (gprev) {
            Timed t(c, s, GNN_K_GEMM_DZ);   // the only term of grad A^{l-1}_p: written, not accumulated
            launch_gemm_nt(gHp, v0.ldh, v0.W, v0.dout, gprev, v0.din, v0.np, v0.din, v0.dout, GemmEpilogue{}, s);
        }
        return;
    }
    for (int32_t h = 0; h < nh; ++h) {
        const GatView v = view(c, layer, p, h);
        float* gHp = v.gH + v.own();
        {
            Timed t(c, s, GNN_K_OTHER);
            launch_gat_rank1(gHp, v.H + v.own(), v.ldh, v.f, v.np, v.gssrc + v.r0 * nh, v.gsdst + v.r0 * nh, nh, v.f,
                             v.a_src, v.a_dst, part, s);
            launch_colsum_finish(part, (v.np + 255) / 256, v.f, ga + (int64_t)h * v.f, s, 2 * v.f);
            launch_colsum_finish(part + v.f, (v.np + 255) / 256, v.f, ga + v.dout + (int64_t)h * v.f, s, 2 * v.f);
        }
        Timed t(c, s, GNN_K_GEMM_DW);
        launch_gemm_tn(in_own, v.din, gHp, v.ldh, gW + (int64_t)h * v.f, v.dout, v.din, v.f, v.np, splitk, s);
    }
    if (gprev) {
        // grad A^{l-1}_p = sum over heads of grad H_p W^T on the head's columns: written by the
        // first contraction (two heads at a time), accumulated by the others
        Timed t(c, s, GNN_K_GEMM_DZ);
        for (int32_t h0 = 0; h0 < nh; h0 += 2) {
            GemmSeg segs[2];
            const int nseg = nh - h0 < 2 ? 1 : 2;
            for (int i = 0; i < nseg; ++i) {
                const GatView vh = view(c, layer, p, h0 + i);
                segs[i].a = vh.gH + vh.own(); segs[i].lda = vh.ldh;
                segs[i].b = vh.W; segs[i].ldb = vh.dout; segs[i].k = vh.f;
            }
            GemmEpilogue ep;
            ep.accumulate = h0 > 0 ? 1 : 0;
            launch_gemm_nt2(segs, nseg, gprev, v0.din, v0.np, v0.din, ep, s);
        }
    }
}

}  // namespace gnnmi
