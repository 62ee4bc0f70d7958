// Graph-attention layers on partitions (one or several heads, the heads' outputs side by side;
// the layer definition is Velickovic et al.'s,
// the model family the paper evaluates next to GCN and GraphSAGE; its section on activation
// regathering notes that attention needs the gathered inputs themselves in the backward pass).
//
// A layer always transforms first.  Forward: sweep 1 computes H_p = A_p^{l-1} W and the scores
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
// arrays of H and grad H (fp floats per vertex) and of attention weights and edge-wise products
// (`hs` floats per head); the scores of a vertex lie side by side, nh floats per vertex, so that
// the row-wise passes fetch a neighbour's scores once for all heads (they run all heads in one
// launch; the pointers below then are head 0's).
struct GatView {
    int64_t r0, np, nb, e0, n, hs;
    int32_t din, dout, nh, f, fp;
    float *H, *gH, *ssrc, *sdst, *gssrc, *gsdst, *bs, *att, *dal, *twatt, *pair, *stg;
    const float *W, *a_src, *a_dst;
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
    char* sc = c->scratch;
    v.H = (float*)c->hbuf + (int64_t)h * v.n * v.fp;
    v.gH = (float*)c->ghbuf + (int64_t)h * v.n * v.fp;
    // scores: element (vertex r, head h) at [r nh + h]
    v.ssrc = (float*)(sc + c->ws.ssrc) + h;
    v.sdst = (float*)(sc + c->ws.sdst) + h;
    v.gssrc = (float*)(sc + c->ws.gssrc) + h;
    v.gsdst = (float*)(sc + c->ws.gsdst) + h;
    v.bs = (float*)(sc + c->ws.bs) + h;
    v.stg = (float*)c->staging + (int64_t)h * v.nb * v.fp;
    v.hs = M.stats.max_nnz;
    v.att = (float*)(sc + c->ws.att) + (int64_t)h * v.hs;
    v.dal = (float*)(sc + c->ws.dal) + (int64_t)h * v.hs;
    v.twatt = (float*)(sc + c->ws.twatt) + (int64_t)h * v.hs;
    v.pair = (float*)(sc + c->ws.pair);       // (att, dpre) of every entry and head, entry-major
    v.W = (const float*)c->w[(size_t)3 * (layer - 1)] + (int64_t)h * v.f;
    v.a_src = (const float*)c->w[(size_t)3 * (layer - 1) + 1] + (int64_t)h * v.f;
    v.a_dst = v.a_src + v.dout;
    return v;
}

GatRowsHost rows_of(gnn_ctx* c, const GatView& v, int32_t p)
{
    GatRowsHost h;
    h.rp = c->D.rp + v.r0;
    h.col = c->D.lcol;
    h.e0 = v.e0;
    h.n_own = v.np;
    h.ssrc_own = v.ssrc + v.r0 * v.nh;
    h.ssrc_bnd = v.bs;
    h.sdst_own = v.sdst + v.r0 * v.nh;
    h.nh = v.nh;
    h.hs = v.hs;
    h.items = plan_items(c->M.plan_fwd, c->D.fwd, p);
    return h;
}

}  // namespace

void gat_transform_fwd(gnn_ctx* c, int32_t layer, int32_t p, hipStream_t s)
{
    const int32_t nh = c->nheads(layer);
    for (int32_t h = 0; h < nh; ++h) {
        const GatView v = view(c, layer, p, h);
        float* Hp = v.H + v.r0 * v.fp;
        if (v.fp != v.f) {
            Timed t(c, s, GNN_K_OTHER);
            launch_fill_zero(Hp, v.np * (int64_t)v.fp * 4, s);
        }
        {
            Timed t(c, s, GNN_K_GEMM_FWD);
            GemmSeg seg;
            seg.a = (const float*)c->layer_input(layer, v.r0); seg.lda = v.din;
            seg.b = v.W; seg.ldb = v.dout; seg.k = v.din;
            launch_gemm_nn(&seg, 1, Hp, v.fp, v.np, v.f, GemmEpilogue{}, s);
        }
        Timed t(c, s, GNN_K_OTHER);
        launch_gat_scores(Hp, v.fp, v.f, v.np, v.a_src, v.a_dst, v.ssrc + v.r0 * v.nh, v.sdst + v.r0 * v.nh, v.nh, s);
    }
}

// rows of H and scores s_src of the boundary vertices of p, head by head
void gat_gather(gnn_ctx* c, int32_t layer, int32_t p, hipStream_t s)
{
    const int32_t nh = c->nheads(layer);
    const int32_t* bnd = c->D.bnd + c->M.boff[(size_t)p];
    Timed t(c, s, GNN_K_GATHER);
    for (int32_t h = 0; h < nh; ++h) {
        const GatView v = view(c, layer, p, h);
        launch_gather_rows(v.H, bnd, v.stg, v.nb, (int64_t)v.fp * 4, s);
        if (h == 0) launch_gather_rows(v.ssrc, bnd, v.bs, v.nb, (int64_t)nh * 4, s);   // all heads' scores
    }
}

void gat_layer_fwd(gnn_ctx* c, int32_t layer, int32_t p, hipStream_t s)
{
    const int32_t nh = c->nheads(layer);
    float* Z = (float*)(c->scratch + c->ws.z);
    float* segpart = (float*)(c->scratch + c->ws.segpart);
    {
        // attention weights of every head
        const GatView v = view(c, layer, p, 0);
        Timed t(c, s, GNN_K_OTHER);
        launch_gat_attention(rows_of(c, v, p), v.att, segpart, s);
    }
    for (int32_t h = 0; h < nh; ++h) {
        const GatView v = view(c, layer, p, h);
        const GatRowsHost rows = rows_of(c, v, p);
        {
            Timed t(c, s, GNN_K_SPMM);
            launch_spmm(rows.rp, rows.col, v.att - v.e0, nullptr, v.H + v.r0 * v.fp, v.np, v.stg, Z, v.np, v.fp,
                        0, 0, rows.items, segpart, 1, SpmmScatter{}, s);
        }
        if (rows.items.nlong > 0) {
            Timed t(c, s, GNN_K_SPMM_REDUCE);
            launch_spmm_reduce(nullptr, Z, v.fp, 0, rows.items, segpart, SpmmScatter{}, s);
        }
        // the head's columns of the output rows
        float* out = (float*)c->act[(size_t)layer - 1] + v.r0 * v.dout + (int64_t)h * v.f;
        const float* bias = c->has_bias ? (const float*)c->w[(size_t)3 * (layer - 1) + 2] + (int64_t)h * v.f : nullptr;
        Timed t(c, s, GNN_K_GEMM_FWD);
        launch_add_padded(out, Z, v.np, v.f, v.fp, bias, 0, layer < c->L ? 1 : 0, s, v.dout);
    }
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
            launch_act_bwd(g_own, (const float*)c->act[(size_t)layer - 1] + v0.r0 * v0.dout, dYbuf, v0.np, v0.dout, gb,
                           colpart, 1.f, s);
            dY = dYbuf;
        } else {
            launch_act_bwd(g_own, nullptr, nullptr, v0.np, v0.dout, gb, colpart, 1.f, s);
        }
    }
    const int64_t t0 = M.toff[(size_t)p];
    const SpmmItems titems = plan_items(M.plan_bwd, c->D.bwd, p);
    const int32_t* bnd = c->D.bnd + M.boff[(size_t)p];
    float* segpart = (float*)(c->scratch + c->ws.segpart);
    const GatRowsHost rows = rows_of(c, v0, p);
    {
        // recompute the attention weights of every head from the regathered scores
        Timed t(c, s, GNN_K_OTHER);
        launch_gat_attention(rows, v0.att, segpart, s);
    }
    // the head's columns of dY as rows of fp floats, head after head (np fp floats each)
    float* pad = (float*)(c->scratch + c->ws.dz);
    const bool padded = nh > 1 || v0.fp != v0.f;
    for (int32_t h = 0; h < nh; ++h) {
        const GatView v = view(c, layer, p, h);
        const float* dYp = dY;
        if (padded) {
            Timed t(c, s, GNN_K_OTHER);
            float* ph = pad + (int64_t)h * v.np * v.fp;
            launch_pad_rows(ph, dY + (int64_t)h * v.f, v.np, v.f, v.fp, s, v.dout);
            dYp = ph;
        }
        Timed t(c, s, GNN_K_SPMM);      // edge-wise products: one source row read per entry
        launch_gat_dots(rows.rp, rows.col, v.e0, v.np, v.H + v.r0 * v.fp, v.stg, dYp, v.fp, v.dal, rows.items, s);
    }
    {
        Timed t(c, s, GNN_K_OTHER);     // every head
        launch_gat_bwd_scalars(rows, v0.att, v0.dal, v0.pair, v0.gsdst + v0.r0 * nh, segpart, s);
        launch_gat_transposed(c->D.trp + t0, c->D.tperm, v0.e0, v0.np, v0.r0, bnd, titems, v0.pair, v0.twatt,
                              v0.gssrc, nh, v0.hs, s);
    }
    for (int32_t h = 0; h < nh; ++h) {
        const GatView v = view(c, layer, p, h);
        const float* dYp = padded ? pad + (int64_t)h * v.np * v.fp : dY;
        SpmmScatter sc;
        sc.n_own = v.np;
        sc.base_row = v.r0;
        sc.idx = bnd;
        {
            Timed t(c, s, GNN_K_SPMM_T);
            launch_spmm(c->D.trp + t0, c->D.tcol, v.twatt - v.e0, nullptr, dYp, v.np, nullptr, v.gH, v.np + v.nb, v.fp,
                        0, 0, titems, segpart, 0, sc, s);
        }
        if (titems.nlong > 0) {
            Timed t(c, s, GNN_K_SPMM_REDUCE);
            launch_spmm_reduce(nullptr, v.gH, v.fp, 0, titems, segpart, sc, s);
        }
    }
}

void gat_transform_bwd(gnn_ctx* c, int32_t layer, int32_t p, hipStream_t s)
{
    const int32_t nh = c->nheads(layer);
    float* part = (float*)(c->scratch + c->ws.colpart);
    float* ga = c->gw[(size_t)3 * (layer - 1) + 1];       // grad a_src (d_l floats), then grad a_dst
    for (int32_t h = 0; h < nh; ++h) {
        const GatView v = view(c, layer, p, h);
        float* gHp = v.gH + v.r0 * v.fp;
        const float* Hp = v.H + v.r0 * v.fp;
        {
            Timed t(c, s, GNN_K_OTHER);
            launch_gat_rank1(gHp, Hp, v.fp, v.f, v.np, v.gssrc + v.r0 * nh, v.gsdst + v.r0 * nh, nh, v.a_src, v.a_dst,
                             part, s);
            if (nh == 1) {
                launch_colsum_finish(part, (v.np + 255) / 256, 2 * v.dout, ga, s);
            } else {
                launch_colsum_finish(part, (v.np + 255) / 256, v.f, ga + (int64_t)h * v.f, s, 2 * v.f);
                launch_colsum_finish(part + v.f, (v.np + 255) / 256, v.f, ga + v.dout + (int64_t)h * v.f, s, 2 * v.f);
            }
        }
        const float* in_own = (const float*)c->layer_input(layer, v.r0);
        Timed t(c, s, GNN_K_GEMM_DW);
        launch_gemm_tn(in_own, v.din, gHp, v.fp, c->gw[(size_t)3 * (layer - 1)] + (int64_t)h * v.f, v.dout, v.din,
                       v.f, v.np, (float*)(c->scratch + c->ws.partial), s);
    }
    if (layer >= 2) {
        // grad A^{l-1}_p = sum over heads of grad H_p W^T on the head's columns: written by the
        // first contraction (two heads at a time), accumulated by the others
        Timed t(c, s, GNN_K_GEMM_DZ);
        const GatView v = view(c, layer, p, 0);
        float* out = c->gact[(size_t)layer - 2] + v.r0 * v.din;
        if (nh == 1) {
            launch_gemm_nt(v.gH + v.r0 * v.fp, v.fp, v.W, v.dout, out, v.din, v.np, v.din, v.dout, GemmEpilogue{}, s);
        } else {
            for (int32_t h0 = 0; h0 < nh; h0 += 2) {
                GemmSeg segs[2];
                const int nseg = nh - h0 < 2 ? 1 : 2;
                for (int i = 0; i < nseg; ++i) {
                    const GatView vh = view(c, layer, p, h0 + i);
                    segs[i].a = vh.gH + vh.r0 * vh.fp; segs[i].lda = vh.fp;
                    segs[i].b = vh.W; segs[i].ldb = vh.dout; segs[i].k = vh.f;
                }
                GemmEpilogue ep;
                ep.accumulate = h0 > 0 ? 1 : 0;
                launch_gemm_nt2(segs, nseg, out, v.din, v.np, v.din, ep, s);
            }
        }
    }
}

}  // namespace gnnmi
