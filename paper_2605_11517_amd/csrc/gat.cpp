// Graph-attention layers on partitions (one head; the layer definition is Velickovic et al.'s,
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

struct GatView {
    int64_t r0, np, nb, e0;
    int32_t din, dout, dp;
    float *H, *gH, *ssrc, *sdst, *gssrc, *gsdst, *bs, *att, *dal, *twatt;
    const float *a_src, *a_dst;
};

GatView view(gnn_ctx* c, int32_t layer, int32_t p)
{
    const HostMeta& M = c->M;
    GatView v;
    v.r0 = M.off[(size_t)p];
    v.np = M.off[(size_t)p + 1] - v.r0;
    v.nb = M.boff[(size_t)p + 1] - M.boff[(size_t)p];
    v.e0 = M.rp[(size_t)v.r0];
    v.din = c->dims[(size_t)layer - 1];
    v.dout = c->dims[(size_t)layer];
    v.dp = c->padded(layer);
    char* sc = c->scratch;
    v.H = (float*)c->hbuf;
    v.gH = (float*)c->ghbuf;
    v.ssrc = (float*)(sc + c->ws.ssrc);
    v.sdst = (float*)(sc + c->ws.sdst);
    v.gssrc = (float*)(sc + c->ws.gssrc);
    v.gsdst = (float*)(sc + c->ws.gsdst);
    v.bs = (float*)(sc + c->ws.bs);
    v.att = (float*)(sc + c->ws.att);
    v.dal = (float*)(sc + c->ws.dal);
    v.twatt = (float*)(sc + c->ws.twatt);
    v.a_src = (const float*)c->w[(size_t)3 * (layer - 1) + 1];
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
    h.ssrc_own = v.ssrc + v.r0;
    h.ssrc_bnd = v.bs;
    h.sdst_own = v.sdst + v.r0;
    h.items = plan_items(c->M.plan_fwd, c->D.fwd, p);
    return h;
}

}  // namespace

void gat_transform_fwd(gnn_ctx* c, int32_t layer, int32_t p, hipStream_t s)
{
    const GatView v = view(c, layer, p);
    float* Hp = v.H + v.r0 * v.dp;
    if (v.dp != v.dout) {
        Timed t(c, s, GNN_K_OTHER);
        launch_fill_zero(Hp, v.np * (int64_t)v.dp * 4, s);
    }
    {
        Timed t(c, s, GNN_K_GEMM_FWD);
        GemmSeg seg;
        seg.a = (const float*)c->layer_input(layer, v.r0); seg.lda = v.din;
        seg.b = (const float*)c->w[(size_t)3 * (layer - 1)]; seg.ldb = v.dout; seg.k = v.din;
        launch_gemm_nn(&seg, 1, Hp, v.dp, v.np, v.dout, GemmEpilogue{}, s);
    }
    Timed t(c, s, GNN_K_OTHER);
    launch_gat_scores(Hp, v.dp, v.dout, v.np, v.a_src, v.a_dst, v.ssrc + v.r0, v.sdst + v.r0, s);
}

// rows of H and scores s_src of the boundary vertices of p
void gat_gather(gnn_ctx* c, int32_t layer, int32_t p, hipStream_t s)
{
    const GatView v = view(c, layer, p);
    const int32_t* bnd = c->D.bnd + c->M.boff[(size_t)p];
    Timed t(c, s, GNN_K_GATHER);
    launch_gather_rows(v.H, bnd, c->staging, v.nb, (int64_t)v.dp * 4, s);
    launch_gather_rows(v.ssrc, bnd, v.bs, v.nb, 4, s);
}

void gat_layer_fwd(gnn_ctx* c, int32_t layer, int32_t p, hipStream_t s)
{
    const GatView v = view(c, layer, p);
    const GatRowsHost rows = rows_of(c, v, p);
    {
        Timed t(c, s, GNN_K_OTHER);
        launch_gat_attention(rows, v.att, (float*)(c->scratch + c->ws.segpart), s);
    }
    float* Z = (float*)(c->scratch + c->ws.z);
    float* segpart = (float*)(c->scratch + c->ws.segpart);
    {
        Timed t(c, s, GNN_K_SPMM);
        launch_spmm(rows.rp, rows.col, v.att - v.e0, nullptr, v.H + v.r0 * v.dp, v.np, c->staging, Z, v.np, v.dp,
                    0, 0, rows.items, segpart, 1, SpmmScatter{}, s);
    }
    if (rows.items.nlong > 0) {
        Timed t(c, s, GNN_K_SPMM_REDUCE);
        launch_spmm_reduce(nullptr, Z, v.dp, 0, rows.items, segpart, SpmmScatter{}, s);
    }
    float* out = (float*)c->act[(size_t)layer - 1] + v.r0 * v.dout;
    const float* bias = c->has_bias ? (const float*)c->w[(size_t)3 * (layer - 1) + 2] : nullptr;
    Timed t(c, s, GNN_K_GEMM_FWD);
    launch_add_padded(out, Z, v.np, v.dout, v.dp, bias, 0, layer < c->L ? 1 : 0, s);
}

// first partition of a layer's backward pass: the accumulators start from zero
void gat_bwd_begin(gnn_ctx* c, int32_t layer, hipStream_t s)
{
    const int64_t n = c->M.n;
    Timed t(c, s, GNN_K_OTHER);
    launch_fill_zero(c->ghbuf, n * (int64_t)c->padded(layer) * 4, s);
    launch_fill_zero(c->scratch + c->ws.gssrc, n * 4, s);
    launch_fill_zero(c->scratch + c->ws.gsdst, n * 4, s);
    // grad A^{l-1} needs no initialisation: each of its rows is written once, by grad H_p W^T
}

void gat_layer_bwd(gnn_ctx* c, int32_t layer, int32_t p, hipStream_t s)
{
    const HostMeta& M = c->M;
    const GatView v = view(c, layer, p);
    const GatRowsHost rows = rows_of(c, v, p);
    float* gb = c->has_bias ? c->gw[(size_t)3 * (layer - 1) + 2] : nullptr;
    float* dYbuf = (float*)(c->scratch + c->ws.dy);
    float* colpart = (float*)(c->scratch + c->ws.colpart);
    const float* g_own = c->gact[(size_t)layer - 1] + v.r0 * v.dout;
    const float* dY = g_own;
    {
        Timed t(c, s, GNN_K_ACT_BWD);
        if (layer < c->L) {
            launch_act_bwd(g_own, (const float*)c->act[(size_t)layer - 1] + v.r0 * v.dout, dYbuf, v.np, v.dout, gb,
                           colpart, 1.f, s);
            dY = dYbuf;
        } else {
            launch_act_bwd(g_own, nullptr, nullptr, v.np, v.dout, gb, colpart, 1.f, s);
        }
    }
    const float* dYp = dY;
    if (v.dp != v.dout) {
        Timed t(c, s, GNN_K_OTHER);
        float* pad = (float*)(c->scratch + c->ws.dz);
        launch_pad_rows(pad, dY, v.np, v.dout, v.dp, s);
        dYp = pad;
    }
    {
        // recompute the attention weights from the regathered scores
        Timed t(c, s, GNN_K_OTHER);
        launch_gat_attention(rows, v.att, (float*)(c->scratch + c->ws.segpart), s);
    }
    {
        Timed t(c, s, GNN_K_SPMM);      // edge-wise products: one source row read per entry
        launch_gat_dots(rows.rp, rows.col, v.e0, v.np, v.H + v.r0 * v.dp, (const float*)c->staging, dYp, v.dp,
                        v.dal, rows.items, s);
    }
    const int64_t t0 = M.toff[(size_t)p];
    const SpmmItems titems = plan_items(M.plan_bwd, c->D.bwd, p);
    const int32_t* bnd = c->D.bnd + M.boff[(size_t)p];
    {
        Timed t(c, s, GNN_K_OTHER);
        launch_gat_bwd_scalars(rows, v.att, v.dal, v.gsdst + v.r0, (float*)(c->scratch + c->ws.segpart), s);
        launch_gat_transposed(c->D.trp + t0, c->D.tperm, v.e0, v.np, v.r0, bnd, titems, v.att, v.dal, v.twatt,
                              v.gssrc, s);
    }
    float* segpart = (float*)(c->scratch + c->ws.segpart);
    SpmmScatter sc;
    sc.n_own = v.np;
    sc.base_row = v.r0;
    sc.idx = bnd;
    {
        Timed t(c, s, GNN_K_SPMM_T);
        launch_spmm(c->D.trp + t0, c->D.tcol, v.twatt - v.e0, nullptr, dYp, v.np, nullptr, v.gH, v.np + v.nb, v.dp,
                    0, 0, titems, segpart, 0, sc, s);
    }
    if (titems.nlong > 0) {
        Timed t(c, s, GNN_K_SPMM_REDUCE);
        launch_spmm_reduce(nullptr, v.gH, v.dp, 0, titems, segpart, sc, s);
    }
}

void gat_transform_bwd(gnn_ctx* c, int32_t layer, int32_t p, hipStream_t s)
{
    const GatView v = view(c, layer, p);
    float* gHp = v.gH + v.r0 * v.dp;
    const float* Hp = v.H + v.r0 * v.dp;
    float* part = (float*)(c->scratch + c->ws.colpart);
    {
        Timed t(c, s, GNN_K_OTHER);
        launch_gat_rank1(gHp, Hp, v.dp, v.dout, v.np, v.gssrc + v.r0, v.gsdst + v.r0, v.a_src, v.a_dst, part, s);
        launch_colsum_finish(part, (v.np + 255) / 256, 2 * v.dout, c->gw[(size_t)3 * (layer - 1) + 1], s);
    }
    const float* in_own = (const float*)c->layer_input(layer, v.r0);
    {
        Timed t(c, s, GNN_K_GEMM_DW);
        launch_gemm_tn(in_own, v.din, gHp, v.dp, c->gw[(size_t)3 * (layer - 1)], v.dout, v.din, v.dout, v.np,
                       (float*)(c->scratch + c->ws.partial), s);
    }
    if (layer >= 2) {
        Timed t(c, s, GNN_K_GEMM_DZ);
        GemmEpilogue ep;                 // the only term of grad A^{l-1}_p: written, not accumulated
        launch_gemm_nt(gHp, v.dp, (const float*)c->w[(size_t)3 * (layer - 1)], v.dout,
                       c->gact[(size_t)layer - 2] + v.r0 * v.din, v.din, v.np, v.din, v.dout, ep, s);
    }
}

}  // namespace gnnmi
