// Context object behind the C ABI and the helpers shared by the resident and the streaming
// schedule.
#pragma once

#include <algorithm>
#include <memory>
#include <string>
#include <vector>

#include "gnn_internal.h"

namespace gnnmi {

struct DevMeta {
    int64_t* rp = nullptr;
    int32_t* lcol = nullptr;
    int32_t* gcol = nullptr;   // the same entries as rows of the whole-graph arrays (fused gather)
    float* ew = nullptr;
    float* rscale = nullptr;
    int32_t* bnd = nullptr;
    int32_t* bnd_local = nullptr;
    int32_t* bnd_flat = nullptr;
    int64_t* trp = nullptr;
    int32_t* tcol = nullptr;
    float* tw = nullptr;
    int32_t* order = nullptr;
    int32_t* tperm = nullptr;
    uint32_t* first = nullptr;   // HostMeta::first_bits
    struct Plan {
        int32_t* range_rows = nullptr;
        int32_t* seg_row = nullptr;
        int64_t* seg_begin = nullptr;
        int32_t* seg_len = nullptr;
        int32_t* long_row = nullptr;
        int32_t* long_first = nullptr;
        int32_t* long_nseg = nullptr;
        int32_t* rows_sorted = nullptr;
    } fwd, bwd;
    // output layer's transposed operator restricted to train vertices (HostMeta::MaskedTranspose)
    struct Masked {
        int64_t* trp = nullptr;
        int32_t* tcol = nullptr;
        float* tw = nullptr;
        int32_t* out_row = nullptr;
        Plan plan;
        bool ready = false;
    } masked_t;
    bool ready = false;
};

struct Workspace {  // byte offsets into `scratch`
    int64_t z = 0, dy = 0, dz = 0, dga = 0, partial = 0, colpart = 0, losspart = 0, scalars = 0,
            segpart = 0;
    int64_t h = 0, gh = 0;     // transform-first layers: H = A W and its gradient, n x padded width
    // graph attention keeping its forward results (gnn_set_keep_forward): floats from `h` to the
    // H of layer l (at [l - 1]); empty otherwise (one H buffer serves every layer in turn)
    std::vector<int64_t> gat_h_off;
    // aggregate-first layers keeping their aggregate Z = S A^{l-1} (gnn_set_keep_forward): byte
    // offset of layer l's whole-graph array (n x d_{l-1}, storage type) at [l - 1], -1: not kept
    std::vector<int64_t> zkeep;
    int64_t h_floats = 0;      // size of that buffer (0: no layer transforms first); the streaming
    int64_t dyall_floats = 0;  // schedule takes it, and the kept dY rows, out of its HBM budget
    int64_t wpad = 0;          // and copies of W, W_s with rows padded to that width (2 x d_in x padded)
    int64_t wt = 0;            // bfloat16 storage: room for one transposed weight matrix
    // fp32 GraphSAGE with hidden transform-first layers: dY of every partition (n x padded width)
    // stays until the layer's second sweep, which then takes both terms of grad A^{l-1} in one
    // contraction instead of writing one and accumulating the other; -1: not needed
    int64_t dyall = -1;
    // second split-K partial region, for contractions that gnn_epoch runs on its side stream
    int64_t partial2 = 0;
    // second Z region: the resident epoch alternates between the two while the contraction of
    // the previous partition still reads the other one on the side stream
    int64_t z2 = 0;
    // graph attention: per-vertex scores and their gradients, staged boundary scores, per-entry
    // attention weights, edge-wise products, attention weights in transposed order, and the
    // (attention weight, score gradient) pairs of all heads per entry
    int64_t ssrc = 0, sdst = 0, gssrc = 0, gsdst = 0, bs = 0, att = 0, dal = 0, twatt = 0, pair = 0;
    int64_t staging_bytes = 0, scratch_bytes = 0;
};

struct StreamEngine;  // streaming.cpp
struct StorageTier;  // storage_tier.cpp

}  // namespace gnnmi

struct gnn_ctx {
    int32_t model = 0, dtype = 0, L = 0, has_bias = 1;
    int64_t hbm_budget = 0;              // 0: everything resident; else bytes of the block caches
    std::vector<int32_t> dims;
    mutable std::string err;
    bool built = false, bound = false;
    gnnmi::HostMeta M;
    gnnmi::DevMeta D;
    gnnmi::Workspace ws;
    // bound buffers.  Resident mode: all device memory.  Streaming mode: feat / act / gact are
    // pinned host memory, everything else device memory.
    const char* feat = nullptr;          // dtype of the context
    std::vector<char*> act;              // act[l-1]: dtype for l < L, fp32 for l = L
    std::vector<float*> gact;
    std::vector<const char*> w;          // W, W_s: dtype; b: fp32
    std::vector<float*> gw;
    std::vector<float*> opt_m, opt_v;    // Adam moments, bound by gnn_bind_optimizer
    std::vector<float*> master;          // bfloat16 storage: fp32 copies of W, W_s the optimizer updates
    float dropout_p = 0.f;               // training: dropout rate after hidden activations
    uint64_t dropout_seed = 0;
    int64_t dropout_epoch = 0;
    const int32_t* labels = nullptr;
    const uint8_t* mask = nullptr;
    char* staging = nullptr;
    char* scratch = nullptr;
    // whole-graph buffers of transform-first layers (set by gnn_bind): H, grad H, kept dY rows
    char* hbuf = nullptr;
    char* ghbuf = nullptr;
    float* dyall_buf = nullptr;
    // layer order: 0 = aggregate, then transform (the paper's); 1 = transform first in layers
    // where that moves fewer rows (resident schedule)
    int32_t order_mode = 0;
    bool transform_first(int32_t layer) const
    {
        if (model == GNN_GAT) return true;       // attention scores are taken from H = A W
        if (order_mode != 1) return false;
        // streaming schedule: only when the whole-graph buffers of such layers (H / grad H, kept
        // dY rows) fit into the HBM budget beside a minimal block cache; and with bfloat16 storage
        // for GCN only (the first backward sweep of a bfloat16 GraphSAGE layer writes the self
        // term into grad A^{l-1} of the partition, which the streaming sweep does not hold then)
        if (streaming() && (!stream_xf_ok || (bf16() && model != GNN_GCN))) return false;
        return wants_transform_first(layer);
    }
    // the cost rule alone
    bool wants_transform_first(int32_t layer) const
    {
        if (model == GNN_GAT) return true;
        if (order_mode != 1) return false;
        const int64_t din = dims[(size_t)layer - 1], dout = dims[(size_t)layer];
        // bfloat16 storage: rows of H must be whole 16-byte vectors; a hidden layer's self term
        // (GraphSAGE) would need an fp32 copy of its output rows, so there only the output layer
        if (bf16() && (dout % 8 != 0 || (layer < L && model != GNN_GCN))) return false;
        // Rows moved per vertex and edge: aggregating first reads rows of the input width in the
        // forward pass, again in the recompute, and writes them in the transposed pass (layers
        // >= 2); transforming first aggregates once forward and once transposed, at the output
        // width, and regathers nothing.
        return 2 * dout < din * (layer >= 2 ? 3 : 2);
    }
    // Resident schedule: the aggregation reads the boundary rows A^{l-1}[B_p[i]] itself, through
    // column indices that name rows of the whole-graph array, and no staging copy is made
    bool fuse_gather = false;
    bool gather_fused() const { return fuse_gather && !streaming() && D.gcol != nullptr; }
    // The output layer's transposed aggregation runs over the operator entries of train vertices
    // only (the gradient of the loss is zero elsewhere); the sub-operator is built by gnn_bind
    bool masked_bwd = false;
    // gnn_epoch, resident, while it walks the partitions of a backward layer in schedule order:
    // the transposed aggregation stores the rows that are first to reach their output row and
    // the target array is not zeroed beforehand (GNNMI_FIRST_TOUCH=0: zero and add as the
    // per-partition entry points do, which may be called in any order)
    bool first_touch = false;
    bool masked_transpose() const { return masked_bwd && !streaming() && model != GNN_GAT && D.masked_t.ready; }
    bool stream_xf_ok = false;               // set by update_stream_xf() once the partitions exist
    // bytes of the whole-graph buffers the transform-first layers (by the cost rule) would need
    int64_t xf_buffer_bytes(int64_t n) const
    {
        int64_t hp = 0, dyw = 0;
        for (int32_t l = 1; l <= L; ++l)
            if (wants_transform_first(l)) {
                hp = std::max<int64_t>(hp, padded(l));
                // (the streaming schedule keeps no dY rows: its second sweep takes them again)
                if (model == GNN_SAGE_MEAN && l >= 2 && l < L && !streaming()) dyw = std::max<int64_t>(dyw, padded(l));
            }
        return (n * hp * 4 + 255) / 256 * 256 + (n * dyw * 4 + 255) / 256 * 256;
    }
    // width of H rows: d_layer rounded up to whole 16-byte vectors
    int32_t padded(int32_t layer) const { return (dims[(size_t)layer] + 3) / 4 * 4; }
    // graph attention, resident: H, the scores and the attention weights of every layer stay from
    // the forward pass until the backward pass has used them (memory instead of recomputation)
    bool keep_forward = false;
    std::vector<uint8_t> att_done;       // L * k: attention weights of (layer, partition) are those of this H
    std::vector<uint8_t> z_done;         // L * k: the kept aggregate of (layer, partition) is that of this forward pass
    // where the aggregate of (layer, partition) goes: its rows of the kept whole-graph array, or
    // the per-partition scratch region
    bool keeps_z(int32_t layer) const
    {
        return keep_forward && !streaming() && model != GNN_GAT && (size_t)layer <= ws.zkeep.size() &&
               ws.zkeep[(size_t)layer - 1] >= 0;
    }
    char* z_region(int32_t layer, int32_t p) const
    {
        if (keeps_z(layer))
            return scratch + ws.zkeep[(size_t)layer - 1] + M.off[(size_t)p] * (int64_t)dims[(size_t)layer - 1] * es();
        return scratch + z_off();
    }
    // graph attention: heads of layer l at [l - 1] (empty: one head everywhere).  With several
    // heads H, grad H and the staged rows are kept head by head: head j of a layer is an array
    // of its own with head_padded(l) floats per vertex (its f = d_l / heads columns rounded up to
    // whole 16-byte vectors), the heads one after the other.
    std::vector<int32_t> heads;
    int32_t nheads(int32_t layer) const { return heads.empty() ? 1 : heads[(size_t)layer - 1]; }
    int32_t head_cols(int32_t layer) const { return dims[(size_t)layer] / nheads(layer); }
    int32_t head_padded(int32_t layer) const { return (head_cols(layer) + 3) / 4 * 4; }
    // floats of H per vertex over all heads (= padded(layer) with one head)
    int32_t hrow(int32_t layer) const { return nheads(layer) * head_padded(layer); }
    int32_t max_heads() const
    {
        int32_t m = 1;
        for (int32_t h : heads) m = std::max(m, h);
        return m;
    }
    std::vector<uint8_t> xf_fwd_done, xf_bwd_done;   // L * k: transform sweeps of such layers
    int32_t h_layer = 0;                             // layer whose H = A W the scratch buffer holds
    // schedule state
    int32_t staged_layer = -1, staged_p = -1;
    std::vector<uint8_t> fwd_done;      // L * k
    std::vector<int32_t> bwd_done;      // per layer: partitions finished since gnn_loss
    bool loss_done = false;
    gnnmi::StreamEngine* stream_engine = nullptr;
    gnnmi::StorageTier* tier = nullptr;    // storage below host memory: feat / act / gact then point into its pool
    // profiling
    int prof = 0;                       // 0 off, 1 every kernel class, 2 the aggregation classes only
    std::vector<hipEvent_t> events;
    std::vector<int> event_class;
    size_t events_used = 0;
    double prof_ms[GNN_K_COUNT] = {0};
    int64_t prof_launches[GNN_K_COUNT] = {0};
    gnn_stream_stats stream_stats{};
    // gnn_epoch, resident schedule: the contractions of a transform-first layer's own sweep run
    // on a side stream beside the neighbouring aggregate-first layer's partitions
    hipStream_t side = nullptr;
    std::vector<hipEvent_t> side_events;   // per schedule step, plus two fences
    bool on_side = false;                  // calls made for the side stream take the second partial region
    hipStream_t fwd_side = nullptr;        // set by gnn_epoch: compute_fwd puts its contraction there
    int z_slot = 0;                        // which Z region compute_fwd uses (0 outside gnn_epoch's forward)
    int64_t z_off() const { return z_slot ? ws.z2 : ws.z; }

    hipError_t deferred = hipSuccess;      // failure of a HIP call inside a void helper, reported by check_launch

    gnn_status fail(gnn_status st, const std::string& msg) const
    {
        err = msg;
        return st;
    }
    bool streaming() const { return hbm_budget != 0; }
    bool bf16() const { return dtype == GNN_BF16; }
    int64_t es() const { return dtype == GNN_BF16 ? 2 : 4; }   // bytes per stored activation/weight
    // bytes per element of act[layer-1] (the logits are always fp32)
    int64_t act_es(int32_t layer) const { return layer == L ? 4 : es(); }
    // rows [r0, ...) of the input of `layer` (A^{layer-1}), width d_{layer-1}
    const char* layer_input(int32_t layer, int64_t r0 = 0) const
    {
        const char* base = layer == 1 ? feat : act[(size_t)layer - 2];
        return base + r0 * (int64_t)dims[(size_t)layer - 1] * es();
    }
};

namespace gnnmi {

// HIP-event bracket around one kernel class (only when profiling is on).
struct Timed {
    gnn_ctx* c;
    hipStream_t s;
    bool on;
    Timed(gnn_ctx* ctx, hipStream_t st, int cls)
        : c(ctx), s(st),
          on(ctx->prof == 1 || (ctx->prof == 2 && (cls == GNN_K_SPMM || cls == GNN_K_SPMM_T)))
    {
        if (on) mark(cls);
    }
    ~Timed()
    {
        if (on) mark(-1);
    }
    void mark(int cls)
    {
        if (c->events_used == c->events.size()) {
            hipEvent_t e;
            if (hipEventCreate(&e) != hipSuccess) return;
            c->events.push_back(e);
            c->event_class.push_back(0);
        }
        c->event_class[c->events_used] = cls;
        (void)hipEventRecord(c->events[c->events_used], s);
        ++c->events_used;
    }
};

inline gnn_status check_launch(gnn_ctx* c, const char* what)
{
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && c->deferred != hipSuccess) e = c->deferred;
    c->deferred = hipSuccess;
    if (e != hipSuccess) return c->fail(GNN_EHIP, std::string(what) + ": " + hipGetErrorString(e));
    return GNN_OK;
}

// The three compute steps of one (layer, partition) pair, on explicit row blocks.  The
// resident schedule passes pointers into the caller's full arrays; the streaming schedule
// passes cache slots and transfer buffers.

// staging[run] = block[local rows] for the whole boundary list of p (resident: block = full A^{l-1})
// is done by the schedules themselves.

// A_p^l = act(Z_p W (+ X_p W_s) + b) with Z_p = S_p [in_own ; staging]; out_own has row stride d_l.
void compute_fwd(gnn_ctx* c, int32_t layer, int32_t p, const char* in_own, char* out_own, hipStream_t s);

// Activation backward, recompute of Z_p, weight/bias gradients (added into grad_w) and, for
// layer >= 2, dZ_p and the gradient of the gathered rows (left in scratch, |R_p| x d_{l-1}
// fp32), or, when fused_gprev (the full grad A^{l-1} array) is given, added straight onto its
// owner rows there (rows in library order, or as numbered by fused_map when that is given).
// Returns the dY_p block (dtype of the context; fp32 path: may alias g_own).
const char* compute_bwd(gnn_ctx* c, int32_t layer, int32_t p, const char* in_own, const float* g_own,
                        const char* act_own, float* fused_gprev, const SpmmScatter* fused_map, hipStream_t s);
// SAGE self term: gprev_own (n_p x d_{l-1} fp32) += dY_p W_s^T
void compute_bwd_self(gnn_ctx* c, int32_t layer, int32_t p, const char* dY, float* gprev_own,
                      hipStream_t s, int accumulate = 1);

// Transform-first layers on explicit row blocks (H, grad H and the kept dY rows are the
// context's whole-graph buffers): the two sweeps of the forward and of the backward pass.
void xf_transform_fwd(gnn_ctx* c, int32_t layer, int32_t p, const char* in_own, hipStream_t s);
void xf_aggregate_fwd(gnn_ctx* c, int32_t layer, int32_t p, const char* in_own, char* out_own, hipStream_t s);
void xf_begin_bwd(gnn_ctx* c, int32_t layer, hipStream_t s);
void xf_aggregate_bwd(gnn_ctx* c, int32_t layer, int32_t p, const char* in_own, const float* g_own,
                      const char* act_own, float* gprev_own, hipStream_t s);
void xf_transform_bwd(gnn_ctx* c, int32_t layer, int32_t p, const char* in_own, const float* g_own,
                      const char* act_own, float* gprev_own, hipStream_t s);

void zero_weight_grads(gnn_ctx* c, hipStream_t s);
SpmmItems plan_items(const HostMeta::Plan& H, const DevMeta::Plan& P, int32_t p);

// dropout after the activation of a hidden layer on the rows [r0, r0 + rows) (no-op when off)
void apply_dropout(gnn_ctx* c, int32_t layer, int64_t r0, int64_t rows, void* out_own, int is_bf16, hipStream_t s);

// gat.cpp: the steps of a graph-attention layer for one partition
void gat_transform_fwd(gnn_ctx* c, int32_t layer, int32_t p, hipStream_t s);
void gat_gather(gnn_ctx* c, int32_t layer, int32_t p, hipStream_t s);
void gat_layer_fwd(gnn_ctx* c, int32_t layer, int32_t p, hipStream_t s);
void gat_bwd_begin(gnn_ctx* c, int32_t layer, hipStream_t s);
void gat_layer_bwd(gnn_ctx* c, int32_t layer, int32_t p, hipStream_t s);
void gat_transform_bwd(gnn_ctx* c, int32_t layer, int32_t p, hipStream_t s);
void collect_profile(gnn_ctx* c);

// storage_tier.cpp: whole per-layer arrays in a pinned pool backed by files.  Array ids: 0..L =
// A^0..A^L, L + l = grad A^l.
gnn_status tier_open(gnn_ctx* c, const char* dir, int64_t host_budget_bytes);
void tier_close(gnn_ctx* c);
int tier_array_id(const gnn_ctx* c, int kind, int layer);    // -1: no such array
int64_t tier_array_bytes(const gnn_ctx* c, int id);
// Makes the arrays need[0..nneed) resident (bit i of overwrite_mask: need[i] is overwritten whole,
// not read) and sets feat / act / gact of the context; next[]: what the phase after reads.
// dead[]: arrays that nothing reads again in this epoch once the phase has run.
// device_idle: the caller has waited for the device since the last phase (required whenever
// tier_needs_io says that something has to be read, evicted or moved).
bool tier_needs_io(gnn_ctx* c, const int* need, int nneed);
gnn_status tier_prepare(gnn_ctx* c, const int* need, int nneed, unsigned overwrite_mask, const int* next, int nnext,
                        const int* dead, int ndead, bool device_idle);
// Arrays used without being in the pool: "virtual" host addresses and block transfers on their files.
char* tier_virtual_base(int id);
bool tier_decode(const void* p, int* id, int64_t* off);
gnn_status tier_file_read(gnn_ctx* c, int id, int64_t off, void* dst, int64_t bytes);
gnn_status tier_file_write(gnn_ctx* c, int id, int64_t off, const void* src, int64_t bytes);
void tier_epoch_begin(gnn_ctx* c);             // the arrays of the last epoch (all but the features) are stale
void tier_keep_results(gnn_ctx* c, bool keep); // false: arrays the epoch is done with are dropped, not written back
gnn_status tier_write(gnn_ctx* c, int id, const void* src);
gnn_status tier_read(gnn_ctx* c, int id, void* dst);
void tier_get_stats(const gnn_ctx* c, gnn_storage_stats* out);

// streaming.cpp
gnn_status stream_engine_create(gnn_ctx* c);
void stream_engine_destroy(gnn_ctx* c);
gnn_status epoch_streaming(gnn_ctx* c, hipStream_t s, float* loss_out);

}  // namespace gnnmi
