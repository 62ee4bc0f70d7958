/*
 * gnnmi - partition-wise full-graph GNN layer forward/backward on one MI355X (gfx950).
 *
 * C ABI of the hot path of storage-offloaded full-graph GNN training as the paper states
 * it: the graph is split into k partitions; for every layer and every destination
 * partition p the source activations the partition needs are gathered (GA_p), aggregated
 * along the partition's 1-hop topology T_p and multiplied by the shared weights; the
 * backward pass regathers instead of keeping a snapshot, recomputes the aggregate,
 * produces the gradient of the gathered rows and scatter-accumulates it onto the owners,
 * with weight gradients summed over partitions (Cache-(Re)Gather-Bypass section, gradient
 * engine section, and the overall-procedure algorithm in the appendix).  The inputs are the
 * ones that algorithm names: graph G in CSR, features F, number of partitions P (here k),
 * number of layers L, weights W^1..W^L.
 *
 * General rules
 *   - Every call returns a gnn_status; nothing throws or aborts across this boundary.
 *   - All argument checks happen before the first HIP call of an entry point.
 *   - "host" pointers are ordinary process memory, "device" pointers are HIP device memory
 *     of the current device.  `stream` is a hipStream_t passed as void*.
 *   - Layers are numbered 1..L as in the paper; A^0 is the feature matrix.
 *   - Vertex order.  The caller's graph uses *original* vertex ids.  Per-vertex DEVICE
 *     arrays (features, activations, gradients, labels, mask) are in *library order*: the
 *     vertices of partition 0 first, then partition 1, ..., ascending original id inside a
 *     partition, so that a partition's rows A_p^l are one contiguous block (the paper
 *     stores activations per partition as well).  gnn_get_order() returns the mapping and
 *     gnn_permute_rows() converts device arrays between the two orders.
 *   - The library owns only the metadata it builds (host copies and their device mirrors).
 *     Features, activations, gradients, weights, staging and scratch belong to the caller.
 */
#ifndef GNNMI_H
#define GNNMI_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gnn_ctx gnn_ctx;

typedef enum {
    GNN_OK = 0,
    GNN_EINVAL = 1,       /* bad argument (null pointer, malformed CSR, size out of range) */
    GNN_ENOMEM = 2,       /* host or device allocation failed / budget too small */
    GNN_EHIP = 3,         /* a HIP runtime call failed; see gnn_last_error() */
    GNN_ESTATE = 4,       /* call out of order (e.g. backward before forward) */
    GNN_EUNSUPPORTED = 5  /* valid request this build does not implement */
} gnn_status;

/* GNN_GAT: graph-attention layers (Velickovic et al.; the second model family of the paper's
 * evaluation): H = A^{l-1} W, e(u->v) = LeakyReLU_0.2(a_src.H[u] + a_dst.H[v]) over the sources
 * of v and v itself, softmax over the sources, A^l = act(sum alpha H[u] + b).  One head per
 * layer unless gnn_set_gat_heads says otherwise.
 * weights[3(l-1)+1] holds the two attention vectors as [2, d_l] (a_src, then a_dst), fp32.
 * GNN_F32 and the resident schedule only. */
typedef enum { GNN_GCN = 0, GNN_SAGE_MEAN = 1, GNN_GAT = 2 } gnn_model;
typedef enum { GNN_F32 = 0, GNN_BF16 = 1 } gnn_dtype; /* storage type of activations/weights */
typedef enum {
    GNN_PART_USER = 0,
    GNN_PART_RANDOM = 1,
    GNN_PART_LP = 2,
    GNN_PART_SWITCHING = 3,
    GNN_PART_SWITCHING_DEVICE = 4
} gnn_part_mode;

typedef struct {
    int32_t model;            /* gnn_model */
    int32_t dtype;            /* gnn_dtype */
    int32_t n_layers;         /* L >= 1 */
    const int32_t *dims;      /* host, L+1 entries d_0..d_L, each >= 1 (copied) */
    int32_t has_bias;         /* 0 or 1 */
    int64_t hbm_budget_bytes; /* 0 = everything resident in HBM; > 0 = streaming schedule: bytes of
                               * device memory the library may allocate for its partition-block
                               * caches (see gnn_bind) */
} gnn_config;

/* Sizes the caller needs to allocate buffers and to account traffic. */
typedef struct {
    int64_t n;            /* vertices */
    int64_t nnz;          /* entries of the aggregation operator (GCN: with one self-loop per vertex) */
    int32_t k;            /* partitions */
    int64_t sum_boundary; /* sum over p of |B_p|;  alpha = (n + sum_boundary) / n for GCN */
    int64_t sum_required; /* sum over p of |own_p u B_p| actually referenced */
    int64_t max_own;      /* largest n_p */
    int64_t max_boundary; /* largest |B_p| */
    int64_t max_nnz;      /* largest number of operator entries in one partition */
} gnn_stats;

/* Kernel classes of the profile returned by gnn_get_profile(). */
typedef enum {
    GNN_K_GATHER = 0,   /* boundary gather and regather */
    GNN_K_SPMM = 1,     /* aggregation, forward and recompute */
    GNN_K_GEMM_FWD = 2, /* Z W (+ X W_s) + b, activation */
    GNN_K_LOSS = 3,
    GNN_K_ACT_BWD = 4,  /* activation mask + bias gradient */
    GNN_K_GEMM_DW = 5,  /* Z^T dY (+ X^T dY) */
    GNN_K_GEMM_DZ = 6,  /* dY W^T (+ dY W_s^T) */
    GNN_K_SPMM_T = 7,   /* transposed aggregation */
    GNN_K_SCATTER = 8,  /* scatter-add onto owners */
    GNN_K_OTHER = 9,    /* zero fills */
    GNN_K_SPMM_REDUCE = 10, /* long-row partial sums of both aggregation directions */
    GNN_K_COUNT = 11
} gnn_kernel_class;

/* ---- lifetime -------------------------------------------------------------------------- */

/* Creates a context for one model (Algorithm "overall procedure": L, the layer widths).
 * cfg and cfg->dims are host memory, copied.  GNN_EINVAL on null/invalid fields,
 * GNN_EUNSUPPORTED for a dtype/model this build lacks.  No HIP call is made. */
gnn_status gnn_create(const gnn_config *cfg, gnn_ctx **out);

/* Frees host and device metadata.  Null is allowed. */
void gnn_destroy(gnn_ctx *ctx);

/* Message of the last failing call on this context (or, for ctx == NULL, of the last failing
 * gnn_create on this thread).  The string is owned by the library. */
const char *gnn_last_error(const gnn_ctx *ctx);

/* ---- partitions (host only; no HIP call) --------------------------------------------- */

/* Splits the graph into k partitions and builds, per partition p: the owned vertex list,
 * the boundary list B_p = cross-partition sources of p's destinations ordered by
 * (partition id, vertex id) (appendix "In-Partition Vertex Ordering"), the local 1-hop
 * topology T_p whose columns index into [own_p ; B_p], its transpose, and the
 * normalisation factors (GCN: 1/sqrt(deg(u) deg(v)) on A + I with deg = row length of
 * A + I; SAGE: 1/in-degree).
 *   n, rowptr[n+1], colidx[rowptr[n]]: host CSR by destination (row v = sources u of edges
 *     u -> v), columns strictly ascending inside a row; the arrays are only read.
 *   mode: GNN_PART_USER takes user_part[n] (values in [0,k)); GNN_PART_RANDOM ranks the
 *     vertices by (splitmix64(seed ^ splitmix64(v)), v) and deals ranks round-robin;
 *     GNN_PART_LP runs 10 synchronous rounds of first-preference label propagation with the
 *     paper's size penalty (balance factor 1.1) and capacity floor(1.1 n / k), starting
 *     from GNN_PART_RANDOM (partitioning section and its appendix);
 *     GNN_PART_SWITCHING is the complete switching-aware partitioner (same passages): from
 *     GNN_PART_RANDOM, per iteration every vertex takes a first and a second preference by
 *     that score among the partitions of its neighbours and its own, the vertices are cut
 *     into 16 contiguous ranges, and in each range, per target partition, the largest group
 *     of candidates sharing a second preference relocates, limited to the range's share of
 *     the relocation capacity floor(1.1 n / k) - |P_j|; it halts when the objective (the
 *     sum of the vertices' scores, evaluated exactly) has improved by less than 0.1 % in 5
 *     consecutive iterations, or after 50.  Deterministic for a given (graph, k, seed).
 *     GNN_PART_SWITCHING_DEVICE is the same rule with the per-vertex preference counting (the
 *     O(edges) part of every iteration) run as a kernel on the current HIP device; the
 *     assignment is identical to GNN_PART_SWITCHING.  It copies the CSR to the device for the
 *     duration of the call (8(n+1) + 4 nnz + 12 n bytes) and supports k <= 4096
 *     (GNN_EUNSUPPORTED beyond); HIP failures give GNN_EHIP.  Every other mode runs on the
 *     host alone and needs no device.
 * Errors: GNN_EINVAL (null, n < 1, k < 1, k > n, malformed CSR, bad user_part),
 * GNN_ENOMEM.  May be called again to repartition; a bound context becomes unbound. */
gnn_status gnn_build_partitions(gnn_ctx *ctx, int64_t n, const int64_t *rowptr,
                                const int32_t *colidx, int32_t k, int32_t mode, uint64_t seed,
                                const int32_t *user_part);

/* Read-back for bit-exact checks.  Returned host pointers stay valid until the next
 * gnn_build_partitions or gnn_destroy.  All ids are original vertex ids. */
gnn_status gnn_get_partition(const gnn_ctx *ctx, const int32_t **part /* n */, int32_t *k);
gnn_status gnn_get_order(const gnn_ctx *ctx, const int32_t **order /* n: original id of row r */,
                         const int64_t **part_offset /* k+1: first row of each partition */);
gnn_status gnn_get_boundary(const gnn_ctx *ctx, int32_t p, const int32_t **idx, int64_t *count);
gnn_status gnn_get_stats(const gnn_ctx *ctx, gnn_stats *out);
/* order[t], t < k: the partition gnn_epoch processes at step t of every layer pass.  Step 0
 * is partition 0; each next step takes the unprocessed partition that shares the most
 * blocks (its own and the owners of its boundary rows) with the one before, lower id among
 * equals, so that cached blocks are reused (appendix on I/O optimisations: the next target
 * is picked statically to exploit already-cached neighbours).  Callers stepping by hand may
 * use any order; sums over partitions are taken in the order of the calls. */
gnn_status gnn_get_schedule(const gnn_ctx *ctx, const int32_t **order /* k */);
/* GNN_PART_SWITCHING only (0 iterations otherwise): iterations run and, in objective[i] for
 * i <= iterations, the mean score per vertex of the state after i iterations (convergence
 * table in the appendix).  At most `capacity` values are written. */
gnn_status gnn_get_partitioner_history(const gnn_ctx *ctx, int32_t *iterations, double *objective,
                                       int32_t capacity);

/* Bytes the caller must provide as `staging` (largest |B_p| rows of the widest gathered
 * layer) and `scratch` (per-partition intermediates: aggregate Z_p, dY_p, dZ_p, gradient of
 * the gathered rows, split-K partial sums, reduction partials). */
gnn_status gnn_workspace_bytes(const gnn_ctx *ctx, int64_t *staging, int64_t *scratch);

/* ---- binding device buffers ------------------------------------------------------------ */

/* Attaches the caller's device buffers (all in library order) and uploads the metadata to
 * the current device on first use.
 *   feat            [n, d_0]   A^0, dtype of the context
 *   act[l-1]        [n, d_l]   A^l for l = 1..L (A^L = logits is always fp32)
 *   grad_act[l-1]   [n, d_l]   dLoss/dA^l, fp32, for l = 1..L
 *   weights[3*(l-1) + 0]  W^l   [d_{l-1}, d_l] row-major (GCN weight / SAGE neighbour weight)
 *   weights[3*(l-1) + 1]  W_s^l same shape, SAGE only (else ignored, may be null)
 *   weights[3*(l-1) + 2]  b^l   [d_l] fp32, when has_bias (else ignored, may be null)
 *   grad_w          same layout as weights, always fp32
 *   labels [n] int32 in [0, d_L);  train_mask [n] uint8
 *   staging, scratch: at least gnn_workspace_bytes(), 256-byte aligned
 *   feat, act[], grad_act[], the weight matrices and their gradients must be 16-byte aligned
 *   (GNN_EINVAL otherwise): rows are read and written as 16-byte vectors
 * The pointer arrays themselves are host memory and are copied.
 *
 * Streaming schedule (hbm_budget_bytes > 0; the one-GPU analogue of the paper's partition-wise
 * cache with copy/compute overlap): feat, act[] and grad_act[] are PINNED HOST buffers of the
 * same shapes and order; everything else stays device memory.  The library then allocates
 * hbm_budget_bytes of device memory as a cache of whole per-layer arrays while they fit and of
 * single partition blocks otherwise (layer l-1 activations, the block whose next use lies
 * furthest ahead is evicted; gradient blocks of layer l-1 as a write-back cache) plus six
 * transfer buffers of max n_p x max d_l x 4 bytes and two side streams, all freed by
 * gnn_destroy or the next gnn_build_partitions.  Only gnn_epoch runs in this mode (the
 * per-partition entry points return GNN_EUNSUPPORTED), at most 4096 partitions, and the budget
 * must hold two activation blocks and two gradient blocks of the widest layer (GNN_ENOMEM
 * otherwise).  When the host buffers are mapped for the device (hipHostMalloc, or torch's
 * pin_memory: hipPointerGetAttributes reports a device pointer), boundary rows of blocks that
 * are not cached are read by the gather kernel directly from them; with host memory that is
 * not mapped every miss loads its whole block.  Results are bit-identical to the resident
 * schedule either way.
 *
 * Errors: GNN_ESTATE before gnn_build_partitions, GNN_EINVAL on a null entry,
 * GNN_EHIP / GNN_ENOMEM if the upload or an allocation fails. */
gnn_status gnn_bind(gnn_ctx *ctx, const void *feat, void *const *act, void *const *grad_act,
                    const void *const *weights, void *const *grad_w, const int32_t *labels,
                    const uint8_t *train_mask, void *staging, void *scratch);

/* dst[r] = src[order[r]] (to_library_order = 1) or dst[order[r]] = src[r] (= 0) for n rows
 * of row_bytes bytes each.  src and dst are device buffers, or pinned host buffers mapped for
 * the device (hipHostMalloc; the kernel then moves the rows over the host link), and must not
 * overlap.  Any alignment is accepted; rows are moved in 16-byte vectors when row_bytes and both
 * addresses are multiples of 16, in narrower units otherwise. */
gnn_status gnn_permute_rows(gnn_ctx *ctx, const void *src, void *dst, int64_t row_bytes,
                            int32_t to_library_order, void *stream);

/* dst[i] = bfloat16(src[i]), round to nearest even, for count elements: how fp32 inputs and
 * weights are put into GNN_BF16 storage (once, before the first epoch).  src (fp32) and dst
 * (raw 16-bit) are device buffers or pinned host buffers mapped for the device. */
gnn_status gnn_to_bf16(gnn_ctx *ctx, const float *src, void *dst, int64_t count, void *stream);

/* ---- the hot path (enqueue on `stream`, do not synchronise) ---------------------------- */

/* Gather / regather: staging[i, :] = A^{layer-1}[B_p[i], :], a bit copy of |B_p| rows
 * (step "GA_p^{l-1} <- Gather(A^{l-1})" of the overall procedure; the same call serves the
 * backward regather of the gradient engine).  GNN_EINVAL for layer outside 1..L or p outside
 * 0..k-1, GNN_ESTATE when unbound. */
gnn_status gnn_gather_boundary(gnn_ctx *ctx, int32_t layer, int32_t p, void *stream);

/* Gather fused into the aggregation (resident schedule).  The gather
 * step exists because A^{l-1} lives outside device memory and only the rows a partition needs
 * are brought in; when A^{l-1} is resident the staging copy is one read and one write of every
 * boundary row on top of the aggregation's own reads of it.  With on = 1 the aggregation
 * kernels take row B_p[i] of A^{l-1} (of H for a transform-first layer) where they would take
 * row i of staging: the operator's column indices are kept a second time as rows of the
 * whole-graph array (4 bytes per operator entry of device memory, allocated by this call or by
 * the next gnn_bind and kept until gnn_destroy).  gnn_gather_boundary then launches nothing and
 * only records which (layer, partition) the following gnn_layer_fwd / gnn_layer_bwd may work
 * on; staging is not written.  Every sum takes its terms in the same order, so all results are
 * the bits of the staged path.  GNN_GAT: the attention passes, the aggregation and the edge-wise
 * products read the rows of H and the scores of boundary vertices the same way.  Default 0 (the
 * paper's step, through staging).  The setting has no effect with a streaming budget
 * (gnn_gather_is_fused reports 0 there).
 * GNN_EINVAL for on outside {0, 1}, GNN_ENOMEM / GNN_EHIP if the index array cannot be set up. */
gnn_status gnn_set_gather_fusion(gnn_ctx *ctx, int32_t on);
/* Backward pass of the output layer over train vertices only (resident schedule, GNN_GCN and
 * GNN_SAGE_MEAN).  The gradient of the loss is zero in every row outside train_mask, so the
 * output layer's transposed aggregation (grad of the gathered rows, scatter-accumulated onto
 * their owners) needs only the operator entries whose destination is a train vertex.  With
 * on = 1, gnn_bind (or this call, on a bound context) copies train_mask to the host once and
 * builds that sub-operator of every partition's transpose: kept entries in their original
 * order, rows left without an entry dropped (about 12 bytes of device memory per kept entry).
 * The entries left out multiply rows that are exactly zero, so results differ from on = 0
 * only by the order in which the kept terms of a long row are added (rounding).  The caller
 * promises not to change the contents of train_mask while the context is bound to it (bind
 * again after changing it).  Default 0.  No effect with a streaming budget, with GNN_GAT, or
 * when the scatter-accumulate is not fused into the aggregation.
 * GNN_EINVAL for on outside {0, 1}; GNN_ENOMEM / GNN_EHIP if the sub-operator cannot be set up. */
gnn_status gnn_set_masked_backward(gnn_ctx *ctx, int32_t on);
/* Size of that sub-operator over all partitions: operator entries kept and rows of the gathered-row
 * gradient that receive a sum; both 0 while it is not in use. */
gnn_status gnn_get_masked_backward_size(const gnn_ctx *ctx, int64_t *entries, int64_t *rows);
/* *out = 1 when the aggregation kernels of this context read the boundary rows themselves. */
gnn_status gnn_gather_is_fused(const gnn_ctx *ctx, int32_t *out);

/* A_p^l <- FW(W^l, GA_p^{l-1}, T_p): aggregation over the partition's topology reading own
 * rows in place and boundary rows from staging, then the transform, bias and (l < L) ReLU,
 * written to the partition's rows of act[l-1].  GNN_ESTATE unless staging holds
 * (layer, p). */
gnn_status gnn_layer_fwd(gnn_ctx *ctx, int32_t layer, int32_t p, void *stream);

/* Mean softmax cross-entropy over the train mask on A^L and its gradient into
 * grad_act[L-1] (rows outside the mask get zero).  Starts a new backward pass: weight
 * gradients are NOT cleared here (gnn_epoch clears them; a caller stepping by hand clears
 * grad_w itself).  The scalar loss stays on the device until gnn_read_loss(). */
gnn_status gnn_loss(gnn_ctx *ctx, void *stream);
/* For callers that cannot allocate or hand over a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): gnn_loss with the mask count and the
 * block partial sums kept in a 4 MiB device array the library holds statically, one copy per
 * GPU for the life of the process, instead of in the bound scratch.  No hipMalloc / hipFree and
 * no allocating routine is called.  Inputs and outputs are the bound ones (A^L, labels, mask ->
 * grad_act[L-1]); the scalar loss is written to loss_dev (device, one float, caller owned) on
 * `stream`; gnn_read_loss does not see it.  Same kernels and summation order as gnn_loss, so the
 * results are the same bits.  Limit: n / 64 + k + 2 <= 1,048,512 (about 67 million vertices):
 * GNN_EINVAL beyond, with a message.
 * Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (two
 * streams, two contexts, two threads) race; calls in sequence are fine, nothing is carried from
 * one call to the next.  Other errors as gnn_loss; GNN_EHIP if the array's address cannot be
 * obtained. */
gnn_status gnn_loss_static(gnn_ctx *ctx, void *stream, float *loss_dev);
/* Synchronises `stream` and returns the last loss of gnn_loss. */
gnn_status gnn_read_loss(gnn_ctx *ctx, void *stream, float *loss_out);

/* (grad GA_p^{l-1}, grad W^l) <-(., +) BW(W^l, A_p^l, grad A_p^l, GA_p^{l-1}): activation
 * mask, recomputed aggregate from the regathered staging, weight/bias gradients ADDED into
 * grad_w, and for layer >= 2 the gradient of the gathered rows scatter-accumulated into
 * grad_act[layer-2].  The first backward call of a layer since gnn_loss zeroes
 * grad_act[layer-2] (the write-back buffer initialisation of the overall procedure).
 * Partitions of one layer must be issued on one stream (the accumulation relies on stream
 * order, not atomics).  GNN_ESTATE unless staging holds (layer, p), the forward pass and
 * gnn_loss have run, and layer+1 has finished its backward. */
gnn_status gnn_layer_bwd(gnn_ctx *ctx, int32_t layer, int32_t p, void *stream);

/* One epoch: forward over all layers and partitions, loss, backward; grad_w is overwritten.
 * Synchronises `stream` before writing *loss_out (host).  Resident schedule, fp32 GCN /
 * GraphSAGE: the forward contraction of an aggregate-first layer below another one, and where
 * such a layer lies below a transform-first one that layer's contractions of its own sweep, run on a stream
 * the context owns, beside the gathers and aggregations of the other partitions, ordered
 * against `stream` by events only (so `stream` may be the null stream or
 * any other); results are the one-stream schedule's bits.  Everything the epoch launched has
 * finished when the call returns. */
gnn_status gnn_epoch(gnn_ctx *ctx, void *stream, float *loss_out);

/* ---- layer order ------------------------------------------------------------------------ */

/* The paper's layers aggregate the gathered rows and then transform them.  Aggregation and
 * transform commute (S (A W) = (S A) W), so a layer whose output is narrower than its input
 * moves fewer bytes when it transforms first: H = A^{l-1} W per partition, then gather,
 * aggregate and scatter-accumulate at the output width, with no regather and no recompute in
 * the backward pass (it needs only the partition's own rows of A^{l-1} and the gradient of H).
 *   GNN_ORDER_AGGREGATE_FIRST (default): every layer as in the paper.
 *   GNN_ORDER_AUTO: a layer transforms first when that moves fewer rows: 2 d_l < 3 d_{l-1}
 *     (layer 1, which needs no input gradient: 2 d_l < 2 d_{l-1}); aggregating first reads
 *     input-wide rows forward, again in the recompute and once more transposed, transforming
 *     first aggregates output-wide rows once forward and once transposed.  With GNN_BF16
 *     only layers whose output rows are whole 16-byte vectors (d_l a multiple of 8), and
 *     among the hidden layers only those of GNN_GCN.  Streaming schedule (hbm_budget_bytes >
 *     0): only when the budget holds the whole-graph buffer of such layers (n rows of their
 *     widest padded output, fp32) beside two whole per-layer arrays of the widest layer and
 *     the smallest block cache, and with GNN_BF16 for GNN_GCN only.  Other layers and
 *     configurations keep the paper's order.
 * Changes the workspace sizes: call before gnn_workspace_bytes / gnn_bind (a bound context
 * becomes unbound).  Results differ from the other order only by rounding. */
typedef enum { GNN_ORDER_AGGREGATE_FIRST = 0, GNN_ORDER_AUTO = 1 } gnn_layer_order;
gnn_status gnn_set_layer_order(gnn_ctx *ctx, int32_t mode);
gnn_status gnn_layer_is_transform_first(const gnn_ctx *ctx, int32_t layer, int32_t *out);

/* Stepping a transform-first layer by hand (gnn_epoch does the same):
 *   forward:  gnn_layer_transform_fwd(layer, p) for every p   (H_p = A_p^{l-1} W^l), then for
 *             every p gnn_gather_boundary(layer, p) (gathers rows of H) and
 *             gnn_layer_fwd(layer, p)  (A_p^l = act(S_p [H_own ; staging] (+ A_p^{l-1} W_s) + b));
 *   backward: gnn_layer_bwd(layer, p) for every p, without a gather (dY_p, grad b, grad W_s,
 *             grad A^{l-1}_own += dY_p W_s^T, grad H [R_p] += S_p^T dY_p), then
 *             gnn_layer_transform_bwd(layer, p) for every p (grad W += A_p^{l-1 T} grad H_p,
 *             grad A^{l-1}_own += grad H_p W^T) before layer-1 starts.
 * One scratch buffer holds H for the layer being worked on: starting the transform sweep of
 * another layer invalidates it.  Graph-attention layers (GNN_GAT) always transform first and
 * their backward pass needs H, the scores and the gathered rows again: for such a layer call
 * gnn_layer_transform_fwd for every p once more before its backward sweep (unless H still
 * holds this layer), and gnn_gather_boundary(layer, p) before each gnn_layer_bwd(layer, p).
 * GNN_ESTATE when the layer aggregates first or a sweep is incomplete. */
gnn_status gnn_layer_transform_fwd(gnn_ctx *ctx, int32_t layer, int32_t p, void *stream);
gnn_status gnn_layer_transform_bwd(gnn_ctx *ctx, int32_t layer, int32_t p, void *stream);

/* Attention heads of one GNN_GAT layer (the paper's evaluation of graph attention names no head
 * count; the layer is the published one, whose hidden layers concatenate their heads).  With
 * `heads` = h the layer's d_l output columns are h groups of f = d_l / h: head j takes its own
 * attention weights from columns [j f, (j + 1) f) of H = A^{l-1} W and of a_src, a_dst, aggregates
 * those columns of H with them, and writes those columns of the output row (concatenation; the
 * bias and the activation act on the whole row).  The shapes of W ([d_{l-1}, d_l]), of the
 * attention vectors ([2, d_l]) and of every activation and gradient array stay as they are.
 * The staged rows of such a layer are head-major (head j: |B_p| rows of f floats rounded up to
 * whole 16-byte vectors).  Changes the workspace sizes: call before gnn_workspace_bytes /
 * gnn_bind (a bound context becomes unbound).  GNN_EINVAL for another model, a layer outside
 * 1..L, or a head count outside 1..64 or not dividing d_l. */
gnn_status gnn_set_gat_heads(gnn_ctx *ctx, int32_t layer, int32_t heads);

/* Resident schedule: keep what the forward pass computed for the backward pass.  The paper's
 * backward pass regathers and recomputes (gradient engine: activation regathering, snapshot
 * avoided) because device memory is what its hierarchy is short of; with on = 1 the context keeps,
 * inside `scratch`,
 *   GNN_GCN, GNN_SAGE_MEAN: the aggregate Z = S A^{l-1} of every layer that aggregates first (n
 *     rows of d_{l-1} elements of the storage type per such layer); gnn_layer_bwd of such a layer
 *     then needs no gnn_gather_boundary before it and aggregates nothing again (gnn_epoch
 *     regathers nothing there);
 *   GNN_GAT: H = A^{l-1} W and the scores of every layer (n rows of the layer's width each,
 *     instead of one buffer serving every layer in turn) and the attention weights of every layer
 *     and partition (4 bytes per operator entry, head and layer), so that gnn_epoch does not run
 *     gnn_layer_transform_fwd again before a layer's backward sweep and gnn_layer_bwd does not
 *     recompute the attention weights.
 * Kept values are the values the recomputation would give: every result has the same bits.  A
 * partition's kept values are those of its latest gnn_layer_fwd (attention: until the next
 * gnn_layer_transform_fwd of that layer); a backward pass that finds none recomputes as without
 * the switch.  Default 0 (the paper's rule).  Changes the workspace sizes: call before
 * gnn_workspace_bytes / gnn_bind (a bound context becomes unbound).  No effect with a streaming
 * budget.  GNN_EINVAL for on outside {0, 1}. */
gnn_status gnn_set_keep_forward(gnn_ctx *ctx, int32_t on);

/* ---- training around the epoch (datasets table: learning rate, dropout, epochs) ---------- */

/* Dropout with rate p in [0, 1) after the activation of every hidden layer in the epochs
 * that follow; p = 0 (the default) switches it off.  The paper fixes only the rate.  The
 * draws are counter-based, so nothing is stored for the backward pass (the dropped elements
 * are the zeros of the stored activation) and the result does not depend on the
 * partitioning: element (v, j) of hidden layer l (1-based; v an original vertex id, d the
 * layer's width) draws splitmix64(key + v d + j) >> 32 with
 * key = splitmix64(seed ^ splitmix64(64 epoch_index + l)) and is zeroed when the draw is
 * below floor(p 2^32), otherwise multiplied by 1 / (1 - p) in fp32.  GNN_EINVAL outside
 * [0, 1). */
gnn_status gnn_set_dropout(gnn_ctx *ctx, float p, uint64_t seed, int64_t epoch_index);

typedef enum { GNN_OPT_SGD = 0, GNN_OPT_ADAM = 1 } gnn_opt_kind;
typedef struct {
    int32_t kind;        /* gnn_opt_kind */
    float lr;
    float beta1, beta2;  /* Adam */
    float eps;           /* Adam */
    float weight_decay;  /* added to the gradient as weight_decay * w */
} gnn_optimizer;

/* Adam moment buffers (device, fp32, zeroed by the caller before the first step), laid out
 * like `weights` in gnn_bind: 3 L entries, null where the tensor does not exist.  Caller
 * owned.  Not needed for GNN_OPT_SGD. */
gnn_status gnn_bind_optimizer(gnn_ctx *ctx, void *const *m, void *const *v);

/* GNN_BF16 only (datasets table: the paper trains in one precision and says nothing of mixed
 * storage; this is the usual arrangement): fp32 master copies of the weight matrices W and W_s
 * (device, caller owned, laid out like `weights` in gnn_bind: 3 L entries, the bias entries
 * are ignored, null where the matrix does not exist).  The caller fills them with the values
 * whose bfloat16 rounding it bound as `weights`.  GNN_EUNSUPPORTED for GNN_F32, GNN_EINVAL for
 * a missing or misaligned (4 bytes) copy. */
gnn_status gnn_bind_master_weights(gnn_ctx *ctx, void *const *master);

/* One optimizer step from grad_w (as left by the last epoch); `step` is the 1-based step
 * number (Adam's bias correction).  GNN_F32: the bound weight buffers are updated in place.
 * GNN_BF16: the step is taken in fp32 on the master copies (weight decay uses the master
 * value), and each bound matrix receives the round-to-nearest-even bfloat16 of its updated
 * master; biases are fp32 and updated in place.  GNN_ESTATE when nothing is bound, for Adam
 * without moments, for GNN_BF16 without master copies. */
gnn_status gnn_optimizer_step(gnn_ctx *ctx, const gnn_optimizer *opt, int64_t step, void *stream);

/* `epochs` times: gnn_set_dropout(p, seed, first_epoch + e), gnn_epoch, gnn_optimizer_step
 * with step first_epoch + e + 1; losses[e] (host) receives each epoch's loss.  Leaves
 * dropout configured for the last epoch. */
gnn_status gnn_train(gnn_ctx *ctx, const gnn_optimizer *opt, int32_t epochs, int64_t first_epoch,
                     float dropout_p, uint64_t dropout_seed, void *stream, float *losses);

/* ---- measurement ------------------------------------------------------------------------ */

/* When enabled, every kernel class of gnn_epoch is bracketed by HIP events on `stream`
 * (GNN_K_GATHER, GNN_K_SPMM, GNN_K_SPMM_T and GNN_K_SCATTER brackets hold exactly one kernel);
 * after the epoch gnn_get_profile() returns, per kernel class, the summed duration in
 * milliseconds and the launch count of the last epoch.  `enabled` = 2 brackets only the
 * aggregation kernels (GNN_K_SPMM, GNN_K_SPMM_T; the other classes then report zero).  Every
 * bracket costs two event packets on the stream, about 10 us of idle time between two kernels:
 * 1 adds 4-6 % to an epoch of some 800 launches, 2 about 1 %; 0 for plain wall-clock timing.
 * Other values: GNN_EINVAL. */
gnn_status gnn_set_profiling(gnn_ctx *ctx, int32_t enabled);
gnn_status gnn_get_profile(const gnn_ctx *ctx, double *ms /* GNN_K_COUNT */,
                           int64_t *launches /* GNN_K_COUNT */);

/* Traffic of the last streaming-schedule epoch (partition-wise cache; appendix on I/O
 * optimisations): block loads host -> HBM and cache hits of the activation cache and of the
 * gradient write-back cache, gradient blocks written back, and the bytes both directions
 * moved in total (cache traffic plus the per-partition transfer buffers).  All zero after a
 * resident epoch.  GNN_EINVAL on null arguments. */
typedef struct {
    int64_t act_loads, act_hits;
    int64_t grad_loads, grad_hits, grad_writebacks;
    int64_t h2d_bytes, d2h_bytes;
    int64_t direct_gathers; /* (partition, source block) pairs whose boundary rows a kernel read */
    int64_t direct_bytes;   /* straight from the pinned host array, and their bytes (in h2d_bytes) */
    int64_t direct_scatters;      /* (partition, owner block) pairs whose gradient rows a kernel added */
    int64_t direct_scatter_bytes; /* straight in the pinned host array; bytes read + written (in h2d/d2h_bytes) */
} gnn_stream_stats;
gnn_status gnn_get_stream_stats(const gnn_ctx *ctx, gnn_stream_stats *out);

/* ---- storage tier below host memory (streaming schedule) -------------------------------- */

/* The paper keeps activations and gradients on storage and caches them in host memory: whole
 * layers while they fit, whole layers evicted in least-recently-used order when they do not, and
 * partition granularity below that (partition-wise cache management section).
 * gnn_storage_open gives a context with a streaming budget (hbm_budget_bytes > 0) that tier:
 * every per-layer array (the features A^0, A^1..A^L, grad A^1..grad A^L, rows in library order)
 * gets a file in `dir` (created at full size; removed again by gnn_storage_close / gnn_destroy),
 * and the library allocates one pinned host pool of host_budget_bytes in which it keeps whole
 * arrays.  Before each phase of gnn_epoch (a layer's forward pass, the loss, a layer's backward
 * pass) the arrays that phase reads or writes are made resident: read from their file unless the
 * phase overwrites them completely, evicting the least recently used arrays that the phase does
 * not need (written to their file first when they changed).  A helper thread reads the next
 * phase's arrays ahead.  When the pool cannot hold a phase's arrays together, room goes to the
 * gather source first, then to the gradient being accumulated, and an array left without room
 * is not cached in host memory at all during that phase: its partition blocks travel between
 * file and device through small pinned buffers as the schedule loads and stores them, and are
 * reused in the HBM block cache only.  The streaming schedule itself is unchanged (HBM caches
 * blocks of whatever the host level holds), so results are the resident schedule's bits with any
 * pool size.
 *
 * Call after gnn_build_partitions and before gnn_bind; gnn_bind then ignores feat, act and
 * grad_act (pass NULL).  The features go in with gnn_storage_write(ctx, 0, 0, src) and results
 * come out with gnn_storage_read; both move one whole array between the tier and ordinary host
 * memory of the caller (kind 0: A^layer, layer 0..L, storage type of the context, logits fp32;
 * kind 1: grad A^layer, layer 1..L, fp32).  Host file I/O is synchronous on the calling thread
 * apart from the helper thread's read-ahead.
 * GNN_ESTATE without partitions or without a streaming budget; GNN_EINVAL for a pool below 4096
 * bytes or when a file cannot be created; GNN_ENOMEM when the pool or the files cannot be
 * allocated; GNN_EHIP for a failed read or write (message in gnn_last_error). */
gnn_status gnn_storage_open(gnn_ctx *ctx, const char *dir, int64_t host_budget_bytes);
gnn_status gnn_storage_close(gnn_ctx *ctx);
/* What happens to an array that leaves the pool after the epoch has read it for the last time
 * (A^l and grad A^l once layer l's backward pass has run, the logits once the loss has).
 * on = 1 (default): it is written to its file like any other, so gnn_storage_read returns every
 * activation and gradient of the last epoch.  on = 0: it is dropped - a training loop reads only
 * the weight gradients, and the next epoch overwrites these arrays before it reads them;
 * gnn_storage_read of a dropped array returns zeros.  (The contents an epoch finds in these
 * arrays when it starts are never written back in either mode.) */
gnn_status gnn_storage_keep_results(gnn_ctx *ctx, int32_t on);
gnn_status gnn_storage_write(gnn_ctx *ctx, int32_t kind, int32_t layer, const void *src_host);
gnn_status gnn_storage_read(gnn_ctx *ctx, int32_t kind, int32_t layer, void *dst_host);
typedef struct {
    int64_t host_pool_bytes; /* size of the pinned pool */
    int64_t array_bytes;     /* all arrays together */
    int64_t loads, hits;     /* arrays read from their file / found in the pool when a phase asked */
    int64_t prefetched;      /* of the loads: read ahead by the helper thread */
    int64_t evictions, writebacks;
    int64_t bytes_read, bytes_written; /* file traffic since gnn_storage_open */
    int64_t compactions;     /* times the arrays in the pool were moved together to join free room */
    int64_t dropped;         /* arrays that left the pool unwritten (gnn_storage_keep_results(0)) */
    int64_t bypassed;        /* (phase, array) pairs worked on in the file, block by block, for want of room */
    int64_t bypass_bytes;    /* file bytes of those block transfers (part of bytes_read / bytes_written) */
} gnn_storage_stats;
gnn_status gnn_get_storage_stats(const gnn_ctx *ctx, gnn_storage_stats *out);

#ifdef __cplusplus
}
#endif
#endif /* GNNMI_H */
