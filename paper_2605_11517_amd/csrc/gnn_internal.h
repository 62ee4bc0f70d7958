// Internal declarations shared by the host code and the kernel launchers of libgnnmi.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <string>
#include <vector>

#include "gnnmi.h"

namespace gnnmi {

// Host-side partition metadata.  "row" always means a vertex in library order
// (partition-major, ascending original id inside a partition).
struct HostMeta {
    int64_t n = 0;
    int32_t k = 0;
    int model = 0;
    std::vector<int32_t> part;      // original id -> partition
    std::vector<int32_t> order;     // row -> original id
    std::vector<int32_t> newid;     // original id -> row
    std::vector<int64_t> off;       // k+1, first row of each partition
    // aggregation operator S, rows in library order; partition p owns entries
    // [rp[off[p]], rp[off[p+1]])
    std::vector<int64_t> rp;        // n+1
    std::vector<int32_t> lcol;      // local column: < n_p -> own row, else n_p + index into B_p
    std::vector<float> ew;          // per-entry weight (GCN); empty for SAGE
    std::vector<float> rscale;      // per-row scale applied after the sum (SAGE: 1/deg); empty for GCN
    // boundary lists
    std::vector<int64_t> boff;      // k+1
    std::vector<int32_t> bnd;       // rows (library order), ascending inside a partition
    std::vector<int32_t> bnd_orig;  // same entries as original ids
    // only when the streaming schedule is requested: B_p split by source partition
    std::vector<int32_t> bnd_local; // row inside its source partition's block
    std::vector<int64_t> brun;      // k * (k+1): brun[p*(k+1)+q] = first entry of B_p owned by q
    std::vector<int32_t> bnd_flat;  // source partition * max_own + row inside its block (arrays whose
                                    // blocks are max_own rows apart); empty if that overflows int32
    // transpose of S per partition: rows are the entries of R_p = [own_p ; B_p]
    std::vector<int64_t> toff;      // k+1, offset of partition p's rows in trp
    std::vector<int64_t> trp;       // sum |R_p| + 1, positions into tcol / tw
    std::vector<int32_t> tcol;      // local destination row (0 .. n_p)
    std::vector<float> tw;          // weight of the entry (GCN, SAGE)
    std::vector<int32_t> tperm;     // GAT: position of the entry in the forward operator, minus the
                                    // partition's first position
    std::vector<int32_t> sched;     // k: order in which an epoch walks the partitions
    // Walking the partitions in that order, which rows of the transposed operator (own rows, then
    // B_p) are the first to name their row of the whole-graph array: bit r of partition p's words
    // (first_off[p] .. first_off[p + 1]) is set for such a row.  An epoch lets them store where
    // the others add, and then needs no zeroed array to add onto.
    std::vector<uint32_t> first_bits;
    std::vector<int64_t> first_off;  // k+1, in 32-bit words
    gnn_stats stats{};
    int32_t part_iterations = 0;          // switching-aware partitioner: iterations run
    std::vector<double> part_objective;   // and the mean score per vertex of every state
    // work decomposition of the aggregation kernels (forward operator and its transpose)
    struct Plan {
        std::vector<int64_t> range_off;   // k+1, offsets into range_rows (partition p has
                                          // range_off[p+1]-range_off[p] boundaries = ranges + 1)
        std::vector<int32_t> range_rows;  // local row boundaries of consecutive row ranges
        std::vector<int64_t> seg_off;     // k+1, offsets into the seg_* arrays
        std::vector<int32_t> seg_row;     // local row a segment belongs to
        std::vector<int64_t> seg_begin;   // first entry (absolute position)
        std::vector<int32_t> seg_len;     // entries in the segment
        std::vector<int64_t> long_off;    // k+1, offsets into long_*
        std::vector<int32_t> long_row;    // local row split into segments
        std::vector<int32_t> long_first;  // its first segment (index local to the partition)
        std::vector<int32_t> long_nseg;   // its number of segments
        int64_t max_segs = 0;             // most segments in any partition
        std::vector<int64_t> rows_off;    // k+1, offsets into rows_sorted
        std::vector<int32_t> rows_sorted; // short rows (local ids) by entry count, longest first
    } plan_fwd, plan_bwd;
    // Transposed operator of the output layer restricted to train vertices (see
    // build_masked_transpose): per partition the rows of R_p that keep at least one entry.
    struct MaskedTranspose {
        std::vector<int64_t> toff;      // k+1, offset of partition p's kept rows in trp / out_row
        std::vector<int64_t> trp;       // kept rows + 1, positions into tcol / tw
        std::vector<int32_t> tcol;      // local destination row (a train vertex of the partition)
        std::vector<float> tw;
        std::vector<int32_t> out_row;   // per kept row: the row of the whole-graph array it adds to
        Plan plan;
        bool ready = false;
    } masked_t;
};

// Rows with more entries than this are cut into segments of this many entries, each handled
// by its own wavefront; shorter rows are grouped into ranges of about this many entries.
constexpr int32_t kSpmmSegment = 512;
constexpr int32_t kSpmmRangeRows = 64;

// Builds everything above.  Returns GNN_OK or an error with `err` set.
gnn_status build_host_meta(int model, int64_t n, const int64_t* rowptr, const int32_t* colidx,
                           int32_t k, int32_t mode, uint64_t seed, const int32_t* user_part,
                           bool want_runs, HostMeta& out, std::string& err);

// The gradient of the loss is zero in every row outside the train mask, so the transposed
// aggregation of the output layer needs only the operator entries whose destination is a train
// vertex.  Builds that sub-operator of every partition's transpose from M and the mask (rows in
// library order): kept entries in their original order, rows without a kept entry dropped, the
// owner row of every kept row, and the work items.  Throws std::bad_alloc.
void build_masked_transpose(HostMeta& M, const uint8_t* mask);

// ---- kernel launchers (all enqueue on `s`; sizes already validated by the caller) --------

// dst[i,:] = src[idx[i],:] for `rows` rows of row_bytes bytes.
void launch_gather_rows(const void* src, const int32_t* idx, void* dst, int64_t rows,
                        int64_t row_bytes, hipStream_t s);
// dst[idx[i],:] = src[i,:]
void launch_scatter_rows(const void* src, const int32_t* idx, void* dst, int64_t rows,
                         int64_t row_bytes, hipStream_t s);

// out[r,:] = rowscale[r] * sum_e w[e] * src(col[e])[:],  e in [rp[r], rp[r+1])
// src(c) = a_rows + c*d if c < n_a else b_rows + (c - n_a)*d.  w / rowscale may be null (= 1).
// rp points at the first row's entry of a global row-pointer array; col / w are indexed with
// the absolute positions stored in rp.  The work is cut into items by a Plan: row ranges
// (short rows, written directly) and segments of long rows (partial sums into `partial`,
// one row of d floats per segment, combined in segment order by a second kernel).
struct SpmmItems {
    const int32_t* range_rows = nullptr;   // nranges + 1 local row boundaries
    int64_t nranges = 0;
    const int32_t* seg_row = nullptr;
    const int64_t* seg_begin = nullptr;
    const int32_t* seg_len = nullptr;
    int64_t nsegs = 0;
    const int32_t* long_row = nullptr;
    const int32_t* long_first = nullptr;
    const int32_t* long_nseg = nullptr;
    int64_t nlong = 0;
    const int32_t* rows_sorted = nullptr;  // short rows, longest first (column-sliced kernel)
    int64_t nshort = 0;
    float avg_len = 0.f;                   // entries per row of this operator block (0: not known)
};
// Optional fused scatter-accumulate for fp32 outputs: instead of out[r,:] = value, the kernel
// does out[map(r),:] += value with map(r) = base_row + r for r < n_own and idx[r - n_own]
// otherwise.  n_own < 0 switches it off.
struct SpmmScatter {
    int64_t n_own = -1;
    int64_t base_row = 0;
    const int32_t* idx = nullptr;
    // optional: bit r set = row r is stored, not added (its output row holds nothing yet)
    const uint32_t* first = nullptr;
    // applied to what is stored (after the add, if any): + bias[column], then max(., 0)
    const float* bias = nullptr;
    int relu = 0;
};
// a_rows / b_rows hold fp32 (in_bf16 = 0) or bfloat16 rows; out is fp32 or bfloat16; the sums
// and `partial` are always fp32.  ld (0: d): the rows of a_rows, b_rows, out and partial start ld
// elements apart and the call works on d of their columns (a column block of wider arrays).
void launch_spmm(const int64_t* rp, const int32_t* col, const float* w, const float* rowscale,
                 const void* a_rows, int64_t n_a, const void* b_rows, void* out, int64_t nrows,
                 int32_t d, int in_bf16, int out_bf16, const SpmmItems& items, float* partial,
                 int column_slices /* allow the XCD column-sliced kernel */, const SpmmScatter& sc,
                 hipStream_t s, int32_t ld = 0);
// The heads of a multi-head aggregation in one launch (fp32): rows of ld = nh f floats, column
// block j of f floats weighted by the entry weights w + j wss; otherwise as launch_spmm (the long
// rows' partial sums are combined by launch_spmm_reduce over all ld columns).  Returns false and
// launches nothing when f is not 16, 32, 64 or 128 floats or the plan lists no short rows: the
// caller then aggregates head by head.
bool launch_spmm_heads(const int64_t* rp, const int32_t* col, const float* w, int64_t wss, int32_t nh, int32_t f,
                       const float* a_rows, int64_t n_a, const float* b_rows, float* out, int32_t ld,
                       const SpmmItems& items, float* partial, const SpmmScatter& sc, hipStream_t s);
// Aggregation fused with the transform, fp32: y[r,:] = act(Z[r,:] W (+ xself[r,:] Ws) + bias) with
// Z as launch_spmm would compute it, kept in LDS.  zlong: n_a x din floats of scratch for the
// rows that are cut into segments.  Only when spmm_gemm_fused_ok() (d_in in 36..128, a multiple
// of 4; d_out <= 256; and GNNMI_FUSE_AGG=1: measured slower than the two kernels it replaces).
bool spmm_gemm_fused_ok(int32_t din, int32_t dout, const SpmmItems& items);
// stage 0: one launch whose first workgroups take the 512-entry segments of the long rows
// (partial sums into `partial`) and whose other workgroups aggregate and transform the short rows;
// stage 1: the long rows' partial sums are combined into their rows of zlong; stage 2: those rows
// are transformed (a launch of a few workgroups).
void launch_spmm_gemm_fused(const int64_t* rp, const int32_t* col, const float* w, const float* rowscale,
                            const float* a_rows, int64_t n_a, const float* b_rows, int32_t din,
                            const SpmmItems& items, float* partial, float* zlong, const float* xself,
                            const float* W, const float* Ws, const float* bias, int relu, float* y,
                            int32_t dout, int stage, hipStream_t s);
// second step of the aggregation: combines the segment partial sums of the long rows
void launch_spmm_reduce(const float* rowscale, void* out, int32_t d, int out_bf16,
                        const SpmmItems& items, float* partial, const SpmmScatter& sc, hipStream_t s,
                        int32_t ld = 0);

// dst[map(i),:] += src[i,:] with map(i) = base_row + i for i < n_own, idx[i - n_own] otherwise.
void launch_scatter_add(const float* src, int64_t nrows, int64_t n_own, int64_t base_row,
                        const int32_t* idx, float* dst, int32_t d, hipStream_t s);

struct GemmSeg {          // one K-segment of a product: A_seg [M x K] times B_seg [K x N]
    const float* a = nullptr;
    int64_t lda = 0;
    const float* b = nullptr;
    int64_t ldb = 0;
    int32_t k = 0;
};
struct GemmEpilogue {
    const float* bias = nullptr;      // per column, may be null
    int relu = 0;
    int accumulate = 0;               // C += result instead of C = result
};
// C[M x N] = sum over segments A[m, k] (row-major, lda) * B[k, n] (row-major, ldb)
void launch_gemm_nn(const GemmSeg* segs, int nseg, float* c, int64_t ldc, int64_t m, int32_t n,
                    const GemmEpilogue& ep, hipStream_t s);
// C[M x N] = A[M x K] * B^T with B stored [N x K] row-major
void launch_gemm_nt(const float* a, int64_t lda, const float* b, int64_t ldb, float* c,
                    int64_t ldc, int64_t m, int32_t n, int32_t k, const GemmEpilogue& ep,
                    hipStream_t s);
// C[M x N] = sum over segments A_seg[M x K_seg] * B_seg^T with B_seg stored [N x K_seg] row-major
void launch_gemm_nt2(const GemmSeg* segs, int nseg, float* c, int64_t ldc, int64_t m, int32_t n,
                     const GemmEpilogue& ep, hipStream_t s);
// C[M x N] += A^T B with A stored [K x M], B stored [K x N] (K = number of vertices, large):
// split over K into `splits` partial products in `partial`, then reduced in a fixed order.
int gemm_tn_splits(int64_t kdim, int32_t m, int32_t n);
void launch_gemm_tn(const float* a, int64_t lda, const float* b, int64_t ldb, float* c,
                    int64_t ldc, int32_t m, int32_t n, int64_t kdim, float* partial,
                    hipStream_t s);

// bfloat16 operands (raw 16-bit storage), fp32 accumulation; C is fp32 or bfloat16.
struct GemmSegBf16 {
    const void* a = nullptr;
    int64_t lda = 0;
    const void* b = nullptr;
    int64_t ldb = 0;
    int32_t k = 0;
};
// bt_scratch: room for B^T (n x k bfloat16) when there is one segment; with it, large products
// run as A (B^T)^T on the wide kernel for k-contiguous operands
void launch_gemm_bf16_nn(const GemmSegBf16* segs, int nseg, void* c, int out_bf16, int64_t ldc,
                         int64_t m, int32_t n, const GemmEpilogue& ep, hipStream_t s,
                         void* bt_scratch = nullptr);
void launch_gemm_bf16_nt(const void* a, int64_t lda, const void* b, int64_t ldb, void* c,
                         int out_bf16, int64_t ldc, int64_t m, int32_t n, int32_t k,
                         const GemmEpilogue& ep, hipStream_t s);
// floats of `partial` a launch_gemm_bf16_tn of these dimensions may use
int64_t gemm_bf16_tn_partial_floats(int64_t kdim, int32_t m, int32_t n);
void launch_gemm_bf16_tn(const void* a, int64_t lda, const void* b, int64_t ldb, float* c,
                         int64_t ldc, int32_t m, int32_t n, int64_t kdim, float* partial,
                         hipStream_t s);
// c[i] += sum over splits of partial[split * stride + i], splits in ascending order
void launch_reduce_partials(const float* partial, int splits, int64_t stride, float* c, int64_t ldc,
                            int32_t m, int32_t n, hipStream_t s);
void launch_to_bf16(const float* src, void* dst, int64_t n, hipStream_t s);

// bfloat16 variant of the activation backward: g fp32, act bfloat16 (or null), dy bfloat16
// (always written, because the contractions that follow take bfloat16 operands).
void launch_act_bwd_bf16(const float* g, const void* act, void* dy, int64_t rows, int32_t d,
                         float* gb, float* partial, float scale, hipStream_t s);

// dy = scale * g * (act > 0) (or dy = g when act == null); colsum partials then gb += colsum.
// scale = 1 / (1 - p) when dropout followed the activation (the dropped elements are the
// zeros of act), else 1.
// `partial` holds ceil(rows / 64) * d floats.
// row_on (act == null only; may be null): rows with row_on[r] == 0 are known to be zero in g and
// are not read.
void launch_act_bwd(const float* g, const float* act, float* dy, int64_t rows, int32_t d,
                    float* gb, float* partial, float scale, hipStream_t s, const uint8_t* row_on = nullptr);
int64_t act_bwd_partial_floats(int64_t rows, int32_t d);

// softmax cross-entropy over masked rows; grad[n, c]; *loss_dev = mean loss.  count_dev
// receives |M| (counted on the device in the same call).
// part_off[k + 1] (host): the rows are processed partition by partition.
void launch_loss(const float* logits, const int32_t* labels, const uint8_t* mask, float* grad,
                 int64_t n, int32_t c, const int64_t* part_off, int32_t k, unsigned long long* count_dev,
                 float* partial, float* loss_dev, hipStream_t s);
int64_t loss_partial_floats(int64_t n, int32_t k);
// the same in three steps, so that the rows can be processed block by block
void launch_count_mask(const uint8_t* mask, int64_t n, unsigned long long* count_dev, hipStream_t s);
int64_t launch_loss_rows(const float* logits, const int32_t* labels, const uint8_t* mask, float* grad,
                         int64_t rows, int32_t c, const unsigned long long* count_dev, float* partial,
                         hipStream_t s);   // returns the number of partial sums written
void launch_loss_finish(const float* partial, int64_t nparts, const unsigned long long* count_dev,
                        float* loss_dev, hipStream_t s);

// The same loss with |M| and the block partial sums in a device array the library holds
// statically (no workspace from the caller, no allocation); loss_partial_floats(n, k) must not
// exceed loss_static_max_partials().
int64_t loss_static_max_partials();
hipError_t launch_loss_static(const float* logits, const int32_t* labels, const uint8_t* mask, float* grad,
                              int64_t n, int32_t c, const int64_t* part_off, int32_t k, float* loss_dev,
                              hipStream_t s);

void launch_fill_zero(void* p, int64_t bytes, hipStream_t s);
// gcol[e] = lcol[e] < n_own ? base + lcol[e] : bnd[lcol[e] - n_own] for e in [0, count)
void launch_global_columns(const int32_t* lcol, int32_t* gcol, int64_t count, int64_t n_own, int64_t base,
                           const int32_t* bnd, hipStream_t s);

// ---- graph attention (kernels_gat.hip) ----------------------------------------------------
// Rows of one partition for the row-wise attention passes: rp points at the partition's first
// row pointer, col / att / dal are indexed with absolute positions (minus e0 for the
// per-partition arrays).  nh heads: the scores of a vertex are nh floats side by side (s_src of a
// local column c and head h is ssrc_own[c nh + h] or ssrc_bnd[(c - n_own) nh + h]), the per-entry
// arrays (att, dal, tw_att) are one array per head, hs floats apart; the passes below handle all
// heads in one launch.
struct GatRowsHost {
    const int64_t* rp = nullptr;
    const int32_t* col = nullptr;
    int64_t e0 = 0, n_own = 0;
    const float* ssrc_own = nullptr;
    const float* ssrc_bnd = nullptr;
    const float* sdst_own = nullptr;
    int32_t nh = 1;
    int64_t hs = 0;
    SpmmItems items;
};
// every head h < nh: ssrc[r nh + h] = H_h[r, :f] . a_src[h f ..], sdst[r nh + h] = H_h[r, :f] . a_dst[h f ..]
// for `rows` rows, H_h = H + h head_off with rows ld floats apart
void launch_gat_scores(const float* H, int32_t ld, int32_t f, int64_t rows, const float* a_src,
                       const float* a_dst, float* ssrc, float* sdst, int32_t nh, int64_t head_off, hipStream_t s);
// att[e - e0] = softmax over each row of LeakyReLU_0.2(s_src(col e) + s_dst(row))
// segwork: 3 floats per head and segment of the partition's long rows (scratch of the segment-parallel passes)
void launch_gat_attention(const GatRowsHost& h, float* att, float* segwork, hipStream_t s);
// dal[e - e0] = dy[row, :d] . src(col e)[:d]  (rows ld floats apart; d and ld multiples of 4).
// nslice > 1: the same for nslice heads lying side by side, in one launch: head j on columns
// [j d, (j + 1) d) of every row, its products in dal + j dal_stride.
void launch_gat_dots(const int64_t* rp, const int32_t* col, int64_t e0, int64_t n_own, const float* a_rows,
                     const float* b_rows, const float* dy, int32_t d, int32_t ld, float* dal, const SpmmItems& items,
                     hipStream_t s, int32_t nslice = 1, int64_t dal_stride = 0);
// gradient of the pre-activation scores (through softmax and LeakyReLU) from att and dal, every
// head: pair[((e - e0) nh + h) 2 + {0, 1}] = att, dpre (an entry's values of all heads side by
// side, for the transposed pass); gs_dst_own[row nh + h] = row sum of dpre
void launch_gat_bwd_scalars(const GatRowsHost& h, const float* att, const float* dal, float* pair,
                            float* gs_dst_own, float* segwork, hipStream_t s);
// transposed rows, every head: tw_att[h hs + pos - e0] = att of entry tperm[pos];
// gs_src[(owner row of transposed row i) nh + h] += sum over the row of dpre of entry tperm[pos];
// segwork: nh floats per segment of the partition's long transposed rows
void launch_gat_transposed(const int64_t* trp, const int32_t* tperm, int64_t e0, int64_t n_own,
                           int64_t base_row, const int32_t* bnd, const SpmmItems& items, const float* pair,
                           float* tw_att, float* gs_src, int32_t nh, int64_t hs, float* segwork, hipStream_t s);
// gH[r, j] += gs_src[r nh + j / fh] a_src[j] + gs_dst[r nh + j / fh] a_dst[j] over `rows` rows and f
// columns (column j belongs to head j / fh of the score arrays; fh = f and offset pointers: one
// head); partial column sums of gs_src H and gs_dst H (2 f floats per block of 256 rows) for the
// gradients of the attention vectors
int64_t gat_rank1_partial_floats(int64_t rows, int32_t f);
void launch_gat_rank1(float* gH, const float* H, int32_t ld, int32_t f, int64_t rows, const float* gs_src,
                      const float* gs_dst, int32_t nh, int32_t fh, const float* a_src, const float* a_dst,
                      float* partial, hipStream_t s);
// out[c] += sum over b < nblocks of partial[b * ldp + c] for c < d (ldp = 0: rows of d floats)
void launch_colsum_finish(const float* partial, int64_t nblocks, int32_t d, float* out, hipStream_t s,
                          int32_t ldp = 0);

// Transform-first layers: out = (accumulate ? out : 0) + z[:, :d] (+ bias), optional relu, with
// z's row stride ldz >= d and out's row stride ldo (0: d); and a row copy into a wider,
// zero-padded row (source rows lds floats apart, 0: d).
void launch_add_padded(float* out, const float* z, int64_t rows, int32_t d, int32_t ldz,
                       const float* bias, int accumulate, int relu, hipStream_t s, int32_t ldo = 0);
// out[i, :] = bfloat16(act(z[i, 0..d) + bias)), z fp32 with row stride ldz
void launch_bias_act_bf16(void* out, const float* z, int64_t rows, int32_t d, int32_t ldz, const float* bias,
                          int relu, hipStream_t s);
void launch_pad_rows(float* dst, const float* src, int64_t rows, int32_t d, int32_t ld, hipStream_t s,
                     int32_t lds = 0);

// Training pieces: dropout on a block of activation rows (orig_of_row[r] = original vertex id
// of row r), and the optimizer steps on one fp32 parameter tensor.
void launch_dropout(void* a, int is_bf16, const int32_t* orig_of_row, int64_t rows, int32_t d,
                    uint64_t key, uint32_t threshold, float scale, hipStream_t s);
// w16 (may be null): bfloat16 copy of the updated values, rounded to nearest even
void launch_adam(float* w, const float* g, float* m, float* v, int64_t n, float lr, float beta1,
                 float beta2, float eps, float weight_decay, float corr1, float corr2, hipStream_t s,
                 void* w16 = nullptr);
void launch_sgd(float* w, const float* g, int64_t n, float lr, float weight_decay, hipStream_t s,
                void* w16 = nullptr);

// Step 1 of one iteration of the switching-aware partitioner for every vertex: first and second
// preference (second = -1 if there is none) from the assignment `part` and the partition sizes;
// *frac_sum += sum over vertices of floor(2^20 #N(v, part v) / #N(v, .)).  k <= switch_pref_max_k().
int switch_pref_max_k();
void launch_switch_pref(int64_t n, const int64_t* rowptr, const int32_t* colidx, const int32_t* part,
                        const int64_t* sizes, int32_t k, int32_t* first, int32_t* second,
                        unsigned long long* frac_sum, hipStream_t s);

}  // namespace gnnmi
