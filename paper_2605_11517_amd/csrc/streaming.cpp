// Streaming schedule: activations and their gradients live in pinned host memory, one block
// per (layer, partition); HBM holds a cache of blocks at partition granularity.
//
// This is the one-GPU analogue of the paper's partition-wise cache (section on partition-wise
// caching; overlap design in the appendix on I/O optimisations), with HBM in the role of the
// host cache and pinned host memory in the role of storage:
//   - for layer l only blocks of layer l-1 are cached, loaded when a partition depends on them
//     and evicted whole blocks at a time.  The order in which blocks are needed is fixed by
//     the partition dependencies (partition p touches its own block, then the owners of its
//     boundary rows in ascending order), so the victim is the block whose next use lies
//     furthest ahead; least-recently-used would evict exactly the block needed next whenever
//     the partitions depend on more blocks than the cache holds;
//   - the boundary list of a partition is ordered by source partition, so the gather walks it
//     one cached block at a time ("a single lookup per partition");
//   - outputs A_p^l bypass the cache: they go from a transfer buffer straight to their host
//     block;
//   - the gradient of layer l-1 is a write-back cache of blocks: first touch zero-fills,
//     eviction and the end of the layer write back;
//   - loads of the next partition's blocks are issued on a side stream while the current
//     partition computes, stores on a second side stream.
// The arithmetic per partition is the resident schedule's, kernel for kernel, so results are
// bit-identical to it.
#include <algorithm>
#include <climits>
#include <cstdint>
#include <cstring>

#include "gnn_ctx.h"

namespace gnnmi {

namespace {

struct Slot {
    int32_t part = -1;
    int64_t last_use = 0;
    bool dirty = false;
    bool pinned = false;
    hipEvent_t ready = nullptr;     // recorded on the load stream after a block arrived
    hipEvent_t released = nullptr;  // recorded on the compute stream after the last kernel using it
    hipEvent_t flushed = nullptr;   // recorded on the store stream after a write-back
    bool has_ready = false, has_released = false, has_flushed = false;
};

struct BlockCache {
    char* pool = nullptr;
    int64_t pool_bytes = 0, slot_bytes = 0, row_bytes = 0;
    std::vector<Slot> slots;        // events are created once for the largest slot count
    int32_t nslots = 0;
    std::vector<int32_t> slot_of;   // partition -> slot or -1
    std::vector<uint8_t> touched;   // write-back cache: block exists (on host or in a slot)
    char* host = nullptr;           // backing array of the current layer
    bool writeback = false;
    int32_t cur_t = 0;              // step (position in the partition order) whose accesses are being issued
    int64_t tick = 0;
    int64_t loads = 0, hits = 0, writebacks = 0;
    char* ptr(int32_t s) const { return pool + (int64_t)s * slot_bytes; }
};

}  // namespace

struct StreamEngine {
    hipStream_t h2d = nullptr, d2h = nullptr;
    char* pool = nullptr;           // hbm_budget bytes, carved into the two caches per layer
    int64_t pool_bytes = 0;
    BlockCache actc, gradc;
    // next_dep[t * k + b] = first step t' >= t whose partition touches block b (k if none);
    // row k is all k.  Steps follow the order of HostMeta::sched.
    std::vector<int32_t> next_dep;
    int32_t k = 0;
    int64_t h2d_bytes = 0, d2h_bytes = 0;   // of the running epoch
    char* io = nullptr;             // 6 transfer buffers
    int64_t io_bytes = 0;           // bytes of one buffer
    hipEvent_t out_ready[2]{}, out_done[2]{}, in_ready[2]{}, in_released[2]{};
    hipEvent_t layer_done = nullptr, compute_done = nullptr;
    bool has_out_done[2] = {false, false}, has_in_released[2] = {false, false};
    char* outbuf(int i) const { return io + (int64_t)i * io_bytes; }
    char* ginbuf(int i) const { return io + (int64_t)(2 + i) * io_bytes; }
    char* ainbuf(int i) const { return io + (int64_t)(4 + i) * io_bytes; }
};

namespace {

#define GNN_HIP(call)                                                                       \
    do {                                                                                    \
        hipError_t e_ = (call);                                                             \
        if (e_ != hipSuccess)                                                               \
            return c->fail(GNN_EHIP, std::string(#call) + ": " + hipGetErrorString(e_));    \
    } while (0)

gnn_status configure(gnn_ctx* c, BlockCache& bc, char* pool, int64_t pool_bytes, int64_t slot_bytes,
                     int64_t row_bytes, char* host, bool writeback)
{
    slot_bytes = (slot_bytes + 255) / 256 * 256;
    if (slot_bytes <= 0) slot_bytes = 256;
    const int64_t n = pool_bytes / slot_bytes;
    if (n < 2)
        return c->fail(GNN_ENOMEM, "hbm_budget_bytes is too small: a block cache needs room for two "
                                   "partition blocks of the widest layer");
    bc.pool = pool;
    bc.pool_bytes = pool_bytes;
    bc.slot_bytes = slot_bytes;
    bc.row_bytes = row_bytes;
    bc.nslots = (int32_t)std::min<int64_t>(n, (int64_t)bc.slots.size());
    bc.host = host;
    bc.writeback = writeback;
    for (Slot& s : bc.slots) {
        s.part = -1;
        s.dirty = false;
        s.pinned = false;
        s.last_use = 0;
    }
    std::fill(bc.slot_of.begin(), bc.slot_of.end(), -1);
    std::fill(bc.touched.begin(), bc.touched.end(), 0);
    return GNN_OK;
}

// Writes a dirty block back to its host rows on the store stream.
gnn_status write_back(gnn_ctx* c, StreamEngine& E, BlockCache& bc, int32_t s)
{
    Slot& sl = bc.slots[(size_t)s];
    const HostMeta& M = c->M;
    const int64_t r0 = M.off[(size_t)sl.part], np = M.off[(size_t)sl.part + 1] - r0;
    if (sl.has_released) GNN_HIP(hipStreamWaitEvent(E.d2h, sl.released, 0));
    if (np > 0)
        GNN_HIP(hipMemcpyAsync(bc.host + r0 * bc.row_bytes, bc.ptr(s), (size_t)(np * bc.row_bytes),
                               hipMemcpyDeviceToHost, E.d2h));
    GNN_HIP(hipEventRecord(sl.flushed, E.d2h));
    sl.has_flushed = true;
    sl.dirty = false;
    ++bc.writebacks;
    E.d2h_bytes += np * bc.row_bytes;
    return GNN_OK;
}

// Position of "step t touches block b" in the access order of a layer: step by step, the
// step's own block first, then the other blocks in ascending order.
inline int64_t access_pos(int32_t k, int32_t t, int32_t own, int32_t b)
{
    return (int64_t)t * (k + 1) + (b == own ? 0 : (int64_t)b + 1);
}

// Position of the first access to block b after position `now` of step cur_t.
int64_t next_use(const StreamEngine& E, const std::vector<int32_t>& sched, int32_t cur_t, int64_t now,
                 int32_t b)
{
    const int32_t k = E.k;
    if (E.next_dep[(size_t)cur_t * k + b] == cur_t) {
        const int64_t here = access_pos(k, cur_t, sched[(size_t)cur_t], b);
        if (here > now) return here;
    }
    const int32_t t2 = E.next_dep[(size_t)(cur_t + 1) * k + b];
    return t2 >= k ? INT64_MAX : access_pos(k, t2, sched[(size_t)t2], b);
}

// Chooses a slot for block `part`: a free one, else the unpinned one whose block is needed
// again last (ties: the least recently used).
int32_t pick_victim(const StreamEngine& E, const std::vector<int32_t>& sched, const BlockCache& bc,
                    int32_t part)
{
    const int64_t now = access_pos(E.k, bc.cur_t, sched[(size_t)bc.cur_t], part);
    int32_t best = -1;
    int64_t best_next = -1;
    for (int32_t s = 0; s < bc.nslots; ++s) {
        const Slot& sl = bc.slots[(size_t)s];
        if (sl.part < 0) return s;
        if (sl.pinned) continue;
        const int64_t nu = next_use(E, sched, bc.cur_t, now, sl.part);
        if (best < 0 || nu > best_next ||
            (nu == best_next && sl.last_use < bc.slots[(size_t)best].last_use)) {
            best = s;
            best_next = nu;
        }
    }
    return best;
}

// Makes partition `part`'s block resident and returns its slot.  `wait` = the compute stream
// must be able to use it right away (otherwise this is a prefetch).  Returns -1 in `slot_out`
// when a prefetch finds no slot to take.
gnn_status acquire(gnn_ctx* c, StreamEngine& E, BlockCache& bc, int32_t part, hipStream_t compute,
                   bool wait, int32_t* slot_out)
{
    const HostMeta& M = c->M;
    int32_t s = bc.slot_of[(size_t)part];
    if (s >= 0) {
        ++bc.hits;
    } else {
        s = pick_victim(E, M.sched, bc, part);
        if (s < 0) {
            if (!wait) { *slot_out = -1; return GNN_OK; }
            return c->fail(GNN_ENOMEM, "streaming cache: every slot is pinned");
        }
        Slot& sl = bc.slots[(size_t)s];
        if (sl.part >= 0) {
            if (sl.dirty) {
                gnn_status st = write_back(c, E, bc, s);
                if (st != GNN_OK) return st;
            }
            bc.slot_of[(size_t)sl.part] = -1;
        }
        const int64_t r0 = M.off[(size_t)part], np = M.off[(size_t)part + 1] - r0;
        const bool fresh = bc.writeback && !bc.touched[(size_t)part];
        if (fresh) {
            // first touch of a gradient block in this layer: start from zero, on the compute stream
            if (sl.has_flushed) GNN_HIP(hipStreamWaitEvent(compute, sl.flushed, 0));
            launch_fill_zero(bc.ptr(s), np * bc.row_bytes, compute);
            sl.has_ready = false;
        } else {
            if (sl.has_released) GNN_HIP(hipStreamWaitEvent(E.h2d, sl.released, 0));
            if (sl.has_flushed) GNN_HIP(hipStreamWaitEvent(E.h2d, sl.flushed, 0));
            if (np > 0)
                GNN_HIP(hipMemcpyAsync(bc.ptr(s), bc.host + r0 * bc.row_bytes, (size_t)(np * bc.row_bytes),
                                       hipMemcpyHostToDevice, E.h2d));
            GNN_HIP(hipEventRecord(sl.ready, E.h2d));
            sl.has_ready = true;
            ++bc.loads;
            E.h2d_bytes += np * bc.row_bytes;
        }
        sl.part = part;
        sl.dirty = false;
        bc.slot_of[(size_t)part] = s;
        if (bc.writeback) bc.touched[(size_t)part] = 1;
    }
    Slot& sl = bc.slots[(size_t)s];
    sl.last_use = ++bc.tick;
    if (wait && sl.has_ready) GNN_HIP(hipStreamWaitEvent(compute, sl.ready, 0));
    *slot_out = s;
    return GNN_OK;
}

gnn_status mark_used(gnn_ctx* c, BlockCache& bc, int32_t s, hipStream_t compute, bool dirty)
{
    Slot& sl = bc.slots[(size_t)s];
    GNN_HIP(hipEventRecord(sl.released, compute));
    sl.has_released = true;
    if (dirty) sl.dirty = true;
    return GNN_OK;
}

// Gather of partition p's boundary rows from the cached blocks of layer l-1, one source
// partition at a time.  Leaves the own block pinned and returns its slot.
gnn_status gather_from_cache(gnn_ctx* c, StreamEngine& E, int32_t layer, int32_t t, hipStream_t s,
                             int32_t* own_slot)
{
    const HostMeta& M = c->M;
    const int32_t k = M.k, p = M.sched[(size_t)t];
    const int64_t row_bytes = (int64_t)c->dims[(size_t)layer - 1] * c->es();
    E.actc.cur_t = t;
    gnn_status st = acquire(c, E, E.actc, p, s, true, own_slot);
    if (st != GNN_OK) return st;
    E.actc.slots[(size_t)*own_slot].pinned = true;
    const int64_t* run = M.brun.data() + (size_t)p * ((size_t)k + 1);
    const int64_t b0 = M.boff[(size_t)p];
    Timed timed(c, s, GNN_K_GATHER);
    for (int32_t q = 0; q < k; ++q) {
        const int64_t len = run[q + 1] - run[q];
        if (len <= 0) continue;
        int32_t sq;
        if ((st = acquire(c, E, E.actc, q, s, true, &sq)) != GNN_OK) return st;
        launch_gather_rows(E.actc.ptr(sq), c->D.bnd_local + b0 + run[q], c->staging + run[q] * row_bytes,
                           len, row_bytes, s);
        if ((st = mark_used(c, E.actc, sq, s, false)) != GNN_OK) return st;
    }
    return GNN_OK;
}

// Issues loads for the blocks the partition of step t will need, as long as a slot can be
// taken for them.
gnn_status prefetch_for(gnn_ctx* c, StreamEngine& E, int32_t t, hipStream_t s)
{
    const HostMeta& M = c->M;
    const int32_t k = M.k;
    if (t >= k) return GNN_OK;
    const int32_t p = M.sched[(size_t)t];
    const int64_t* run = M.brun.data() + (size_t)p * ((size_t)k + 1);
    int32_t budget = E.actc.nslots - 1;      // never cycle the whole cache for a prefetch
    int32_t slot;
    E.actc.cur_t = t;
    gnn_status st = acquire(c, E, E.actc, p, s, false, &slot);
    if (st != GNN_OK) return st;
    --budget;
    for (int32_t q = 0; q < k && budget > 0; ++q) {
        if (run[q + 1] - run[q] <= 0) continue;
        if (E.actc.slot_of[(size_t)q] < 0) {
            if ((st = acquire(c, E, E.actc, q, s, false, &slot)) != GNN_OK) return st;
            if (slot < 0) break;
        }
        --budget;
    }
    return GNN_OK;
}

}  // namespace

gnn_status stream_engine_create(gnn_ctx* c)
{
    stream_engine_destroy(c);
    const HostMeta& M = c->M;
    StreamEngine* E = new (std::nothrow) StreamEngine();
    if (!E) return c->fail(GNN_ENOMEM, "out of host memory");
    c->stream_engine = E;
    {
        const int32_t k = M.k;
        E->k = k;
        E->next_dep.assign(((size_t)k + 1) * (size_t)k, k);
        for (int32_t t = k - 1; t >= 0; --t) {
            const int32_t p = M.sched[(size_t)t];
            const int64_t* run = M.brun.data() + (size_t)p * ((size_t)k + 1);
            for (int32_t b = 0; b < k; ++b) {
                const bool dep = b == p || run[b + 1] > run[b];
                E->next_dep[(size_t)t * k + b] = dep ? t : E->next_dep[(size_t)(t + 1) * k + b];
            }
        }
    }
    int64_t dmax = 0;
    for (int32_t d : c->dims) dmax = std::max<int64_t>(dmax, d);
    E->io_bytes = (std::max<int64_t>(1, M.stats.max_own * dmax * 4) + 255) / 256 * 256;
    E->pool_bytes = c->hbm_budget;
    // the tightest layer must still fit two activation blocks and two gradient blocks
    const int64_t need = 2 * ((M.stats.max_own * dmax * c->es() + 255) / 256 * 256) +
                         2 * ((M.stats.max_own * dmax * 4 + 255) / 256 * 256);
    if (E->pool_bytes < need) {
        stream_engine_destroy(c);
        return c->fail(GNN_ENOMEM, "hbm_budget_bytes is too small: needs room for two activation blocks "
                                   "and two gradient blocks of the widest layer (" + std::to_string(need) + " bytes)");
    }
    auto fail_hip = [&](hipError_t e, const char* what) {
        std::string msg = std::string(what) + ": " + hipGetErrorString(e);
        stream_engine_destroy(c);
        (void)hipGetLastError();
        return c->fail(e == hipErrorOutOfMemory ? GNN_ENOMEM : GNN_EHIP, msg);
    };
    hipError_t e;
    if ((e = hipStreamCreate(&E->h2d)) != hipSuccess) return fail_hip(e, "hipStreamCreate");
    if ((e = hipStreamCreate(&E->d2h)) != hipSuccess) return fail_hip(e, "hipStreamCreate");
    if ((e = hipMalloc((void**)&E->pool, (size_t)E->pool_bytes)) != hipSuccess) return fail_hip(e, "hipMalloc(block cache)");
    if ((e = hipMalloc((void**)&E->io, (size_t)(6 * E->io_bytes))) != hipSuccess) return fail_hip(e, "hipMalloc(transfer buffers)");
    // at most one slot per partition is ever useful
    const int64_t min_slot = std::max<int64_t>(256, M.stats.max_own * 1 * 2);
    const int64_t max_slots = std::min<int64_t>((int64_t)M.k + 1, E->pool_bytes / min_slot + 1);
    for (BlockCache* bc : {&E->actc, &E->gradc}) {
        bc->slots.resize((size_t)std::max<int64_t>(2, max_slots));
        bc->slot_of.assign((size_t)M.k, -1);
        bc->touched.assign((size_t)M.k, 0);
        for (Slot& s : bc->slots) {
            if ((e = hipEventCreateWithFlags(&s.ready, hipEventDisableTiming)) != hipSuccess) return fail_hip(e, "hipEventCreate");
            if ((e = hipEventCreateWithFlags(&s.released, hipEventDisableTiming)) != hipSuccess) return fail_hip(e, "hipEventCreate");
            if ((e = hipEventCreateWithFlags(&s.flushed, hipEventDisableTiming)) != hipSuccess) return fail_hip(e, "hipEventCreate");
        }
    }
    for (int i = 0; i < 2; ++i) {
        if ((e = hipEventCreateWithFlags(&E->out_ready[i], hipEventDisableTiming)) != hipSuccess) return fail_hip(e, "hipEventCreate");
        if ((e = hipEventCreateWithFlags(&E->out_done[i], hipEventDisableTiming)) != hipSuccess) return fail_hip(e, "hipEventCreate");
        if ((e = hipEventCreateWithFlags(&E->in_ready[i], hipEventDisableTiming)) != hipSuccess) return fail_hip(e, "hipEventCreate");
        if ((e = hipEventCreateWithFlags(&E->in_released[i], hipEventDisableTiming)) != hipSuccess) return fail_hip(e, "hipEventCreate");
    }
    if ((e = hipEventCreateWithFlags(&E->layer_done, hipEventDisableTiming)) != hipSuccess) return fail_hip(e, "hipEventCreate");
    if ((e = hipEventCreateWithFlags(&E->compute_done, hipEventDisableTiming)) != hipSuccess) return fail_hip(e, "hipEventCreate");
    return GNN_OK;
}

void stream_engine_destroy(gnn_ctx* c)
{
    StreamEngine* E = c->stream_engine;
    if (!E) return;
    if (E->h2d) (void)hipStreamSynchronize(E->h2d);
    if (E->d2h) (void)hipStreamSynchronize(E->d2h);
    for (BlockCache* bc : {&E->actc, &E->gradc})
        for (Slot& s : bc->slots) {
            if (s.ready) (void)hipEventDestroy(s.ready);
            if (s.released) (void)hipEventDestroy(s.released);
            if (s.flushed) (void)hipEventDestroy(s.flushed);
        }
    for (int i = 0; i < 2; ++i) {
        if (E->out_ready[i]) (void)hipEventDestroy(E->out_ready[i]);
        if (E->out_done[i]) (void)hipEventDestroy(E->out_done[i]);
        if (E->in_ready[i]) (void)hipEventDestroy(E->in_ready[i]);
        if (E->in_released[i]) (void)hipEventDestroy(E->in_released[i]);
    }
    if (E->layer_done) (void)hipEventDestroy(E->layer_done);
    if (E->compute_done) (void)hipEventDestroy(E->compute_done);
    if (E->pool) (void)hipFree(E->pool);
    if (E->io) (void)hipFree(E->io);
    if (E->h2d) (void)hipStreamDestroy(E->h2d);
    if (E->d2h) (void)hipStreamDestroy(E->d2h);
    delete E;
    c->stream_engine = nullptr;
}

gnn_status epoch_streaming(gnn_ctx* c, hipStream_t s, float* loss_out)
{
    StreamEngine& E = *c->stream_engine;
    const HostMeta& M = c->M;
    const int32_t L = c->L, k = M.k;
    const int64_t max_np = M.stats.max_own;
    gnn_status st;

    // Everything the side streams do must come after what the caller enqueued before this call.
    GNN_HIP(hipEventRecord(E.layer_done, s));
    GNN_HIP(hipStreamWaitEvent(E.h2d, E.layer_done, 0));
    GNN_HIP(hipStreamWaitEvent(E.d2h, E.layer_done, 0));
    for (BlockCache* bc : {&E.actc, &E.gradc})
        for (Slot& sl : bc->slots) sl.has_ready = sl.has_released = sl.has_flushed = false;
    E.has_out_done[0] = E.has_out_done[1] = false;
    E.has_in_released[0] = E.has_in_released[1] = false;
    E.h2d_bytes = E.d2h_bytes = 0;
    for (BlockCache* bc : {&E.actc, &E.gradc}) bc->loads = bc->hits = bc->writebacks = 0;

    zero_weight_grads(c, s);

    // After a layer: the next layer's loads must see this layer's stores, and because the
    // cache is re-cut into slots of another size, neither loads nor zero fills of the next
    // layer may start before this layer's kernels and write-backs are done with the pool.
    auto end_of_layer = [&]() -> gnn_status {
        GNN_HIP(hipEventRecord(E.layer_done, E.d2h));
        GNN_HIP(hipStreamWaitEvent(E.h2d, E.layer_done, 0));
        GNN_HIP(hipStreamWaitEvent(s, E.layer_done, 0));
        GNN_HIP(hipEventRecord(E.compute_done, s));
        GNN_HIP(hipStreamWaitEvent(E.h2d, E.compute_done, 0));
        GNN_HIP(hipStreamWaitEvent(E.d2h, E.compute_done, 0));
        return GNN_OK;
    };
    // Sends transfer buffer `ob` (filled on the compute stream) to `dst` on the store stream.
    auto store_out = [&](int ob, char* dst, int64_t bytes) -> gnn_status {
        GNN_HIP(hipEventRecord(E.out_ready[ob], s));
        GNN_HIP(hipStreamWaitEvent(E.d2h, E.out_ready[ob], 0));
        if (bytes > 0) GNN_HIP(hipMemcpyAsync(dst, E.outbuf(ob), (size_t)bytes, hipMemcpyDeviceToHost, E.d2h));
        E.d2h_bytes += bytes;
        GNN_HIP(hipEventRecord(E.out_done[ob], E.d2h));
        E.has_out_done[ob] = true;
        return GNN_OK;
    };
    auto wait_out_free = [&](int ob) -> gnn_status {
        if (E.has_out_done[ob]) GNN_HIP(hipStreamWaitEvent(s, E.out_done[ob], 0));
        return GNN_OK;
    };

    // ---------------------------------------------------------------------------- forward
    for (int32_t l = 1; l <= L; ++l) {
        const int32_t din = c->dims[(size_t)l - 1], dout = c->dims[(size_t)l];
        st = configure(c, E.actc, E.pool, E.pool_bytes, max_np * din * c->es(), (int64_t)din * c->es(),
                       const_cast<char*>(c->layer_input(l)), false);
        if (st != GNN_OK) return st;
        const int64_t out_row = (int64_t)dout * c->act_es(l);
        for (int32_t t = 0; t < k; ++t) {
            const int32_t p = M.sched[(size_t)t];
            const int64_t r0 = M.off[(size_t)p], np = M.off[(size_t)p + 1] - r0;
            int32_t own;
            if ((st = gather_from_cache(c, E, l, t, s, &own)) != GNN_OK) return st;
            if ((st = prefetch_for(c, E, t + 1, s)) != GNN_OK) return st;
            const int ob = t & 1;
            if ((st = wait_out_free(ob)) != GNN_OK) return st;
            compute_fwd(c, l, p, E.actc.ptr(own), E.outbuf(ob), s);
            if ((st = mark_used(c, E.actc, own, s, false)) != GNN_OK) return st;
            E.actc.slots[(size_t)own].pinned = false;
            if ((st = store_out(ob, c->act[(size_t)l - 1] + r0 * out_row, np * out_row)) != GNN_OK) return st;
        }
        if ((st = end_of_layer()) != GNN_OK) return st;
    }

    // ------------------------------------------------------------------------------- loss
    float* scal = (float*)(c->scratch + c->ws.scalars);
    unsigned long long* count_dev = (unsigned long long*)(scal + 16);
    float* losspart = (float*)(c->scratch + c->ws.losspart);
    // Loads rows [r0, r0 + np) of a host array into transfer buffer `dst` on the load stream.
    auto load_in = [&](char* dst, const char* src, int64_t bytes, int ib, bool first) -> gnn_status {
        if (first && E.has_in_released[ib]) GNN_HIP(hipStreamWaitEvent(E.h2d, E.in_released[ib], 0));
        if (bytes > 0) GNN_HIP(hipMemcpyAsync(dst, src, (size_t)bytes, hipMemcpyHostToDevice, E.h2d));
        E.h2d_bytes += bytes;
        return GNN_OK;
    };
    {
        const int32_t C = c->dims[(size_t)L];
        launch_count_mask(c->mask, M.n, count_dev, s);
        int64_t nparts = 0;
        for (int32_t p = 0; p < k; ++p) {
            const int64_t r0 = M.off[(size_t)p], np = M.off[(size_t)p + 1] - r0;
            const int ib = p & 1;
            if ((st = load_in(E.ainbuf(ib), c->act[(size_t)L - 1] + r0 * C * 4, np * C * 4, ib, true)) != GNN_OK) return st;
            GNN_HIP(hipEventRecord(E.in_ready[ib], E.h2d));
            GNN_HIP(hipStreamWaitEvent(s, E.in_ready[ib], 0));
            if ((st = wait_out_free(ib)) != GNN_OK) return st;
            {
                Timed t(c, s, GNN_K_LOSS);
                nparts += launch_loss_rows((const float*)E.ainbuf(ib), c->labels + r0, c->mask + r0,
                                           (float*)E.outbuf(ib), np, C, count_dev, losspart + nparts, s);
            }
            GNN_HIP(hipEventRecord(E.in_released[ib], s));
            E.has_in_released[ib] = true;
            if ((st = store_out(ib, (char*)(c->gact[(size_t)L - 1] + r0 * C), np * C * 4)) != GNN_OK) return st;
        }
        launch_loss_finish(losspart, nparts, count_dev, scal, s);
        if ((st = end_of_layer()) != GNN_OK) return st;
    }

    // --------------------------------------------------------------------------- backward
    for (int32_t l = L; l >= 1; --l) {
        const int32_t din = c->dims[(size_t)l - 1], dout = c->dims[(size_t)l];
        const int64_t act_row = (int64_t)dout * c->act_es(l);
        const bool need_prev = l >= 2;
        // Split of the pool between the two caches.  A gradient block that is evicted costs a
        // write-back and a reload, an activation block only a reload: when every gradient
        // block of the layer fits beside two activation blocks the gradient cache gets them
        // all, otherwise two thirds of the pool.
        int64_t act_pool = E.pool_bytes;
        if (need_prev) {
            const int64_t a_slot = (max_np * din * c->es() + 255) / 256 * 256;
            const int64_t g_slot = (max_np * din * 4 + 255) / 256 * 256;
            int64_t grad_pool = (int64_t)k * g_slot;
            if (E.pool_bytes - grad_pool < 2 * a_slot) {
                grad_pool = E.pool_bytes / 3 * 2 / 256 * 256;
                grad_pool = std::min(grad_pool, E.pool_bytes - 2 * a_slot);
                grad_pool = std::max(grad_pool, 2 * g_slot);
            }
            act_pool = (E.pool_bytes - grad_pool) / 256 * 256;
        }
        st = configure(c, E.actc, E.pool, act_pool, max_np * din * c->es(), (int64_t)din * c->es(),
                       const_cast<char*>(c->layer_input(l)), false);
        if (st != GNN_OK) return st;
        if (need_prev) {
            st = configure(c, E.gradc, E.pool + act_pool, E.pool_bytes - act_pool, max_np * din * 4,
                           (int64_t)din * 4, (char*)c->gact[(size_t)l - 2], true);
            if (st != GNN_OK) return st;
        }
        // transfer buffers of partition p: its gradient block and (hidden layers) its activations
        auto load_io = [&](int32_t t) -> gnn_status {
            const int32_t p = M.sched[(size_t)t];
            const int64_t r0 = M.off[(size_t)p], np = M.off[(size_t)p + 1] - r0;
            const int ib = t & 1;
            gnn_status r = load_in(E.ginbuf(ib), (const char*)(c->gact[(size_t)l - 1] + r0 * dout),
                                   np * dout * 4, ib, true);
            if (r != GNN_OK) return r;
            if (l < L) {
                r = load_in(E.ainbuf(ib), c->act[(size_t)l - 1] + r0 * act_row, np * act_row, ib, false);
                if (r != GNN_OK) return r;
            }
            GNN_HIP(hipEventRecord(E.in_ready[ib], E.h2d));
            return GNN_OK;
        };
        if ((st = load_io(0)) != GNN_OK) return st;
        for (int32_t t = 0; t < k; ++t) {
            const int32_t p = M.sched[(size_t)t];
            const int64_t np = M.off[(size_t)p + 1] - M.off[(size_t)p];
            const int ib = t & 1;
            int32_t own;
            if ((st = gather_from_cache(c, E, l, t, s, &own)) != GNN_OK) return st;
            if ((st = prefetch_for(c, E, t + 1, s)) != GNN_OK) return st;
            if (t + 1 < k && (st = load_io(t + 1)) != GNN_OK) return st;
            GNN_HIP(hipStreamWaitEvent(s, E.in_ready[ib], 0));
            const char* dY = compute_bwd(c, l, p, E.actc.ptr(own), (const float*)E.ginbuf(ib),
                                         l < L ? E.ainbuf(ib) : nullptr, nullptr, s);
            if ((st = mark_used(c, E.actc, own, s, false)) != GNN_OK) return st;
            E.actc.slots[(size_t)own].pinned = false;
            if (need_prev) {
                // scatter-accumulate the gradient of the gathered rows, owner block by owner block
                const float* dGA = (const float*)(c->scratch + c->ws.dga);
                const int64_t* run = M.brun.data() + (size_t)p * ((size_t)k + 1);
                const int64_t b0 = M.boff[(size_t)p];
                int32_t gown;
                E.gradc.cur_t = t;
                if ((st = acquire(c, E, E.gradc, p, s, true, &gown)) != GNN_OK) return st;
                E.gradc.slots[(size_t)gown].pinned = true;
                {
                    Timed timed(c, s, GNN_K_SCATTER);
                    launch_scatter_add(dGA, np, np, 0, nullptr, (float*)E.gradc.ptr(gown), din, s);
                    for (int32_t q = 0; q < k; ++q) {
                        const int64_t len = run[q + 1] - run[q];
                        if (len <= 0) continue;
                        int32_t gq;
                        if ((st = acquire(c, E, E.gradc, q, s, true, &gq)) != GNN_OK) return st;
                        launch_scatter_add(dGA + (np + run[q]) * din, len, 0, 0, c->D.bnd_local + b0 + run[q],
                                           (float*)E.gradc.ptr(gq), din, s);
                        if ((st = mark_used(c, E.gradc, gq, s, true)) != GNN_OK) return st;
                    }
                }
                compute_bwd_self(c, l, p, dY, (float*)E.gradc.ptr(gown), s);
                if ((st = mark_used(c, E.gradc, gown, s, true)) != GNN_OK) return st;
                E.gradc.slots[(size_t)gown].pinned = false;
            }
            // dY may alias the gradient transfer buffer: release it only now
            GNN_HIP(hipEventRecord(E.in_released[ib], s));
            E.has_in_released[ib] = true;
        }
        if (need_prev) {
            // end of the layer: every gradient block goes back to its host rows
            for (int32_t sidx = 0; sidx < E.gradc.nslots; ++sidx)
                if (E.gradc.slots[(size_t)sidx].part >= 0 && E.gradc.slots[(size_t)sidx].dirty)
                    if ((st = write_back(c, E, E.gradc, sidx)) != GNN_OK) return st;
        }
        if ((st = end_of_layer()) != GNN_OK) return st;
    }

    GNN_HIP(hipStreamSynchronize(s));
    GNN_HIP(hipStreamSynchronize(E.h2d));
    GNN_HIP(hipStreamSynchronize(E.d2h));
    GNN_HIP(hipMemcpy(loss_out, scal, sizeof(float), hipMemcpyDeviceToHost));
    c->loss_done = true;
    c->stream_stats.act_loads = E.actc.loads;
    c->stream_stats.act_hits = E.actc.hits;
    c->stream_stats.grad_loads = E.gradc.loads;
    c->stream_stats.grad_hits = E.gradc.hits;
    c->stream_stats.grad_writebacks = E.gradc.writebacks;
    c->stream_stats.h2d_bytes = E.h2d_bytes;
    c->stream_stats.d2h_bytes = E.d2h_bytes;
    return check_launch(c, "gnn_epoch (streaming)");
}

}  // namespace gnnmi
