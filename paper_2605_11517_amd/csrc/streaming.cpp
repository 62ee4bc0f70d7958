// Streaming schedule: activations and their gradients live in pinned host memory, one block
// per (layer, partition); a pool of HBM caches them.
//
// This is the one-GPU analogue of the paper's partition-wise cache (section on partition-wise
// caching; overlap design in the appendix on I/O optimisations), with HBM in the role of the
// host cache and pinned host memory in the role of storage:
//   - the pool holds whole per-layer arrays while they fit ("layer-wise" caching: an array of k
//     partition blocks, each block loaded or produced at most once) and falls back to a cache
//     of single partition blocks for an array that does not fit (the paper's partition-wise
//     eviction).  When room is needed the array of the lowest layer goes first: forward needs it
//     no more and backward needs it last;
//   - in the block cache a block is loaded when a partition depends on it and evicted whole.  The
//     order in which blocks are needed is fixed by the partition dependencies (a partition
//     touches its own block, then the owners of its boundary rows in ascending order), so the
//     victim is the block whose next use lies furthest ahead; least-recently-used would evict
//     exactly the block needed next whenever the partitions depend on more blocks than fit;
//   - the boundary list of a partition is ordered by source partition, so the gather walks it
//     one cached block at a time ("a single lookup per partition");
//   - outputs A_p^l bypass the cache on their way out: they are stored to their host block
//     straight from where the kernel wrote them (a transfer buffer, or their block of a resident
//     array, where the next layer then finds them without a load);
//   - the gradient of layer l-1 is written back: first touch zero-fills, eviction and the end of
//     the layer write back;
//   - loads of the next partition's blocks are issued on a side stream while the current
//     partition computes, stores on a second side stream.
// The arithmetic per partition is the resident schedule's, kernel for kernel, so results are
// bit-identical to it.
#include <algorithm>
#include <climits>
#include <cstdint>
#include <cstring>
#include <initializer_list>
#include <memory>
#include <utility>

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
    bool waited = false;            // the compute stream has already waited for `ready`
};

struct BlockCache {
    char* pool = nullptr;
    int64_t pool_bytes = 0, slot_bytes = 0, row_bytes = 0;
    std::vector<Slot> slots;
    int32_t nslots = 0;
    std::vector<int32_t> slot_of;   // partition -> slot or -1
    std::vector<uint8_t> touched;   // write-back cache: block exists (on host or in a slot)
    char* host = nullptr;           // backing array
    const char* host_dev = nullptr; // the same memory as kernels see it (null: not mapped for the device)
    bool writeback = false;
    bool identity = false;          // a whole array: block p lives in slot p and is never evicted
    // write-back cache whose host array kernels can reach: rows of blocks that are not cached are
    // added to straight in host memory.  Per block: an event after the last such kernel (a later
    // load of the block waits for it) and one after the last write-back (a later kernel waits)
    std::vector<hipEvent_t> blk_direct, blk_flushed;
    std::vector<uint8_t> has_blk_direct, has_blk_flushed;
    int32_t cur_t = 0;              // step (position in the partition order) whose accesses are being issued
    int64_t tick = 0;
    char* ptr(int32_t s) const { return pool + (int64_t)s * slot_bytes; }
    bool holds(int32_t part) const { return slot_of[(size_t)part] >= 0; }
};

enum ArrayKind { ARR_ACT = 0, ARR_GRAD = 1 };

// A whole per-vertex array of one layer kept in the pool: (ARR_ACT, l) = A^l (l = 0: the
// features), (ARR_GRAD, l) = grad A^l.
struct Resident {
    int kind = 0, layer = 0;
    int64_t off = 0, bytes = 0;
    BlockCache bc;
};

}  // namespace

struct StreamEngine {
    hipStream_t h2d = nullptr, d2h = nullptr;
    char* pool = nullptr;
    int64_t pool_bytes = 0;
    std::vector<std::pair<int64_t, int64_t>> free_list;    // (offset, bytes), ascending, coalesced
    std::vector<std::unique_ptr<Resident>> arrays;
    BlockCache actc, gradc;         // block caches for arrays that are not resident
    std::vector<Slot> spare;        // slots (with their events) of released arrays
    // next_dep[t * k + b] = first step t' >= t whose partition touches block b (k if none);
    // row k is all k.  Steps follow the order of HostMeta::sched.
    std::vector<int32_t> next_dep;
    int32_t k = 0;
    int64_t h2d_bytes = 0, d2h_bytes = 0;   // of the running epoch
    int64_t direct_gathers = 0, direct_bytes = 0;   // boundary rows read straight from host memory
    int64_t direct_scatters = 0, direct_scatter_bytes = 0;   // gradient rows added straight in host memory
    int64_t loads[2] = {0, 0}, hits[2] = {0, 0}, writebacks = 0;
    char* io = nullptr;             // 8 transfer buffers
    int64_t io_bytes = 0;           // bytes of one buffer
    char* xf = nullptr;             // whole-graph buffers of transform-first layers (H / grad H, kept dY)
    hipEvent_t out_ready[2]{}, out_done[2]{}, in_ready[2]{}, in_released[2]{};
    hipEvent_t layer_done = nullptr, compute_done = nullptr;
    bool has_out_done[2] = {false, false}, has_in_released[2] = {false, false};
    char* outbuf(int i) const { return io + (int64_t)i * io_bytes; }
    char* ginbuf(int i) const { return io + (int64_t)(2 + i) * io_bytes; }
    char* ainbuf(int i) const { return io + (int64_t)(4 + i) * io_bytes; }
    char* xinbuf(int i) const { return io + (int64_t)(6 + i) * io_bytes; }   // A^{l-1} blocks of such layers
    // Storage tier, arrays that are not in host memory: their blocks pass through these pinned
    // buffers on the way between file and device (allocated on first use)
    struct Bounce {
        char* buf = nullptr;
        hipEvent_t done = nullptr;   // after the copy that uses the buffer
        bool busy = false, is_write = false;
        int arr = -1;
        int64_t off = 0, bytes = 0;
    };
    std::vector<Bounce> bounce;
    size_t next_bounce = 0;
};

namespace {

#define GNN_HIP(call)                                                                       \
    do {                                                                                    \
        hipError_t e_ = (call);                                                             \
        if (e_ != hipSuccess)                                                               \
            return c->fail(GNN_EHIP, std::string(#call) + ": " + hipGetErrorString(e_));    \
    } while (0)

inline int64_t round256(int64_t b) { return (std::max<int64_t>(b, 1) + 255) / 256 * 256; }

// ---- copies between host arrays and the device ---------------------------------------------------
// A host address is either real (pinned memory: the caller's arrays, or the storage tier's pool)
// or names a block of an array that the tier keeps on storage only (tier_decode).  The latter go
// through a pinned buffer: file -> buffer -> device at once, device -> buffer now and buffer ->
// file once that copy has run (at the latest when the buffer is needed again, when the same array
// is read, or when the phase ends).
constexpr int kBounceBuffers = 4;

gnn_status bounce_finish(gnn_ctx* c, StreamEngine::Bounce& b)
{
    if (!b.busy) return GNN_OK;
    GNN_HIP(hipEventSynchronize(b.done));
    b.busy = false;
    if (b.is_write) return tier_file_write(c, b.arr, b.off, b.buf, b.bytes);
    return GNN_OK;
}

gnn_status bounce_drain(gnn_ctx* c, StreamEngine& E, bool writes_only)
{
    // oldest first: blocks reach the file in the order they were produced
    for (size_t i = 0; i < E.bounce.size(); ++i) {
        StreamEngine::Bounce& b = E.bounce[(E.next_bounce + i) % E.bounce.size()];
        if (writes_only && !b.is_write) continue;
        gnn_status st = bounce_finish(c, b);
        if (st != GNN_OK) return st;
    }
    return GNN_OK;
}

gnn_status bounce_get(gnn_ctx* c, StreamEngine& E, StreamEngine::Bounce** out)
{
    if (E.bounce.empty()) {
        E.bounce.resize(kBounceBuffers);
        for (auto& b : E.bounce) {
            GNN_HIP(hipHostMalloc((void**)&b.buf, (size_t)E.io_bytes, hipHostMallocDefault));
            GNN_HIP(hipEventCreateWithFlags(&b.done, hipEventDisableTiming));
        }
    }
    StreamEngine::Bounce& b = E.bounce[E.next_bounce];
    E.next_bounce = (E.next_bounce + 1) % E.bounce.size();
    gnn_status st = bounce_finish(c, b);      // the buffer used longest ago
    if (st != GNN_OK) return st;
    *out = &b;
    return GNN_OK;
}

gnn_status copy_h2d(gnn_ctx* c, StreamEngine& E, void* dst_dev, const void* src_host, int64_t bytes, hipStream_t stream)
{
    int id;
    int64_t off;
    if (!c->tier || !tier_decode(src_host, &id, &off)) {
        GNN_HIP(hipMemcpyAsync(dst_dev, src_host, (size_t)bytes, hipMemcpyHostToDevice, stream));
        return GNN_OK;
    }
    if (bytes > E.io_bytes) return c->fail(GNN_EINVAL, "storage tier: a block larger than the transfer buffers");
    gnn_status st = bounce_drain(c, E, true);  // what was produced before must be in the file
    if (st != GNN_OK) return st;
    StreamEngine::Bounce* b;
    if ((st = bounce_get(c, E, &b)) != GNN_OK) return st;
    if ((st = tier_file_read(c, id, off, b->buf, bytes)) != GNN_OK) return st;
    GNN_HIP(hipMemcpyAsync(dst_dev, b->buf, (size_t)bytes, hipMemcpyHostToDevice, stream));
    GNN_HIP(hipEventRecord(b->done, stream));
    b->busy = true;
    b->is_write = false;
    return GNN_OK;
}

gnn_status copy_d2h(gnn_ctx* c, StreamEngine& E, void* dst_host, const void* src_dev, int64_t bytes, hipStream_t stream)
{
    int id;
    int64_t off;
    if (!c->tier || !tier_decode(dst_host, &id, &off)) {
        GNN_HIP(hipMemcpyAsync(dst_host, src_dev, (size_t)bytes, hipMemcpyDeviceToHost, stream));
        return GNN_OK;
    }
    if (bytes > E.io_bytes) return c->fail(GNN_EINVAL, "storage tier: a block larger than the transfer buffers");
    StreamEngine::Bounce* b;
    gnn_status st = bounce_get(c, E, &b);
    if (st != GNN_OK) return st;
    GNN_HIP(hipMemcpyAsync(b->buf, src_dev, (size_t)bytes, hipMemcpyDeviceToHost, stream));
    GNN_HIP(hipEventRecord(b->done, stream));
    b->busy = true;
    b->is_write = true;
    b->arr = id;
    b->off = off;
    b->bytes = bytes;
    return GNN_OK;
}

// ---- pool regions ---------------------------------------------------------------------------
int64_t pool_alloc(StreamEngine& E, int64_t bytes)
{
    for (size_t i = 0; i < E.free_list.size(); ++i) {
        auto& f = E.free_list[i];
        if (f.second >= bytes) {
            const int64_t off = f.first;
            f.first += bytes;
            f.second -= bytes;
            if (f.second == 0) E.free_list.erase(E.free_list.begin() + (long)i);
            return off;
        }
    }
    return -1;
}
void pool_free(StreamEngine& E, int64_t off, int64_t bytes)
{
    auto it = E.free_list.begin();
    while (it != E.free_list.end() && it->first < off) ++it;
    it = E.free_list.insert(it, {off, bytes});
    if (it + 1 != E.free_list.end() && it->first + it->second == (it + 1)->first) {
        it->second += (it + 1)->second;
        E.free_list.erase(it + 1);
    }
    if (it != E.free_list.begin() && (it - 1)->first + (it - 1)->second == it->first) {
        (it - 1)->second += it->second;
        E.free_list.erase(it);
    }
}
std::pair<int64_t, int64_t> largest_free(const StreamEngine& E)
{
    std::pair<int64_t, int64_t> best{0, 0};
    for (const auto& f : E.free_list)
        if (f.second > best.second) best = f;
    return best;
}

gnn_status new_slot(gnn_ctx* c, StreamEngine& E, Slot& out)
{
    if (!E.spare.empty()) {
        out = E.spare.back();
        E.spare.pop_back();
    } else {
        out = Slot{};
        GNN_HIP(hipEventCreateWithFlags(&out.ready, hipEventDisableTiming));
        GNN_HIP(hipEventCreateWithFlags(&out.released, hipEventDisableTiming));
        GNN_HIP(hipEventCreateWithFlags(&out.flushed, hipEventDisableTiming));
    }
    out.part = -1;
    out.dirty = out.pinned = false;
    out.last_use = 0;
    out.has_ready = out.has_released = out.has_flushed = false;
    out.waited = false;
    return GNN_OK;
}

// (Re)cuts a cache over `pool_bytes` at `pool` into slots of `slot_bytes`; contents are dropped.
// Boundary rows of blocks that are not in the cache are gathered by the kernel straight from
// the pinned host array (GNNMI_STREAM_DIRECT=0: every miss loads the whole block instead).
bool direct_gather_enabled()
{
    static const bool on = [] {
        const char* e = std::getenv("GNNMI_STREAM_DIRECT");
        return !(e && e[0] == '0');
    }();
    return on;
}

gnn_status configure(gnn_ctx* c, StreamEngine& E, BlockCache& bc, char* pool, int64_t pool_bytes,
                     int64_t slot_bytes, int64_t row_bytes, char* host, bool writeback, bool identity)
{
    // blocks of a whole array lie exactly max_own rows apart, so that one flat row index reaches
    // every block; the slots of a block cache start on 256-byte boundaries
    if (!identity) slot_bytes = round256(slot_bytes);
    int64_t n = pool_bytes / slot_bytes;
    if (n < 2 && !identity)
        return c->fail(GNN_ENOMEM, "hbm_budget_bytes is too small: a block cache needs room for two "
                                   "partition blocks of the widest layer");
    n = std::min<int64_t>(n, (int64_t)E.k);          // one slot per partition is all that is useful
    bc.pool = pool;
    bc.pool_bytes = pool_bytes;
    bc.slot_bytes = slot_bytes;
    bc.row_bytes = row_bytes;
    bc.host = host;
    bc.host_dev = nullptr;
    int vid;
    int64_t voff;
    if (host && !identity && direct_gather_enabled() && !tier_decode(host, &vid, &voff)) {
        // pinned host memory that is mapped for the device can be read (and written) by kernels directly
        hipPointerAttribute_t at;
        if (hipPointerGetAttributes(&at, host) == hipSuccess && at.type == hipMemoryTypeHost && at.devicePointer)
            bc.host_dev = (const char*)at.devicePointer;
        else
            (void)hipGetLastError();
    }
    if (writeback && bc.host_dev) {
        while ((int32_t)bc.blk_direct.size() < E.k) {
            hipEvent_t a, b;
            GNN_HIP(hipEventCreateWithFlags(&a, hipEventDisableTiming));
            bc.blk_direct.push_back(a);
            GNN_HIP(hipEventCreateWithFlags(&b, hipEventDisableTiming));
            bc.blk_flushed.push_back(b);
        }
        bc.has_blk_direct.assign((size_t)E.k, 0);
        bc.has_blk_flushed.assign((size_t)E.k, 0);
    }
    bc.writeback = writeback;
    bc.identity = identity;
    while ((int64_t)bc.slots.size() > n) {
        E.spare.push_back(bc.slots.back());
        bc.slots.pop_back();
    }
    while ((int64_t)bc.slots.size() < n) {
        Slot sl;
        gnn_status st = new_slot(c, E, sl);
        if (st != GNN_OK) return st;
        bc.slots.push_back(sl);
    }
    bc.nslots = (int32_t)n;
    for (Slot& s : bc.slots) {
        s.part = -1;
        s.dirty = s.pinned = false;
        s.last_use = 0;
        s.has_ready = s.has_released = s.has_flushed = false;
        s.waited = false;
    }
    bc.slot_of.assign((size_t)E.k, -1);
    bc.touched.assign((size_t)E.k, 0);
    return GNN_OK;
}

// Writes a dirty block back to its host rows on the store stream.
gnn_status write_back(gnn_ctx* c, StreamEngine& E, BlockCache& bc, int32_t s)
{
    Slot& sl = bc.slots[(size_t)s];
    const HostMeta& M = c->M;
    const int64_t r0 = M.off[(size_t)sl.part], np = M.off[(size_t)sl.part + 1] - r0;
    if (sl.has_released) GNN_HIP(hipStreamWaitEvent(E.d2h, sl.released, 0));
    if (np > 0) {
        gnn_status cst = copy_d2h(c, E, bc.host + r0 * bc.row_bytes, bc.ptr(s), np * bc.row_bytes, E.d2h);
        if (cst != GNN_OK) return cst;
    }
    GNN_HIP(hipEventRecord(sl.flushed, E.d2h));
    sl.has_flushed = true;
    if (!bc.blk_flushed.empty()) {
        GNN_HIP(hipEventRecord(bc.blk_flushed[(size_t)sl.part], E.d2h));
        bc.has_blk_flushed[(size_t)sl.part] = 1;
    }
    sl.dirty = false;
    ++E.writebacks;
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
    if (bc.identity) return part;
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
    const int kind = bc.writeback ? 1 : 0;
    int32_t s = bc.slot_of[(size_t)part];
    if (s >= 0) {
        ++E.hits[kind];
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
            sl.waited = false;
        } else {
            if (sl.has_released) GNN_HIP(hipStreamWaitEvent(E.h2d, sl.released, 0));
            if (sl.has_flushed) GNN_HIP(hipStreamWaitEvent(E.h2d, sl.flushed, 0));
            if (!bc.has_blk_direct.empty() && bc.has_blk_direct[(size_t)part])
                GNN_HIP(hipStreamWaitEvent(E.h2d, bc.blk_direct[(size_t)part], 0));    // rows added in host memory
            if (!bc.has_blk_flushed.empty() && bc.has_blk_flushed[(size_t)part])
                GNN_HIP(hipStreamWaitEvent(E.h2d, bc.blk_flushed[(size_t)part], 0));   // its own last write-back
            if (np > 0) {
                gnn_status cst = copy_h2d(c, E, bc.ptr(s), bc.host + r0 * bc.row_bytes, np * bc.row_bytes, E.h2d);
                if (cst != GNN_OK) return cst;
            }
            GNN_HIP(hipEventRecord(sl.ready, E.h2d));
            sl.has_ready = true;
            sl.waited = false;
            ++E.loads[kind];
            E.h2d_bytes += np * bc.row_bytes;
        }
        sl.part = part;
        sl.dirty = false;
        bc.slot_of[(size_t)part] = s;
        if (bc.writeback) bc.touched[(size_t)part] = 1;
    }
    Slot& sl = bc.slots[(size_t)s];
    sl.last_use = ++bc.tick;
    if (wait && sl.has_ready && !sl.waited) {
        GNN_HIP(hipStreamWaitEvent(compute, sl.ready, 0));
        sl.waited = true;
    }
    *slot_out = s;
    return GNN_OK;
}

gnn_status mark_used(gnn_ctx* c, BlockCache& bc, int32_t s, hipStream_t compute, bool dirty)
{
    Slot& sl = bc.slots[(size_t)s];
    if (dirty) sl.dirty = true;
    if (bc.identity) return GNN_OK;      // never evicted: nothing has to wait for its last reader
    GNN_HIP(hipEventRecord(sl.released, compute));
    sl.has_released = true;
    return GNN_OK;
}

inline bool has_empty_slot(const BlockCache& bc)
{
    for (const Slot& sl : bc.slots)
        if (sl.part < 0) return true;
    return false;
}

// Gather of the boundary rows of the partition of step t from the cached blocks of layer l-1,
// one source partition at a time.  Leaves the own block pinned and returns its slot.
gnn_status gather_from_cache(gnn_ctx* c, StreamEngine& E, BlockCache& bc, int32_t layer, int32_t t,
                             hipStream_t s, int32_t* own_slot)
{
    const HostMeta& M = c->M;
    const int32_t k = M.k, p = M.sched[(size_t)t];
    const int64_t row_bytes = (int64_t)c->dims[(size_t)layer - 1] * c->es();
    bc.cur_t = t;
    gnn_status st = acquire(c, E, bc, p, s, true, own_slot);
    if (st != GNN_OK) return st;
    bc.slots[(size_t)*own_slot].pinned = true;
    const int64_t* run = M.brun.data() + (size_t)p * ((size_t)k + 1);
    const int64_t b0 = M.boff[(size_t)p];
    Timed timed(c, s, GNN_K_GATHER);
    const bool flat = bc.identity && c->D.bnd_flat;
    for (int32_t q = 0; q < k; ++q) {
        const int64_t len = run[q + 1] - run[q];
        if (len <= 0) continue;
        int32_t sq;
        if (bc.host_dev && bc.slot_of[(size_t)q] < 0 && !has_empty_slot(bc)) {
            // Not cached, and caching it would evict a block that every later partition also
            // needs: read just the rows over the link.  (A partition depends on nearly every
            // other one, so a cache smaller than the array cycles whole blocks for a fraction of
            // their rows; the kernel reads pinned host rows at the full rate of the link.)
            launch_gather_rows(bc.host_dev + M.off[(size_t)q] * row_bytes, c->D.bnd_local + b0 + run[q],
                               c->staging + run[q] * row_bytes, len, row_bytes, s);
            ++E.direct_gathers;
            E.direct_bytes += len * row_bytes;
            E.h2d_bytes += len * row_bytes;
            continue;
        }
        if ((st = acquire(c, E, bc, q, s, true, &sq)) != GNN_OK) return st;
        if (flat) continue;
        launch_gather_rows(bc.ptr(sq), c->D.bnd_local + b0 + run[q], c->staging + run[q] * row_bytes,
                           len, row_bytes, s);
        if ((st = mark_used(c, bc, sq, s, false)) != GNN_OK) return st;
    }
    // a whole array: every block is in place, one launch gathers across all of them
    if (flat) launch_gather_rows(bc.pool, c->D.bnd_flat + b0, c->staging, M.boff[(size_t)p + 1] - b0, row_bytes, s);
    return GNN_OK;
}

// Issues loads for the blocks the partition of step t will need, as long as a slot can be
// taken for them.
gnn_status prefetch_for(gnn_ctx* c, StreamEngine& E, BlockCache& bc, int32_t t, hipStream_t s)
{
    const HostMeta& M = c->M;
    const int32_t k = M.k;
    if (t >= k) return GNN_OK;
    const int32_t p = M.sched[(size_t)t];
    const int64_t* run = M.brun.data() + (size_t)p * ((size_t)k + 1);
    int32_t budget = bc.nslots - 1;      // never cycle the whole cache for a prefetch
    int32_t slot;
    bc.cur_t = t;
    gnn_status st = acquire(c, E, bc, p, s, false, &slot);
    if (st != GNN_OK) return st;
    --budget;
    for (int32_t q = 0; q < k && budget > 0; ++q) {
        if (run[q + 1] - run[q] <= 0) continue;
        if (bc.slot_of[(size_t)q] < 0) {
            if (bc.host_dev && !has_empty_slot(bc)) break;   // its rows will be read from the host
            if ((st = acquire(c, E, bc, q, s, false, &slot)) != GNN_OK) return st;
            if (slot < 0) break;
        }
        --budget;
    }
    return GNN_OK;
}

// ---- whole arrays in the pool -----------------------------------------------------------------
struct Key {
    int kind, layer;
};
inline bool same(const Resident& r, Key key) { return r.kind == key.kind && r.layer == key.layer; }

Resident* find_array(StreamEngine& E, Key key)
{
    for (auto& r : E.arrays)
        if (same(*r, key)) return r.get();
    return nullptr;
}

gnn_status release_array(gnn_ctx* c, StreamEngine& E, Resident* r)
{
    for (int32_t s = 0; s < r->bc.nslots; ++s)
        if (r->bc.slots[(size_t)s].part >= 0 && r->bc.slots[(size_t)s].dirty) {
            gnn_status st = write_back(c, E, r->bc, s);
            if (st != GNN_OK) return st;
        }
    for (Slot& sl : r->bc.slots) E.spare.push_back(sl);
    r->bc.slots.clear();
    pool_free(E, r->off, r->bytes);
    for (size_t i = 0; i < E.arrays.size(); ++i)
        if (E.arrays[i].get() == r) {
            E.arrays.erase(E.arrays.begin() + (long)i);
            break;
        }
    return GNN_OK;
}

bool is_protected(const Resident& r, const Key* keep, int nkeep)
{
    for (int i = 0; i < nkeep; ++i)
        if (same(r, keep[i])) return true;
    return false;
}

// The array to give up when room is needed: among those the current phase does not use, the one
// of the lowest layer (forward will not read it again, backward reads it last).
Resident* pick_array_victim(StreamEngine& E, const Key* keep, int nkeep)
{
    Resident* v = nullptr;
    for (auto& r : E.arrays) {
        if (is_protected(*r, keep, nkeep)) continue;
        if (!v || r->layer < v->layer || (r->layer == v->layer && r->kind < v->kind)) v = r.get();
    }
    return v;
}

// Returns the array `key` if it is in the pool, else tries to give it k slots, evicting arrays
// the phase does not use and then, in the order given, arrays it could use but values less
// (entries may be null; the ones given up are set to null).  `evict` = false: only take free
// room.  *out = nullptr when it does not fit.
gnn_status ensure_array(gnn_ctx* c, StreamEngine& E, Key key, int64_t slot_bytes, int64_t row_bytes,
                        char* host, bool writeback, const Key* keep, int nkeep, Resident*** lesser,
                        int nlesser, bool evict, Resident** out)
{
    *out = find_array(E, key);
    if (*out) return GNN_OK;
    const int64_t bytes = round256((int64_t)E.k * slot_bytes);
    if (bytes > E.pool_bytes) return GNN_OK;
    // worth trying only if it fits once everything that may go has gone
    int64_t could = 0;
    for (const auto& f : E.free_list) could += f.second;
    for (const auto& r : E.arrays) {
        bool may_go = evict && !is_protected(*r, keep, nkeep);
        for (int i = 0; i < nlesser && evict; ++i)
            if (*lesser[i] == r.get()) may_go = true;
        if (may_go) could += r->bytes;
    }
    if (could < bytes) return GNN_OK;
    int64_t off = pool_alloc(E, bytes);
    while (off < 0 && evict) {
        Resident* v = pick_array_victim(E, keep, nkeep);
        for (int i = 0; i < nlesser && !v; ++i)
            if (*lesser[i]) {
                v = *lesser[i];
                *lesser[i] = nullptr;
            }
        if (!v) return GNN_OK;
        gnn_status st = release_array(c, E, v);
        if (st != GNN_OK) return st;
        off = pool_alloc(E, bytes);
    }
    if (off < 0) return GNN_OK;
    std::unique_ptr<Resident> r(new Resident());
    r->kind = key.kind;
    r->layer = key.layer;
    r->off = off;
    r->bytes = bytes;
    gnn_status st = configure(c, E, r->bc, E.pool + off, bytes, slot_bytes, row_bytes, host, writeback, true);
    if (st != GNN_OK) {
        pool_free(E, off, bytes);
        return st;
    }
    *out = r.get();
    E.arrays.push_back(std::move(r));
    return GNN_OK;
}

// Frees every array except those in `keep`: a block cache is about to take what is left.
gnn_status release_others(gnn_ctx* c, StreamEngine& E, const Key* keep, int nkeep)
{
    for (;;) {
        Resident* v = pick_array_victim(E, keep, nkeep);
        if (!v) return GNN_OK;
        gnn_status st = release_array(c, E, v);
        if (st != GNN_OK) return st;
    }
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
    E->io_bytes = round256(M.stats.max_own * dmax * 4);
    // transform-first layers keep H (then grad H) and, for hidden GraphSAGE layers, the dY rows of
    // every partition on the device for a whole layer pass: that comes out of the budget first
    int64_t xf_bytes = 0;
    for (int32_t l = 1; l <= c->L; ++l)
        if (c->transform_first(l)) xf_bytes = c->xf_buffer_bytes(M.n);
    E->pool_bytes = c->hbm_budget / 256 * 256 - xf_bytes;
    // the tightest layer must still fit two activation blocks and two gradient blocks
    const int64_t need = 2 * round256(M.stats.max_own * dmax * c->es()) + 2 * round256(M.stats.max_own * dmax * 4);
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
    // Non-blocking: a caller's compute stream may be the null stream, which would otherwise
    // order itself against every copy on these two (each kernel waiting for the copy before it
    // and the other way round); all real dependencies are expressed with events.
    if ((e = hipStreamCreateWithFlags(&E->h2d, hipStreamNonBlocking)) != hipSuccess) return fail_hip(e, "hipStreamCreate");
    if ((e = hipStreamCreateWithFlags(&E->d2h, hipStreamNonBlocking)) != hipSuccess) return fail_hip(e, "hipStreamCreate");
    if ((e = hipMalloc((void**)&E->pool, (size_t)E->pool_bytes)) != hipSuccess) return fail_hip(e, "hipMalloc(block cache)");
    if ((e = hipMalloc((void**)&E->io, (size_t)(8 * E->io_bytes))) != hipSuccess) return fail_hip(e, "hipMalloc(transfer buffers)");
    if (xf_bytes > 0) {
        if ((e = hipMalloc((void**)&E->xf, (size_t)xf_bytes)) != hipSuccess) return fail_hip(e, "hipMalloc(transform-first buffers)");
        const int64_t hbytes = (c->ws.h_floats * 4 + 255) / 256 * 256;
        c->hbuf = c->ghbuf = E->xf;
        c->dyall_buf = c->ws.dyall_floats > 0 ? (float*)(E->xf + hbytes) : nullptr;
    }
    E->free_list.assign(1, {0, E->pool_bytes});
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
    auto drop = [](std::vector<Slot>& v) {
        for (Slot& s : v) {
            if (s.ready) (void)hipEventDestroy(s.ready);
            if (s.released) (void)hipEventDestroy(s.released);
            if (s.flushed) (void)hipEventDestroy(s.flushed);
        }
        v.clear();
    };
    drop(E->actc.slots);
    drop(E->gradc.slots);
    for (BlockCache* bc : {&E->actc, &E->gradc}) {
        for (hipEvent_t e : bc->blk_direct) (void)hipEventDestroy(e);
        for (hipEvent_t e : bc->blk_flushed) (void)hipEventDestroy(e);
        bc->blk_direct.clear();
        bc->blk_flushed.clear();
    }
    drop(E->spare);
    for (auto& r : E->arrays) drop(r->bc.slots);
    for (int i = 0; i < 2; ++i) {
        if (E->out_ready[i]) (void)hipEventDestroy(E->out_ready[i]);
        if (E->out_done[i]) (void)hipEventDestroy(E->out_done[i]);
        if (E->in_ready[i]) (void)hipEventDestroy(E->in_ready[i]);
        if (E->in_released[i]) (void)hipEventDestroy(E->in_released[i]);
    }
    if (E->layer_done) (void)hipEventDestroy(E->layer_done);
    if (E->compute_done) (void)hipEventDestroy(E->compute_done);
    for (auto& b : E->bounce) {
        if (b.done) (void)hipEventDestroy(b.done);
        if (b.buf) (void)hipHostFree(b.buf);
    }
    if (E->pool) (void)hipFree(E->pool);
    if (E->io) (void)hipFree(E->io);
    if (E->xf) (void)hipFree(E->xf);
    c->hbuf = c->ghbuf = nullptr;
    c->dyall_buf = nullptr;
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
    // nothing survives from an earlier epoch: the weights, and possibly the features, have changed
    while (!E.arrays.empty())
        if ((st = release_array(c, E, E.arrays.back().get())) != GNN_OK) return st;
    E.has_out_done[0] = E.has_out_done[1] = false;
    E.has_in_released[0] = E.has_in_released[1] = false;
    E.h2d_bytes = E.d2h_bytes = 0;
    E.loads[0] = E.loads[1] = E.hits[0] = E.hits[1] = E.writebacks = 0;
    E.direct_gathers = E.direct_bytes = 0;
    E.direct_scatters = E.direct_scatter_bytes = 0;

    zero_weight_grads(c, s);

    // Between phases: the next phase's loads must see this phase's stores, and because regions of
    // the pool change hands, neither loads nor kernels of the next phase may start before this
    // phase's kernels and stores are done with the pool.
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
        if (bytes > 0) {
            gnn_status cst = copy_d2h(c, E, dst, E.outbuf(ob), bytes, E.d2h);
            if (cst != GNN_OK) return cst;
        }
        E.d2h_bytes += bytes;
        GNN_HIP(hipEventRecord(E.out_done[ob], E.d2h));
        E.has_out_done[ob] = true;
        return GNN_OK;
    };
    auto wait_out_free = [&](int ob) -> gnn_status {
        if (E.has_out_done[ob]) GNN_HIP(hipStreamWaitEvent(s, E.out_done[ob], 0));
        return GNN_OK;
    };
    // Block p of a resident array has just been produced on the compute stream: it is valid from
    // now on, and goes to its host rows on the store stream (`bytes` of it).
    auto produced = [&](Resident* r, int32_t p, char* dst, int64_t bytes) -> gnn_status {
        Slot& sl = r->bc.slots[(size_t)p];
        sl.part = p;
        sl.dirty = false;
        sl.has_ready = false;
        r->bc.slot_of[(size_t)p] = p;
        GNN_HIP(hipEventRecord(sl.released, s));
        sl.has_released = true;
        GNN_HIP(hipStreamWaitEvent(E.d2h, sl.released, 0));
        if (bytes > 0) {
            gnn_status cst = copy_d2h(c, E, dst, r->bc.ptr(p), bytes, E.d2h);
            if (cst != GNN_OK) return cst;
        }
        E.d2h_bytes += bytes;
        return GNN_OK;
    };
    auto act_slot_bytes = [&](int32_t layer) {     // a block of A^layer
        return std::max<int64_t>(1, max_np) * (int64_t)c->dims[(size_t)layer] * (layer == 0 ? c->es() : c->act_es(layer));
    };
    auto act_row_bytes = [&](int32_t layer) {
        return (int64_t)c->dims[(size_t)layer] * (layer == 0 ? c->es() : c->act_es(layer));
    };
    auto act_host = [&](int32_t layer) {
        return layer == 0 ? const_cast<char*>(c->feat) : c->act[(size_t)layer - 1];
    };
    auto grad_slot_bytes = [&](int32_t layer) {
        return std::max<int64_t>(1, max_np) * (int64_t)c->dims[(size_t)layer] * 4;
    };

    // Loads rows of a host array into transfer buffer `dst` on the load stream.
    auto load_in = [&](char* dst, const char* src, int64_t bytes, int ib, bool first) -> gnn_status {
        if (first && E.has_in_released[ib]) GNN_HIP(hipStreamWaitEvent(E.h2d, E.in_released[ib], 0));
        if (bytes > 0) {
            gnn_status cst = copy_h2d(c, E, dst, src, bytes, E.h2d);
            if (cst != GNN_OK) return cst;
        }
        E.h2d_bytes += bytes;
        return GNN_OK;
    };
    // One sweep over the partitions of a transform-first layer.  want(t, i) names the host rows of
    // input block i (0: grad A^l, 1: A^l, 2: A^{l-1}) of step t unless the block is in the pool
    // already (then it sets *dev); body(t, ptrs) enqueues the step's kernels.  The blocks of
    // step t + 1 are loaded into the other set of transfer buffers while step t computes.
    struct BlockReq {
        const char* host = nullptr;   // rows to load, or null
        int64_t bytes = 0;
        const char* dev = nullptr;    // where the kernels find the block
        Resident* arr = nullptr;      // block `part` of a whole array: the step waits for its load
        int32_t part = -1;
    };
    auto xf_sweep = [&](auto&& want, auto&& body) -> gnn_status {
        std::vector<BlockReq> req((size_t)3 * 2);
        auto stage = [&](int32_t t) -> gnn_status {
            const int ib = t & 1;
            bool first = true;
            for (int i = 0; i < 3; ++i) {
                BlockReq& r = req[(size_t)ib * 3 + (size_t)i];
                r = BlockReq{};
                gnn_status r_st = want(t, i, r);
                if (r_st != GNN_OK) return r_st;
                if (!r.host) continue;
                char* buf = i == 0 ? E.ginbuf(ib) : i == 1 ? E.ainbuf(ib) : E.xinbuf(ib);
                if ((r_st = load_in(buf, r.host, r.bytes, ib, first)) != GNN_OK) return r_st;
                first = false;
                r.dev = buf;
            }
            GNN_HIP(hipEventRecord(E.in_ready[ib], E.h2d));
            return GNN_OK;
        };
        gnn_status r_st = stage(0);
        if (r_st != GNN_OK) return r_st;
        for (int32_t t = 0; t < k; ++t) {
            const int ib = t & 1;
            if (t + 1 < k && (r_st = stage(t + 1)) != GNN_OK) return r_st;
            GNN_HIP(hipStreamWaitEvent(s, E.in_ready[ib], 0));
            for (int i = 0; i < 3; ++i) {
                BlockReq& r = req[(size_t)ib * 3 + (size_t)i];
                int32_t slot;
                if (r.arr && (r_st = acquire(c, E, r.arr->bc, r.part, s, true, &slot)) != GNN_OK) return r_st;
            }
            if ((r_st = body(t, &req[(size_t)ib * 3])) != GNN_OK) return r_st;
            GNN_HIP(hipEventRecord(E.in_released[ib], s));
            E.has_in_released[ib] = true;
        }
        return GNN_OK;
    };
    // a block of a whole array in the pool: its load is issued here (first use) and the step
    // that reads it waits for it
    auto from_array = [&](Resident* r, int32_t p, BlockReq& out) -> gnn_status {
        int32_t slot;
        gnn_status r_st = acquire(c, E, r->bc, p, s, false, &slot);
        if (r_st != GNN_OK) return r_st;
        out.dev = r->bc.ptr(slot);
        out.arr = r;
        out.part = p;
        return GNN_OK;
    };

    // Storage tier below host memory: before a phase enqueues anything, the arrays it reads or
    // writes are brought into the pinned pool (and the least recently used others leave it).  The
    // device must have finished with whatever may leave, so a phase boundary at which something
    // has to move becomes a host synchronisation; arrays may come back at another address, so the
    // host pointers kept by whole arrays in the HBM pool are renewed (those arrays are clean at a
    // phase boundary).
    // need: (array, overwritten whole by the phase) in the order in which they should get room
    auto tier_phase = [&](std::initializer_list<std::pair<int, bool>> need,
                          std::initializer_list<int> next, std::initializer_list<int> dead) -> gnn_status {
        if (!c->tier) return GNN_OK;
        std::vector<int> nd, nx, dd;
        unsigned overwrite_mask = 0;
        for (const auto& nw : need)
            if (nw.first >= 0) {
                if (nw.second) overwrite_mask |= 1u << nd.size();
                nd.push_back(nw.first);
            }
        for (int id : next) if (id >= 0) nx.push_back(id);
        for (int id : dead) if (id >= 0) dd.push_back(id);
        // only when something has to be read, evicted or moved: otherwise every array stays where
        // it is and the phase is enqueued behind the last one as without the tier
        // blocks of the last phase still on their way to a file
        gnn_status b_st = bounce_drain(c, E, false);
        if (b_st != GNN_OK) return b_st;
        const bool io = tier_needs_io(c, nd.data(), (int)nd.size());
        if (io) {
            GNN_HIP(hipStreamSynchronize(s));
            GNN_HIP(hipStreamSynchronize(E.d2h));
            GNN_HIP(hipStreamSynchronize(E.h2d));
        }
        gnn_status t_st = tier_prepare(c, nd.data(), (int)nd.size(), overwrite_mask, nx.data(), (int)nx.size(),
                                       dd.data(), (int)dd.size(), io);
        if (t_st != GNN_OK) return t_st;
        for (auto& r : E.arrays)
            r->bc.host = r->kind == ARR_ACT ? act_host(r->layer) : (char*)c->gact[(size_t)r->layer - 1];
        return GNN_OK;
    };
    auto act_id = [&](int32_t layer) { return layer >= 0 && layer <= L ? (int)layer : -1; };
    auto grad_id = [&](int32_t layer) { return layer >= 1 && layer <= L ? (int)(L + layer) : -1; };

    // ---------------------------------------------------------------------------- forward
    for (int32_t l = 1; l <= L; ++l) {
        const int32_t dout = c->dims[(size_t)l];
        const Key keep[2] = {{ARR_ACT, l - 1}, {ARR_ACT, l}};
        // reads A^{l-1}, writes every row of A^l
        if (l == 1 && c->tier) tier_epoch_begin(c);
        if ((st = tier_phase({{act_id(l - 1), false}, {act_id(l), true}}, {}, {})) != GNN_OK) return st;
        if (c->transform_first(l)) {
            // Transform-first layer: sweep 1 computes H_p = A_p^{l-1} W for every partition into the
            // whole-graph buffer, sweep 2 gathers and aggregates rows of H.  No partition needs
            // another partition's block of A^{l-1}, so nothing is cached for the gather: an input
            // block comes from a whole array if the pool already holds one, else through a transfer
            // buffer (twice for GraphSAGE, whose self term reads it again in sweep 2).
            Resident* in = nullptr;
            Resident* out = nullptr;
            if ((st = ensure_array(c, E, keep[0], act_slot_bytes(l - 1), act_row_bytes(l - 1), act_host(l - 1), false,
                                   keep, 2, nullptr, 0, true, &in)) != GNN_OK) return st;
            if ((st = ensure_array(c, E, keep[1], act_slot_bytes(l), act_row_bytes(l), act_host(l), false, keep,
                                   2, nullptr, 0, true, &out)) != GNN_OK) return st;
            const int64_t in_row = act_row_bytes(l - 1), out_row = (int64_t)dout * c->act_es(l);
            const bool sage = c->model == GNN_SAGE_MEAN;
            auto want_input = [&](int32_t t, int i, BlockReq& r) -> gnn_status {
                if (i != 2) return GNN_OK;
                const int32_t p = M.sched[(size_t)t];
                if (in) return from_array(in, p, r);
                const int64_t r0 = M.off[(size_t)p], np = M.off[(size_t)p + 1] - r0;
                r.host = act_host(l - 1) + r0 * in_row;
                r.bytes = np * in_row;
                return GNN_OK;
            };
            st = xf_sweep(want_input, [&](int32_t t, const BlockReq* b) -> gnn_status {
                xf_transform_fwd(c, l, M.sched[(size_t)t], b[2].dev, s);
                return GNN_OK;
            });
            if (st != GNN_OK) return st;
            auto want_self = [&](int32_t t, int i, BlockReq& r) -> gnn_status {
                return sage ? want_input(t, i, r) : GNN_OK;
            };
            st = xf_sweep(want_self, [&](int32_t t, const BlockReq* b) -> gnn_status {
                const int32_t p = M.sched[(size_t)t];
                const int64_t r0 = M.off[(size_t)p], np = M.off[(size_t)p + 1] - r0;
                const int64_t b0 = M.boff[(size_t)p], nb = M.boff[(size_t)p + 1] - b0;
                {
                    Timed timed(c, s, GNN_K_GATHER);
                    launch_gather_rows(c->hbuf, c->D.bnd + b0, c->staging, nb, (int64_t)c->padded(l) * c->es(), s);
                }
                char* host_rows = c->act[(size_t)l - 1] + r0 * out_row;
                gnn_status r_st;
                if (out) {
                    xf_aggregate_fwd(c, l, p, b[2].dev, out->bc.ptr(p), s);
                    return produced(out, p, host_rows, np * out_row);
                }
                const int ob = t & 1;
                if ((r_st = wait_out_free(ob)) != GNN_OK) return r_st;
                xf_aggregate_fwd(c, l, p, b[2].dev, E.outbuf(ob), s);
                return store_out(ob, host_rows, np * out_row);
            });
            if (st != GNN_OK) return st;
            if ((st = end_of_layer()) != GNN_OK) return st;
            continue;
        }
        // the layer's input as a whole array if it fits, and then its output as well; an input
        // that does not fit is streamed through a block cache over the whole pool
        Resident* in = nullptr;
        Resident* out = nullptr;
        if ((st = ensure_array(c, E, keep[0], act_slot_bytes(l - 1), act_row_bytes(l - 1), act_host(l - 1), false,
                               keep, 2, nullptr, 0, true, &in)) != GNN_OK) return st;
        if (in && (st = ensure_array(c, E, keep[1], act_slot_bytes(l), act_row_bytes(l), act_host(l), false, keep,
                                     2, nullptr, 0, true, &out)) != GNN_OK) return st;
        BlockCache* src = in ? &in->bc : &E.actc;
        if (!in) {
            if ((st = release_others(c, E, nullptr, 0)) != GNN_OK) return st;
            const auto region = largest_free(E);
            st = configure(c, E, E.actc, E.pool + region.first, region.second, act_slot_bytes(l - 1),
                           act_row_bytes(l - 1), act_host(l - 1), false, false);
            if (st != GNN_OK) return st;
        }
        const int64_t out_row = (int64_t)dout * c->act_es(l);
        for (int32_t t = 0; t < k; ++t) {
            const int32_t p = M.sched[(size_t)t];
            const int64_t r0 = M.off[(size_t)p], np = M.off[(size_t)p + 1] - r0;
            int32_t own;
            if ((st = gather_from_cache(c, E, *src, l, t, s, &own)) != GNN_OK) return st;
            if ((st = prefetch_for(c, E, *src, t + 1, s)) != GNN_OK) return st;
            char* host_rows = c->act[(size_t)l - 1] + r0 * out_row;
            if (out) {
                compute_fwd(c, l, p, src->ptr(own), out->bc.ptr(p), s);
                if ((st = produced(out, p, host_rows, np * out_row)) != GNN_OK) return st;
            } else {
                const int ob = t & 1;
                if ((st = wait_out_free(ob)) != GNN_OK) return st;
                compute_fwd(c, l, p, src->ptr(own), E.outbuf(ob), s);
                if ((st = store_out(ob, host_rows, np * out_row)) != GNN_OK) return st;
            }
            if ((st = mark_used(c, *src, own, s, false)) != GNN_OK) return st;
            src->slots[(size_t)own].pinned = false;
        }
        if ((st = end_of_layer()) != GNN_OK) return st;
    }

    // ------------------------------------------------------------------------------- loss
    float* scal = (float*)(c->scratch + c->ws.scalars);
    unsigned long long* count_dev = (unsigned long long*)(scal + 16);
    float* losspart = (float*)(c->scratch + c->ws.losspart);
    {
        const int32_t C = c->dims[(size_t)L];
        const Key keep[3] = {{ARR_ACT, L}, {ARR_GRAD, L}, {ARR_ACT, L - 1}};
        // reads the logits, writes every row of grad A^L; the backward pass of layer L reads A^{L-1} next
        // (the output layer has no activation to differentiate: the logits are not read again)
        if ((st = tier_phase({{act_id(L), false}, {grad_id(L), true}}, {act_id(L - 1)}, {act_id(L)})) != GNN_OK) return st;
        Resident* logits = find_array(E, keep[0]);
        Resident* gout = nullptr;
        // kept for the backward pass of layer L only if there is free room for it
        if ((st = ensure_array(c, E, keep[1], grad_slot_bytes(L), (int64_t)C * 4, (char*)c->gact[(size_t)L - 1],
                               false, keep, 3, nullptr, 0, false, &gout)) != GNN_OK) return st;
        launch_count_mask(c->mask, M.n, count_dev, s);
        int64_t nparts = 0;
        for (int32_t p = 0; p < k; ++p) {
            const int64_t r0 = M.off[(size_t)p], np = M.off[(size_t)p + 1] - r0;
            const int ib = p & 1;
            const float* x;
            const bool have = logits && logits->bc.holds(p);
            if (have) {
                x = (const float*)logits->bc.ptr(p);
            } else {
                if ((st = load_in(E.ainbuf(ib), c->act[(size_t)L - 1] + r0 * C * 4, np * C * 4, ib, true)) != GNN_OK) return st;
                GNN_HIP(hipEventRecord(E.in_ready[ib], E.h2d));
                GNN_HIP(hipStreamWaitEvent(s, E.in_ready[ib], 0));
                x = (const float*)E.ainbuf(ib);
            }
            float* g;
            if (gout) g = (float*)gout->bc.ptr(p);
            else {
                if ((st = wait_out_free(ib)) != GNN_OK) return st;
                g = (float*)E.outbuf(ib);
            }
            {
                Timed timed(c, s, GNN_K_LOSS);
                nparts += launch_loss_rows(x, c->labels + r0, c->mask + r0, g, np, C, count_dev, losspart + nparts, s);
            }
            if (!have) {
                GNN_HIP(hipEventRecord(E.in_released[ib], s));
                E.has_in_released[ib] = true;
            }
            char* host_rows = (char*)(c->gact[(size_t)L - 1] + r0 * C);
            if (gout) st = produced(gout, p, host_rows, np * C * 4);
            else st = store_out(ib, host_rows, np * C * 4);
            if (st != GNN_OK) return st;
        }
        launch_loss_finish(losspart, nparts, count_dev, scal, s);
        if ((st = end_of_layer()) != GNN_OK) return st;
        // the logits are not read again (the output layer has no activation to differentiate)
        if (logits && (st = release_array(c, E, logits)) != GNN_OK) return st;
    }

    // --------------------------------------------------------------------------- backward
    for (int32_t l = L; l >= 1; --l) {
        const int32_t din = c->dims[(size_t)l - 1], dout = c->dims[(size_t)l];
        const int64_t act_row = (int64_t)dout * c->act_es(l);
        const bool need_prev = l >= 2;
        const Key keep[4] = {{ARR_GRAD, l - 1}, {ARR_ACT, l - 1}, {ARR_GRAD, l}, {ARR_ACT, l}};
        const int64_t a_slot = act_slot_bytes(l - 1), g_slot = grad_slot_bytes(l - 1);
        const int64_t a_blk = round256(a_slot), g_blk = round256(g_slot);      // slots of a block cache
        // reads grad A^l, A^l (hidden layers) and A^{l-1}, writes every row of grad A^{l-1}; the
        // layer below reads A^{l-2} next
        // (room goes first to the gather source, whose rows are read by many partitions, then to the
        // gradient being accumulated; grad A^l and A^l are read one own block per partition)
        if ((st = tier_phase({{act_id(l - 1), false}, {grad_id(l - 1), true}, {grad_id(l), false},
                              {l < L ? act_id(l) : -1, false}},
                             {act_id(l - 2)}, {grad_id(l), l < L ? act_id(l) : -1})) != GNN_OK) return st;
        if (c->transform_first(l)) {
            // Transform-first layer: sweep 1 scatter-accumulates S_p^T dY_p into the whole-graph
            // buffer grad H (so no block of grad A^{l-1} is ever cycled through a cache), sweep 2
            // produces grad A_p^{l-1} block by block, each written once.  Input blocks come from
            // whole arrays still in the pool, else through transfer buffers.
            Resident* gin = find_array(E, keep[2]);
            Resident* ain = l < L ? find_array(E, keep[3]) : nullptr;
            Resident* srcarr = nullptr;
            Resident* gout = nullptr;
            // A^{l-1} is read in both sweeps: a whole array if it fits beside what is there; then
            // the output grad A^{l-1}, which the layer below reads next
            if ((st = ensure_array(c, E, keep[1], a_slot, act_row_bytes(l - 1), act_host(l - 1), false, keep, 4,
                                   nullptr, 0, true, &srcarr)) != GNN_OK) return st;
            if (need_prev && (st = ensure_array(c, E, keep[0], g_slot, (int64_t)din * 4, (char*)c->gact[(size_t)l - 2],
                                                false, keep, 4, nullptr, 0, true, &gout)) != GNN_OK) return st;
            const bool sage = c->model == GNN_SAGE_MEAN;
            const bool hidden_sage = sage && need_prev && l < L;    // its second sweep takes dY_p again
            const int64_t in_row = act_row_bytes(l - 1);
            auto block = [&](int32_t t, int i, BlockReq& r) -> gnn_status {
                const int32_t p = M.sched[(size_t)t];
                const int64_t r0 = M.off[(size_t)p], np = M.off[(size_t)p + 1] - r0;
                Resident* arr = i == 0 ? gin : i == 1 ? ain : srcarr;
                if (arr && (i == 2 || arr->bc.holds(p))) {
                    if (i == 2) return from_array(arr, p, r);
                    r.dev = arr->bc.ptr(p);
                    return GNN_OK;
                }
                if (i == 0) { r.host = (const char*)(c->gact[(size_t)l - 1] + r0 * dout); r.bytes = np * dout * 4; }
                else if (i == 1) { r.host = c->act[(size_t)l - 1] + r0 * act_row; r.bytes = np * act_row; }
                else { r.host = act_host(l - 1) + r0 * in_row; r.bytes = np * in_row; }
                return GNN_OK;
            };
            xf_begin_bwd(c, l, s);
            st = xf_sweep([&](int32_t t, int i, BlockReq& r) -> gnn_status {
                              if (i == 1 && l == L) return GNN_OK;        // the output layer has no activation
                              if (i == 2 && !sage) return GNN_OK;         // A^{l-1} feeds the self-weight gradient only
                              return block(t, i, r);
                          },
                          [&](int32_t t, const BlockReq* b) -> gnn_status {
                              xf_aggregate_bwd(c, l, M.sched[(size_t)t], b[2].dev, (const float*)b[0].dev, b[1].dev, nullptr, s);
                              return GNN_OK;
                          });
            if (st != GNN_OK) return st;
            st = xf_sweep([&](int32_t t, int i, BlockReq& r) -> gnn_status {
                              if (i == 1 && !hidden_sage) return GNN_OK;
                              // dY of a GraphSAGE layer: grad A^L itself, or taken again from grad A^l and A^l
                              if (i == 0 && !((sage && l == L && need_prev) || hidden_sage)) return GNN_OK;
                              return block(t, i, r);
                          },
                          [&](int32_t t, const BlockReq* b) -> gnn_status {
                              const int32_t p = M.sched[(size_t)t];
                              const int64_t r0 = M.off[(size_t)p], np = M.off[(size_t)p + 1] - r0;
                              if (!need_prev) {
                                  xf_transform_bwd(c, l, p, b[2].dev, (const float*)b[0].dev, nullptr, nullptr, s);
                                  return GNN_OK;
                              }
                              char* host_rows = (char*)(c->gact[(size_t)l - 2] + r0 * din);
                              gnn_status r_st;
                              if (gout) {
                                  xf_transform_bwd(c, l, p, b[2].dev, (const float*)b[0].dev, b[1].dev, (float*)gout->bc.ptr(p), s);
                                  return produced(gout, p, host_rows, np * din * 4);
                              }
                              const int ob = t & 1;
                              if ((r_st = wait_out_free(ob)) != GNN_OK) return r_st;
                              xf_transform_bwd(c, l, p, b[2].dev, (const float*)b[0].dev, b[1].dev, (float*)E.outbuf(ob), s);
                              return store_out(ob, host_rows, np * din * 4);
                          });
            if (st != GNN_OK) return st;
            if ((st = end_of_layer()) != GNN_OK) return st;
            if (Resident* r = find_array(E, keep[2]))
                if ((st = release_array(c, E, r)) != GNN_OK) return st;
            if (Resident* r = find_array(E, keep[3]))
                if ((st = release_array(c, E, r)) != GNN_OK) return st;
            continue;
        }
        // Whole arrays where they fit: the gradient being accumulated first (a block of it that is
        // evicted costs a write-back and a reload), then the gather source; the partition's own
        // gradient and activation blocks are taken from arrays that are still in the pool.
        Resident* acc = nullptr;
        Resident* srcarr = find_array(E, keep[1]);
        Resident* gin = find_array(E, keep[2]);
        Resident* ain = l < L ? find_array(E, keep[3]) : nullptr;
        {
            Resident** lesser[3] = {&ain, &gin, &srcarr};
            if (need_prev && (st = ensure_array(c, E, keep[0], g_slot, (int64_t)din * 4, (char*)c->gact[(size_t)l - 2],
                                                true, keep, 4, lesser, 3, true, &acc)) != GNN_OK) return st;
            if (!srcarr && (acc || !need_prev) &&
                (st = ensure_array(c, E, keep[1], a_slot, act_row_bytes(l - 1), act_host(l - 1), false, keep, 4,
                                   lesser, 2, true, &srcarr)) != GNN_OK) return st;
        }
        if ((need_prev && !acc) || !srcarr) {
            // something is streamed: its block cache is worth more than the partition's own blocks
            // staying in the pool
            Key stay[2];
            int nstay = 0;
            if (acc) stay[nstay++] = keep[0];
            if (srcarr) stay[nstay++] = keep[1];
            if ((st = release_others(c, E, stay, nstay)) != GNN_OK) return st;
            gin = ain = nullptr;
            const int64_t need = (need_prev && !acc ? 2 * g_blk : 0) + (!srcarr ? 2 * a_blk : 0);
            if (largest_free(E).second < need && srcarr) {
                if ((st = release_array(c, E, srcarr)) != GNN_OK) return st;
                srcarr = nullptr;
            }
            if (largest_free(E).second < (need_prev && !acc ? 2 * g_blk : 0) + (!srcarr ? 2 * a_blk : 0) && acc) {
                if ((st = release_array(c, E, acc)) != GNN_OK) return st;
                acc = nullptr;
            }
        }
        BlockCache* src = srcarr ? &srcarr->bc : &E.actc;
        BlockCache* dst = acc ? &acc->bc : &E.gradc;
        {
            const bool stream_acc = need_prev && !acc, stream_src = !srcarr;
            const auto region = largest_free(E);
            int64_t grad_bytes = 0;
            if (stream_acc && stream_src) {
                // a gradient block that is evicted costs two transfers, an activation block one:
                // all k gradient blocks when they fit beside two activation blocks, else two thirds
                grad_bytes = (int64_t)k * g_blk;
                if (region.second - grad_bytes < 2 * a_blk) {
                    grad_bytes = region.second / 3 * 2 / 256 * 256;
                    grad_bytes = std::min(grad_bytes, region.second - 2 * a_blk);
                    grad_bytes = std::max(grad_bytes, 2 * g_blk);
                }
            } else if (stream_acc) {
                grad_bytes = region.second;
            }
            if (stream_src) {
                st = configure(c, E, E.actc, E.pool + region.first, (region.second - grad_bytes) / 256 * 256, a_slot,
                               act_row_bytes(l - 1), act_host(l - 1), false, false);
                if (st != GNN_OK) return st;
            }
            if (stream_acc) {
                st = configure(c, E, E.gradc, E.pool + region.first + (region.second - grad_bytes), grad_bytes,
                               g_slot, (int64_t)din * 4, (char*)c->gact[(size_t)l - 2], true, false);
                if (st != GNN_OK) return st;
            }
        }
        // transfer buffers of the partition of step t: its gradient block and (hidden layers) its
        // activations, unless they are in the pool already
        auto load_io = [&](int32_t t) -> gnn_status {
            const int32_t p = M.sched[(size_t)t];
            const int64_t r0 = M.off[(size_t)p], np = M.off[(size_t)p + 1] - r0;
            const int ib = t & 1;
            bool first = true;
            if (!(gin && gin->bc.holds(p))) {
                gnn_status r = load_in(E.ginbuf(ib), (const char*)(c->gact[(size_t)l - 1] + r0 * dout),
                                       np * dout * 4, ib, first);
                if (r != GNN_OK) return r;
                first = false;
            }
            if (l < L && !(ain && ain->bc.holds(p))) {
                gnn_status r = load_in(E.ainbuf(ib), c->act[(size_t)l - 1] + r0 * act_row, np * act_row, ib, first);
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
            if ((st = gather_from_cache(c, E, *src, l, t, s, &own)) != GNN_OK) return st;
            if ((st = prefetch_for(c, E, *src, t + 1, s)) != GNN_OK) return st;
            if (t + 1 < k && (st = load_io(t + 1)) != GNN_OK) return st;
            GNN_HIP(hipStreamWaitEvent(s, E.in_ready[ib], 0));
            const float* g_own = gin && gin->bc.holds(p) ? (const float*)gin->bc.ptr(p) : (const float*)E.ginbuf(ib);
            const char* a_own = nullptr;
            if (l < L) a_own = ain && ain->bc.holds(p) ? ain->bc.ptr(p) : E.ainbuf(ib);
            // The accumulator as a whole array: the transposed aggregation adds its rows straight
            // onto their owners, as in the resident schedule, once every owner block exists.
            const bool fused = need_prev && acc && c->D.bnd_flat;
            const int64_t* run = M.brun.data() + (size_t)p * ((size_t)k + 1);
            const int64_t b0 = M.boff[(size_t)p];
            int32_t gown = -1;
            SpmmScatter map;
            if (fused) {
                dst->cur_t = t;
                if ((st = acquire(c, E, *dst, p, s, true, &gown)) != GNN_OK) return st;
                if ((st = mark_used(c, *dst, gown, s, true)) != GNN_OK) return st;
                for (int32_t q = 0; q < k; ++q) {
                    if (run[q + 1] - run[q] <= 0) continue;
                    int32_t gq;
                    if ((st = acquire(c, E, *dst, q, s, true, &gq)) != GNN_OK) return st;
                    if ((st = mark_used(c, *dst, gq, s, true)) != GNN_OK) return st;
                }
                map.n_own = np;
                map.base_row = (int64_t)p * max_np;
                map.idx = c->D.bnd_flat + b0;
            }
            const char* dY = compute_bwd(c, l, p, src->ptr(own), g_own, a_own, fused ? (float*)dst->pool : nullptr,
                                         fused ? &map : nullptr, s);
            if ((st = mark_used(c, *src, own, s, false)) != GNN_OK) return st;
            src->slots[(size_t)own].pinned = false;
            if (fused) {
                compute_bwd_self(c, l, p, dY, (float*)dst->ptr(gown), s);
            } else if (need_prev) {
                // scatter-accumulate the gradient of the gathered rows, owner block by owner block
                const float* dGA = (const float*)(c->scratch + c->ws.dga);
                dst->cur_t = t;
                if ((st = acquire(c, E, *dst, p, s, true, &gown)) != GNN_OK) return st;
                dst->slots[(size_t)gown].pinned = true;
                {
                    Timed timed(c, s, GNN_K_SCATTER);
                    launch_scatter_add(dGA, np, np, 0, nullptr, (float*)dst->ptr(gown), din, s);
                    for (int32_t q = 0; q < k; ++q) {
                        const int64_t len = run[q + 1] - run[q];
                        if (len <= 0) continue;
                        if (dst->host_dev && !dst->blk_direct.empty() && dst->slot_of[(size_t)q] < 0 &&
                            !has_empty_slot(*dst)) {
                            // The owner block is not cached and caching it would push out a block that
                            // later partitions add to as well (each partition touches nearly every
                            // owner): add these rows where the block lives, in the pinned host array
                            // (the paper accumulates on the host too).  The kernel reads and writes
                            // the rows over the link; stream order keeps the sum in partition order.
                            const int64_t q0 = M.off[(size_t)q], nq = M.off[(size_t)q + 1] - q0;
                            float* hostq = (float*)const_cast<char*>(dst->host_dev) + q0 * din;
                            if (dst->has_blk_flushed[(size_t)q])
                                GNN_HIP(hipStreamWaitEvent(s, dst->blk_flushed[(size_t)q], 0));
                            if (!dst->touched[(size_t)q]) {
                                launch_fill_zero(hostq, nq * (int64_t)din * 4, s);
                                dst->touched[(size_t)q] = 1;
                                E.d2h_bytes += nq * (int64_t)din * 4;
                            }
                            launch_scatter_add(dGA + (np + run[q]) * din, len, 0, 0, c->D.bnd_local + b0 + run[q],
                                               hostq, din, s);
                            GNN_HIP(hipEventRecord(dst->blk_direct[(size_t)q], s));
                            dst->has_blk_direct[(size_t)q] = 1;
                            ++E.direct_scatters;
                            E.direct_scatter_bytes += 2 * len * (int64_t)din * 4;
                            E.h2d_bytes += len * (int64_t)din * 4;
                            E.d2h_bytes += len * (int64_t)din * 4;
                            continue;
                        }
                        int32_t gq;
                        if ((st = acquire(c, E, *dst, q, s, true, &gq)) != GNN_OK) return st;
                        launch_scatter_add(dGA + (np + run[q]) * din, len, 0, 0, c->D.bnd_local + b0 + run[q],
                                           (float*)dst->ptr(gq), din, s);
                        if ((st = mark_used(c, *dst, gq, s, true)) != GNN_OK) return st;
                    }
                }
                compute_bwd_self(c, l, p, dY, (float*)dst->ptr(gown), s);
                if ((st = mark_used(c, *dst, gown, s, true)) != GNN_OK) return st;
                dst->slots[(size_t)gown].pinned = false;
            }
            // dY may alias the gradient transfer buffer: release it only now
            GNN_HIP(hipEventRecord(E.in_released[ib], s));
            E.has_in_released[ib] = true;
        }
        if (need_prev) {
            // end of the layer: every gradient block goes back to its host rows (and, in a whole
            // array, stays where it is for the next layer's backward pass)
            if (dst->identity) {
                GNN_HIP(hipEventRecord(E.compute_done, s));
                GNN_HIP(hipStreamWaitEvent(E.d2h, E.compute_done, 0));
            }
            for (int32_t sidx = 0; sidx < dst->nslots; ++sidx)
                if (dst->slots[(size_t)sidx].part >= 0 && dst->slots[(size_t)sidx].dirty)
                    if ((st = write_back(c, E, *dst, sidx)) != GNN_OK) return st;
        }
        if ((st = end_of_layer()) != GNN_OK) return st;
        // grad A^l and A^l are dead from here on
        if (Resident* r = find_array(E, keep[2]))
            if ((st = release_array(c, E, r)) != GNN_OK) return st;
        if (Resident* r = find_array(E, keep[3]))
            if ((st = release_array(c, E, r)) != GNN_OK) return st;
    }

    GNN_HIP(hipStreamSynchronize(s));
    GNN_HIP(hipStreamSynchronize(E.h2d));
    GNN_HIP(hipStreamSynchronize(E.d2h));
    if (c->tier && (st = bounce_drain(c, E, false)) != GNN_OK) return st;
    GNN_HIP(hipMemcpy(loss_out, scal, sizeof(float), hipMemcpyDeviceToHost));
    c->loss_done = true;
    c->stream_stats.act_loads = E.loads[0];
    c->stream_stats.act_hits = E.hits[0];
    c->stream_stats.grad_loads = E.loads[1];
    c->stream_stats.grad_hits = E.hits[1];
    c->stream_stats.grad_writebacks = E.writebacks;
    c->stream_stats.h2d_bytes = E.h2d_bytes;
    c->stream_stats.d2h_bytes = E.d2h_bytes;
    c->stream_stats.direct_gathers = E.direct_gathers;
    c->stream_stats.direct_bytes = E.direct_bytes;
    c->stream_stats.direct_scatters = E.direct_scatters;
    c->stream_stats.direct_scatter_bytes = E.direct_scatter_bytes;
    return check_launch(c, "gnn_epoch (streaming)");
}

}  // namespace gnnmi
