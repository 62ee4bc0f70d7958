// Storage tier below host memory for the streaming schedule (the paper's partition-wise cache
// management section, first two modes of its replacement policy; appendix on running without
// GPUDirect Storage).
//
// The streaming schedule treats pinned host memory as the backing store of every per-layer
// array (A^0 = features, A^1..A^L, grad A^1..grad A^L) and HBM as their cache.  With this tier
// the backing store is a directory of files, one per array, and pinned host memory becomes a
// cache of whole arrays in a pool of a fixed size:
//   - while the pool holds every array nothing is ever written to or read from the files after
//     the first placement ("the cache retains complete layers");
//   - when room is needed, whole arrays leave in least-recently-used order, written to their file
//     first if they changed since they were last stored there ("evicts entire layers in LRU
//     order");
//   - an array that a phase overwrites completely (the output activations of a forward layer, the
//     gradient a backward layer produces) is given room without being read;
//   - the arrays of the next phase are brought in by a helper thread while the current phase
//     computes, as long as that needs no room of an array the current phase uses.
// When the pool cannot hold the arrays of one phase together (the regime of the paper's third
// mode, partition-wise eviction), the arrays that do not fit are not cached in host memory at
// all: the phase reads and writes them partition block by partition block, straight between
// their file and the device through a few small pinned buffers (the schedule's side: "virtual"
// host addresses, see tier_virtual_base) - the paper's bypass path for data with little reuse in
// host memory.  Reuse of such blocks then happens in the HBM block cache alone.  The arrays a
// phase names first (its gather source, then the gradient it accumulates) get the room.
//
// All file traffic is plain pread / pwrite in large chunks on host threads; device work never
// touches an array that is not in the pool, because the schedule asks for the arrays of a phase
// (tier_prepare) before it enqueues anything of that phase and waits for the device to finish
// with a phase before the next request may evict.
#include <fcntl.h>
#include <sys/stat.h>
#include <unistd.h>

#include <algorithm>
#include <cerrno>
#include <condition_variable>
#include <cstring>
#include <mutex>
#include <thread>

#include "gnn_ctx.h"

namespace gnnmi {

struct TierArray {
    int64_t bytes = 0;
    int fd = -1;
    int64_t off = -1;           // offset in the pool, -1: not in host memory
    bool dirty = false;         // host copy newer than the file
    bool on_disk = false;       // the file holds the array
    bool busy = false;          // the helper thread is loading it
    bool dead = false;          // not read again before the next epoch overwrites it
    bool bypass = false;        // used by the running phase without being in the pool
    int64_t last_use = 0;
};

struct StorageTier {
    std::string dir;
    char* pool = nullptr;
    int64_t pool_bytes = 0;
    std::vector<std::pair<int64_t, int64_t>> free_list;   // (offset, bytes), ascending, coalesced
    std::vector<TierArray> arr;                           // 0..L: A^l, L+1..2L: grad A^l
    int64_t tick = 0;
    bool keep_results = true;   // write arrays back even when the epoch itself will not read them again
    gnn_storage_stats stats{};
    // helper thread: loads the arrays named in `wanted` when that needs no eviction
    std::mutex mu;
    std::condition_variable cv;
    std::thread worker;
    std::vector<int> wanted;
    std::vector<int> cur_need;  // arrays of the running phase: the helper thread leaves them alone
    bool device_idle_at_phase_start = false;   // else the device may still read arrays of the phase before
    bool stop = false, working = false;
    std::string worker_error;
};

namespace {

constexpr int64_t kChunk = (int64_t)64 << 20;

int64_t tier_alloc(StorageTier& T, int64_t bytes)
{
    for (size_t i = 0; i < T.free_list.size(); ++i) {
        auto& f = T.free_list[i];
        if (f.second >= bytes) {
            const int64_t off = f.first;
            f.first += bytes;
            f.second -= bytes;
            if (f.second == 0) T.free_list.erase(T.free_list.begin() + (long)i);
            return off;
        }
    }
    return -1;
}

void tier_free(StorageTier& T, int64_t off, int64_t bytes)
{
    auto it = T.free_list.begin();
    while (it != T.free_list.end() && it->first < off) ++it;
    it = T.free_list.insert(it, {off, bytes});
    if (it + 1 != T.free_list.end() && it->first + it->second == (it + 1)->first) {
        it->second += (it + 1)->second;
        T.free_list.erase(it + 1);
    }
    if (it != T.free_list.begin() && (it - 1)->first + (it - 1)->second == it->first) {
        (it - 1)->second += it->second;
        T.free_list.erase(it);
    }
}

bool write_all(int fd, const char* src, int64_t bytes, std::string& err)
{
    for (int64_t done = 0; done < bytes;) {
        const ssize_t w = pwrite(fd, src + done, (size_t)std::min(kChunk, bytes - done), (off_t)done);
        if (w < 0) {
            if (errno == EINTR) continue;
            err = std::string("pwrite: ") + std::strerror(errno);
            return false;
        }
        done += w;
    }
    return true;
}

bool read_all(int fd, char* dst, int64_t bytes, std::string& err)
{
    for (int64_t done = 0; done < bytes;) {
        const ssize_t r = pread(fd, dst + done, (size_t)std::min(kChunk, bytes - done), (off_t)done);
        if (r < 0) {
            if (errno == EINTR) continue;
            err = std::string("pread: ") + std::strerror(errno);
            return false;
        }
        if (r == 0) {
            err = "pread: file shorter than the array";
            return false;
        }
        done += r;
    }
    return true;
}

// Takes array `id` out of host memory (lock held; never a busy one).
bool evict(StorageTier& T, int id, std::string& err)
{
    TierArray& a = T.arr[(size_t)id];
    if (a.dirty && a.dead && !T.keep_results) {
        // nobody will read it: the next epoch overwrites it
        a.dirty = false;
        a.on_disk = false;
        ++T.stats.dropped;
    }
    if (a.dirty) {
        if (!write_all(a.fd, T.pool + a.off, a.bytes, err)) return false;
        a.dirty = false;
        a.on_disk = true;
        T.stats.bytes_written += a.bytes;
        ++T.stats.writebacks;
    }
    tier_free(T, a.off, a.bytes);
    a.off = -1;
    ++T.stats.evictions;
    return true;
}

// Room for array `id` (lock held).  `keep`: arrays that must stay.  background = true (the helper
// thread, while the device works on the arrays in `keep`): only arrays the epoch is done with may
// leave and nothing is moved; a.off stays -1 when that is not enough.
bool make_room(StorageTier& T, int id, const std::vector<int>& keep, bool background, std::string& err)
{
    TierArray& a = T.arr[(size_t)id];
    for (;;) {
        a.off = tier_alloc(T, a.bytes);
        if (a.off >= 0) return true;
        int victim = -1;
        for (int j = 0; j < (int)T.arr.size(); ++j) {
            const TierArray& v = T.arr[(size_t)j];
            if (v.off < 0 || v.busy || j == id) continue;
            if (background && (!v.dead || !T.device_idle_at_phase_start)) continue;
            if (std::find(keep.begin(), keep.end(), j) != keep.end()) continue;
            // arrays the epoch is done with go first, then the least recently used
            if (victim < 0 || (v.dead && !T.arr[(size_t)victim].dead) ||
                (v.dead == T.arr[(size_t)victim].dead && v.last_use < T.arr[(size_t)victim].last_use))
                victim = j;
        }
        if (victim < 0 && background) return true;      // (a.off stays -1)
        if (victim < 0) {
            // nothing left to evict: if the free room is enough but scattered, move the arrays
            // together (the device is idle and the helper thread is not reading)
            int64_t free_total = 0;
            for (const auto& f : T.free_list) free_total += f.second;
            if (free_total >= a.bytes && T.free_list.size() > 1) {
                std::vector<int> order;
                for (int j = 0; j < (int)T.arr.size(); ++j)
                    if (T.arr[(size_t)j].off >= 0) order.push_back(j);
                std::sort(order.begin(), order.end(),
                          [&](int x, int y) { return T.arr[(size_t)x].off < T.arr[(size_t)y].off; });
                int64_t at = 0;
                for (int j : order) {
                    TierArray& v = T.arr[(size_t)j];
                    if (v.off != at) std::memmove(T.pool + at, T.pool + v.off, (size_t)v.bytes);
                    v.off = at;
                    at += v.bytes;
                }
                T.free_list.assign(1, {at, T.pool_bytes - at});
                ++T.stats.compactions;
                continue;
            }
            err = "the host pool of the storage tier cannot hold the arrays of one phase together";
            return false;
        }
        if (!evict(T, victim, err)) return false;
    }
}

void worker_main(StorageTier* T)
{
    std::unique_lock<std::mutex> lk(T->mu);
    for (;;) {
        T->cv.wait(lk, [&] { return T->stop || !T->wanted.empty(); });
        if (T->stop) return;
        const int id = T->wanted.back();
        T->wanted.pop_back();
        TierArray& a = T->arr[(size_t)id];
        if (a.off >= 0 || !a.on_disk || a.busy) continue;
        std::string err;
        if (!make_room(*T, id, T->cur_need, true, err)) {
            T->worker_error = err;
            continue;
        }
        if (a.off < 0) continue;                 // no room: the phase will load it
        a.busy = true;
        T->working = true;
        char* dst = T->pool + a.off;
        const int fd = a.fd;
        const int64_t bytes = a.bytes;
        lk.unlock();
        const bool ok = read_all(fd, dst, bytes, err);
        lk.lock();
        a.busy = false;
        T->working = false;
        if (ok) {
            T->stats.bytes_read += bytes;
            ++T->stats.loads;
            ++T->stats.prefetched;
            a.dead = false;
            a.last_use = ++T->tick;
        } else {
            tier_free(*T, a.off, a.bytes);
            a.off = -1;
            T->worker_error = err;
        }
        T->cv.notify_all();
    }
}

}  // namespace

int tier_array_id(const gnn_ctx* c, int kind, int layer)
{
    if (kind == 0) return layer >= 0 && layer <= c->L ? layer : -1;
    return layer >= 1 && layer <= c->L ? c->L + layer : -1;
}

int64_t tier_array_bytes(const gnn_ctx* c, int id)
{
    const int32_t L = c->L;
    const int layer = id <= L ? id : id - L;
    const int64_t es = id > L ? 4 : (layer == 0 ? c->es() : c->act_es(layer));
    return c->M.n * (int64_t)c->dims[(size_t)layer] * es;
}

void tier_close(gnn_ctx* c)
{
    StorageTier* T = c->tier;
    if (!T) return;
    if (T->worker.joinable()) {
        {
            std::lock_guard<std::mutex> lk(T->mu);
            T->stop = true;
        }
        T->cv.notify_all();
        T->worker.join();
    }
    for (size_t i = 0; i < T->arr.size(); ++i) {
        if (T->arr[i].fd >= 0) close(T->arr[i].fd);
        const std::string path = T->dir + "/array_" + std::to_string(i) + ".bin";
        (void)unlink(path.c_str());
    }
    if (T->pool) (void)hipHostFree(T->pool);
    delete T;
    c->tier = nullptr;
}

gnn_status tier_open(gnn_ctx* c, const char* dir, int64_t host_budget_bytes)
{
    tier_close(c);
    const int32_t L = c->L;
    StorageTier* T = new (std::nothrow) StorageTier();
    if (!T) return c->fail(GNN_ENOMEM, "out of host memory");
    c->tier = T;
    T->dir = dir;
    T->arr.resize((size_t)2 * L + 1);
    for (size_t i = 0; i < T->arr.size(); ++i) T->arr[i].bytes = (tier_array_bytes(c, (int)i) + 4095) / 4096 * 4096;
    if (host_budget_bytes < 4096) {
        tier_close(c);
        return c->fail(GNN_EINVAL, "gnn_storage_open: host_budget_bytes must be at least 4096");
    }
    T->pool_bytes = host_budget_bytes / 4096 * 4096;
    hipError_t e = hipHostMalloc((void**)&T->pool, (size_t)T->pool_bytes, hipHostMallocDefault);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        T->pool = nullptr;
        tier_close(c);
        return c->fail(GNN_ENOMEM, std::string("gnn_storage_open: hipHostMalloc: ") + hipGetErrorString(e));
    }
    T->free_list.assign(1, {0, T->pool_bytes});
    for (size_t i = 0; i < T->arr.size(); ++i) {
        const std::string path = T->dir + "/array_" + std::to_string(i) + ".bin";
        T->arr[i].fd = open(path.c_str(), O_RDWR | O_CREAT | O_TRUNC, 0600);
        if (T->arr[i].fd < 0) {
            const std::string msg = "gnn_storage_open: " + path + ": " + std::strerror(errno);
            tier_close(c);
            return c->fail(GNN_EINVAL, msg);
        }
        // full size from the start: blocks are read and written at their offsets
        if (ftruncate(T->arr[i].fd, (off_t)T->arr[i].bytes) != 0) {
            const std::string msg = "gnn_storage_open: " + path + ": " + std::strerror(errno);
            tier_close(c);
            return c->fail(GNN_ENOMEM, msg);
        }
    }
    T->worker = std::thread(worker_main, T);
    return GNN_OK;
}

// Points the context's per-layer host pointers at wherever the arrays are now (null: on storage).
static void publish(gnn_ctx* c)
{
    StorageTier& T = *c->tier;
    const int32_t L = c->L;
    auto at = [&](int id) -> char* {
        const TierArray& a = T.arr[(size_t)id];
        if (a.off >= 0) return T.pool + a.off;
        return a.bypass ? tier_virtual_base(id) : nullptr;
    };
    c->feat = at(0);
    for (int32_t l = 1; l <= L; ++l) {
        c->act[(size_t)l - 1] = at(l);
        c->gact[(size_t)l - 1] = (float*)at(L + l);
    }
}

void tier_keep_results(gnn_ctx* c, bool keep)
{
    std::lock_guard<std::mutex> lk(c->tier->mu);
    c->tier->keep_results = keep;
}

// A new epoch overwrites every array but the features before it reads them: what the last epoch
// left in them need not be written anywhere.
void tier_epoch_begin(gnn_ctx* c)
{
    StorageTier& T = *c->tier;
    std::unique_lock<std::mutex> lk(T.mu);
    T.wanted.clear();
    T.cv.wait(lk, [&] { return !T.working; });
    for (size_t i = 1; i < T.arr.size(); ++i) {
        T.arr[i].dirty = false;
        T.arr[i].on_disk = false;
        T.arr[i].dead = true;
    }
}

// Whether tier_prepare for these arrays would read, evict or move anything (then the device must
// be idle first); stops the helper thread's read-ahead as a side effect.
bool tier_needs_io(gnn_ctx* c, const int* need, int nneed)
{
    StorageTier& T = *c->tier;
    std::unique_lock<std::mutex> lk(T.mu);
    T.wanted.clear();
    T.cv.wait(lk, [&] { return !T.working; });
    for (int i = 0; i < nneed; ++i)
        if (T.arr[(size_t)need[i]].off < 0) return true;
    return false;
}

gnn_status tier_prepare(gnn_ctx* c, const int* need, int nneed, unsigned overwrite_mask, const int* next, int nnext,
                        const int* dead, int ndead, bool device_idle)
{
    StorageTier& T = *c->tier;
    std::unique_lock<std::mutex> lk(T.mu);
    T.wanted.clear();
    T.cv.wait(lk, [&] { return !T.working; });
    T.device_idle_at_phase_start = device_idle;
    if (!T.worker_error.empty()) {
        const std::string msg = "storage tier: " + T.worker_error;
        T.worker_error.clear();
        return c->fail(GNN_EHIP, msg);
    }
    std::vector<int> keep(need, need + nneed);
    std::string err;
    for (TierArray& a : T.arr) a.bypass = false;
    for (int i = 0; i < nneed; ++i) {
        const int id = need[i];
        TierArray& a = T.arr[(size_t)id];
        const bool overwrite = (overwrite_mask >> i) & 1u;
        if (a.off < 0) {
            if (!device_idle) return c->fail(GNN_ESTATE, "storage tier: an array has to be brought in while the device may be busy");
            if (!make_room(T, id, keep, false, err)) {
                // no room beside the arrays named before it: the phase works on its file, block by block
                a.bypass = true;
                ++T.stats.bypassed;
                if (overwrite) a.on_disk = true;       // every block is written during the phase
                a.dead = false;
                a.last_use = ++T.tick;
                continue;
            }
            if (!overwrite) {
                if (!a.on_disk) {
                    // never written: the schedule reads an array only after a phase produced it
                    std::memset(T.pool + a.off, 0, (size_t)a.bytes);
                } else {
                    if (!read_all(a.fd, T.pool + a.off, a.bytes, err)) return c->fail(GNN_EHIP, "storage tier: " + err);
                    T.stats.bytes_read += a.bytes;
                    ++T.stats.loads;
                }
            }
        } else {
            ++T.stats.hits;
        }
        if (overwrite) {
            a.dirty = true;
            a.on_disk = false;
        }
        a.dead = false;
        a.last_use = ++T.tick;
    }
    // (takes effect when the next phase asks for room: by then this phase has run)
    for (int i = 0; i < ndead; ++i) T.arr[(size_t)dead[i]].dead = true;
    T.cur_need = keep;
    publish(c);
    // the helper thread brings in what the next phase reads, in free room only
    for (int i = nnext - 1; i >= 0; --i)
        if (T.arr[(size_t)next[i]].off < 0 && T.arr[(size_t)next[i]].on_disk) T.wanted.push_back(next[i]);
    if (!T.wanted.empty()) T.cv.notify_all();
    return GNN_OK;
}

// Whole-array transfers between the caller and the tier (library order).
gnn_status tier_write(gnn_ctx* c, int id, const void* src)
{
    StorageTier& T = *c->tier;
    std::unique_lock<std::mutex> lk(T.mu);
    T.wanted.clear();
    T.cv.wait(lk, [&] { return !T.working; });
    TierArray& a = T.arr[(size_t)id];
    const int64_t bytes = tier_array_bytes(c, id);
    std::string err;
    if (a.off >= 0) {
        std::memcpy(T.pool + a.off, src, (size_t)bytes);
        a.dirty = true;
        a.on_disk = false;
        return GNN_OK;
    }
    // straight to its file: it takes no room until a phase needs it
    if (!write_all(a.fd, (const char*)src, bytes, err)) return c->fail(GNN_EHIP, "storage tier: " + err);
    a.on_disk = true;
    a.dirty = false;
    T.stats.bytes_written += bytes;
    return GNN_OK;
}

gnn_status tier_read(gnn_ctx* c, int id, void* dst)
{
    StorageTier& T = *c->tier;
    std::unique_lock<std::mutex> lk(T.mu);
    T.wanted.clear();
    T.cv.wait(lk, [&] { return !T.working; });
    TierArray& a = T.arr[(size_t)id];
    const int64_t bytes = tier_array_bytes(c, id);
    std::string err;
    if (a.off >= 0) {
        std::memcpy(dst, T.pool + a.off, (size_t)bytes);
        return GNN_OK;
    }
    if (!a.on_disk) {
        std::memset(dst, 0, (size_t)bytes);
        return GNN_OK;
    }
    if (!read_all(a.fd, (char*)dst, bytes, err)) return c->fail(GNN_EHIP, "storage tier: " + err);
    T.stats.bytes_read += bytes;
    return GNN_OK;
}

// Arrays that a phase uses without having them in the pool are handed to the schedule as
// addresses in a range no allocation can lie in: 2^62 + id * 2^48 + byte offset.  The schedule
// does its usual pointer arithmetic on them and the two copy routines below recognise them.
char* tier_virtual_base(int id) { return reinterpret_cast<char*>((uintptr_t)1 << 62) + ((uintptr_t)id << 48); }

bool tier_decode(const void* p, int* id, int64_t* off)
{
    const uintptr_t v = reinterpret_cast<uintptr_t>(p);
    if (!(v >> 62)) return false;
    *id = (int)((v >> 48) & 0x3FFF);
    *off = (int64_t)(v & (((uintptr_t)1 << 48) - 1));
    return true;
}

gnn_status tier_file_read(gnn_ctx* c, int id, int64_t off, void* dst, int64_t bytes)
{
    StorageTier& T = *c->tier;
    TierArray& a = T.arr[(size_t)id];
    for (int64_t done = 0; done < bytes;) {
        const ssize_t r = pread(a.fd, (char*)dst + done, (size_t)std::min(kChunk, bytes - done), (off_t)(off + done));
        if (r < 0 && errno == EINTR) continue;
        if (r <= 0) return c->fail(GNN_EHIP, std::string("storage tier: pread: ") + (r < 0 ? std::strerror(errno) : "short file"));
        done += r;
    }
    std::lock_guard<std::mutex> lk(T.mu);
    T.stats.bytes_read += bytes;
    T.stats.bypass_bytes += bytes;
    return GNN_OK;
}

gnn_status tier_file_write(gnn_ctx* c, int id, int64_t off, const void* src, int64_t bytes)
{
    StorageTier& T = *c->tier;
    TierArray& a = T.arr[(size_t)id];
    for (int64_t done = 0; done < bytes;) {
        const ssize_t w = pwrite(a.fd, (const char*)src + done, (size_t)std::min(kChunk, bytes - done), (off_t)(off + done));
        if (w < 0 && errno == EINTR) continue;
        if (w < 0) return c->fail(GNN_EHIP, std::string("storage tier: pwrite: ") + std::strerror(errno));
        done += w;
    }
    std::lock_guard<std::mutex> lk(T.mu);
    T.stats.bytes_written += bytes;
    T.stats.bypass_bytes += bytes;
    return GNN_OK;
}

void tier_get_stats(const gnn_ctx* c, gnn_storage_stats* out)
{
    StorageTier& T = *c->tier;
    std::lock_guard<std::mutex> lk(T.mu);
    *out = T.stats;
    out->host_pool_bytes = T.pool_bytes;
    int64_t total = 0;
    for (const TierArray& a : T.arr) total += a.bytes;
    out->array_bytes = total;
}

}  // namespace gnnmi
