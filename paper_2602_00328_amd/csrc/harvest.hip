// Host side of libharvest.so: the C ABI of include/harvest.h over the kernels in kernels.h.
//
// Structure
//   ClassState  - per object class: host mirror of the directory, slot allocators, device directory.
//   StreamState - per caller stream: device scratch (HBM list, host list, miss list, counters), a side stream for
//                 the host-tier gather, fork/join events and the "last operation" event the revocation drain waits on.
//   Staging     - pinned host blocks through which host-built lists reach the device without blocking the caller.
//   edit chain  - every directory edit is a dir_write kernel that waits for the edit before it, on whatever stream that
//                 ran, so edits reach the device in the order the host made them (paper Section 3.2: revocation is
//                 ordered).  Placements and write-backs edit on the caller's stream, right behind their copy;
//                 register, restore and revoke, which have no caller stream, edit on the library's control stream.
//                 Each class has a chain of its own.
//   drain       - a revocation waits for the other streams' work on the host (it blocks anyway); no library stream is ever
//                 parked behind a caller's stream.  The poisoning that follows runs on a stream of its own.
#include "../../include/harvest.h"
#include "kernels.h"
#include <hip/hip_ext.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <deque>
#include <list>
#include <map>
#include <memory>
#include <mutex>
#include <set>
#include <unordered_set>
#include <vector>

using namespace hv;

#define HIP_TRY(expr)                                                                                   \
    do {                                                                                                \
        hipError_t e_ = (expr);                                                                         \
        if (e_ != hipSuccess) {                                                                         \
            fprintf(stderr, "libharvest: %s failed: %s (%s:%d)\n", #expr, hipGetErrorString(e_), __FILE__, \
                    __LINE__);                                                                          \
            return HARVEST_EHIP;                                                                        \
        }                                                                                               \
    } while (0)

// Failure injection for the CPU tests of the error paths (built only with -DHARVEST_FAULT_INJECTION, never into the
// product library): harvest_test_fail_at(n) makes the n-th device step from now fail as a HIP error would.  "Device
// step" = every place in place / evict / revoke where a HIP call can fail; a context without a device walks the same
// steps without making the calls, so the roll-back code runs on a CPU.
#ifdef HARVEST_FAULT_INJECTION
#include <atomic>
static std::atomic<int> g_fail_at{ 0 };
extern "C" void harvest_test_fail_at(int nth) { g_fail_at = nth; }
static inline bool fault_due()
{
    int v = g_fail_at.load();
    if (v <= 0) return false;
    g_fail_at = v - 1;
    return v == 1;
}
#else
static inline constexpr bool fault_due() { return false; }
#endif

// A device step of a call that has a roll-back: fails when the injected fault is due, is skipped without a device.
#define DEV_TRY(expr)                                  \
    do {                                               \
        if (fault_due()) return HARVEST_EHIP;          \
        if (!ctx->no_device) HIP_TRY(expr);            \
    } while (0)

namespace {

// Free space of the shared cache pool, in granules: maximal free runs, indexed by offset (to merge neighbours on free)
// and by (length, offset) (to find the best fit: the shortest run that is long enough, the lowest of equals).
struct SegAlloc {
    std::map<uint64_t, uint64_t> by_off;                  // offset -> length
    std::set<std::pair<uint64_t, uint64_t>> by_len;       // (length, offset)
    uint64_t n_free = 0;

    void add(uint64_t off, uint64_t len) { by_off[off] = len; by_len.insert({ len, off }); }
    void drop(uint64_t off, uint64_t len) { by_off.erase(off); by_len.erase({ len, off }); }
    void reset(uint64_t n_granules)
    {
        by_off.clear(); by_len.clear();
        n_free = n_granules;
        if (n_granules) add(0, n_granules);
    }
    int64_t take(uint64_t need)
    {
        if (!need) return -1;
        auto it = by_len.lower_bound({ need, 0 });
        if (it == by_len.end()) return -1;
        uint64_t len = it->first, off = it->second;
        drop(off, len);
        if (len > need) add(off + need, len - need);       // the segment sits at the low end of the run
        n_free -= need;
        return (int64_t)off;
    }
    void give(uint64_t off, uint64_t len)
    {
        n_free += len;
        auto next = by_off.lower_bound(off);
        if (next != by_off.begin()) {
            auto prev = std::prev(next);
            if (prev->first + prev->second == off) {
                off = prev->first; len += prev->second;
                uint64_t po = prev->first, pl = prev->second;
                drop(po, pl);
            }
        }
        next = by_off.lower_bound(off + 1);
        if (next != by_off.end() && next->first == off + len) {
            uint64_t no = next->first, nl = next->second;
            len += nl;
            drop(no, nl);
        }
        add(off, len);
    }
};

struct ClassState {
    harvest_class_config cfg{};
    bool used = false;
    uint64_t host_dev[2] = { 0, 0 };        // device-visible address of the pinned host pool planes
    uint32_t n_objects = 0;
    std::vector<uint8_t> tier;              // mirror of the directory
    std::vector<int64_t> slot;              // cache / local slot or -1
    std::vector<uint32_t> gen;
    std::vector<int64_t> host_slot;         // -1 = lossy
    std::vector<harvest_revoke_cb> cb;
    std::vector<void *> cb_user;
    std::vector<uint8_t> host_used;
    std::set<uint32_t> cache_free, local_free;   // begin() = lowest free slot
    // cache tier carved from the context's shared pool instead of equal-size slots: an object owns obj_granules
    // granules from granule number `slot` on, laid out [layer][plane][chunk]
    SegAlloc *seg = nullptr;
    uint64_t seg_base = 0, granule = 0, obj_granules = 0, n_granules = 0;
    uint64_t cache_in_use = 0;
    bool adjacent = false;                  // equal-size cache slots laid out [layer][slot][plane][chunk] in one buffer
    uint64_t *d_dir = nullptr;
    // The edits of this class's directory form one chain on the device, in the order the host made them: every edit is a
    // dir_write kernel on some stream (the caller's for place / evict, the control stream for register / restore /
    // revoke) that first waits for edit_evt - the class's previous edit - unless that ran on the same stream, and then
    // records edit_evt itself.  A chain per class: a KV fetch has no reason to wait for an expert's placement.
    hipEvent_t edit_evt = nullptr;
    hipStream_t edit_stream = nullptr;      // where the latest edit was enqueued
    uint64_t edit_seq = 0;                  // number of edits enqueued so far
    uint64_t must_seq = 0;                  // edit_seq after the latest edit that every later fetch has to see (register,
                                            // restore, revoke, demotion); a placement is not one: until it is seen, the
                                            // older entry names the host copy, which holds the same bytes
    // duplicate detection within one call without hashing: an object is marked with the number of the call
    std::vector<uint32_t> stamp;
    uint32_t epoch = 0;

    void new_call()
    {
        if (++epoch == 0) { std::fill(stamp.begin(), stamp.end(), 0u); epoch = 1; }
        if (stamp.size() < n_objects) stamp.resize(n_objects, 0u);
    }
    bool first_time(uint32_t id)               // false: this call has named the object before
    {
        if (stamp[id] == epoch) return false;
        stamp[id] = epoch;
        return true;
    }

    // host-side statistics
    uint64_t n_placed = 0, n_enospc = 0, n_revoked = 0, n_evicted = 0, n_demoted = 0;

    uint64_t packed(uint32_t id) const
    {
        uint32_t t = tier[id];
        uint32_t s = t == T_HOST ? (uint32_t)host_slot[id] : (t == T_NONE ? 0u : (uint32_t)slot[id]);
        return make_entry(t, s, gen[id]);
    }
    // Room in the cache tier for one object: the lowest free slot, or a best-fit segment.  -1: none.
    int64_t cache_take()
    {
        int64_t s = -1;
        if (seg) s = seg->take(obj_granules);
        else if (!cache_free.empty()) {
            s = *cache_free.begin();
            cache_free.erase(cache_free.begin());
        }
        if (s >= 0) cache_in_use++;
        return s;
    }
    void cache_release(int64_t s)
    {
        if (seg) seg->give((uint64_t)s, obj_granules);
        else cache_free.insert((uint32_t)s);
        cache_in_use--;
    }
    uint64_t cache_base(uint32_t plane) const
    {
        if (seg) return seg_base + plane * cfg.chunk_bytes;
        return adjacent ? (uint64_t)cfg.d_cache_pool[0] + plane * cfg.chunk_bytes : (uint64_t)cfg.d_cache_pool[plane];
    }
    // the planes of an object's chunk are neighbours in the cache tier: one source run per request instead of two
    bool cache_planes_adjacent() const { return cfg.n_planes == 2 && (seg || adjacent); }
    uint64_t addr(int t, uint32_t plane, uint32_t layer, uint64_t s) const
    {
        if (t == T_CACHE && seg) return cache_base(plane) + s * granule + (uint64_t)layer * cfg.n_planes * cfg.chunk_bytes;
        if (t == T_CACHE && adjacent)
            return cache_base(plane) + ((uint64_t)layer * cfg.n_cache_slots + s) * cfg.n_planes * cfg.chunk_bytes;
        uint64_t base = t == T_HOST ? host_dev[plane]
                                    : (t == T_CACHE ? (uint64_t)cfg.d_cache_pool[plane] : (uint64_t)cfg.d_local_pool[plane]);
        uint64_t ns = t == T_HOST ? cfg.n_host_slots : (t == T_CACHE ? cfg.n_cache_slots : cfg.n_local_slots);
        return base + ((uint64_t)layer * ns + s) * cfg.chunk_bytes;
    }
};

// What a call has changed in the host mirror so far, undone in reverse order unless the call commits: the calls that edit
// the directory change the mirror first and the device afterwards, and a device step that fails in between must leave
// no trace ("on error nothing is enqueued or changed").
struct Undo {
    enum Kind : uint8_t { PLACED, REVOKED, DEMOTED, TOOK_CACHE_SLOT, COUNTED_ENOSPC, COUNTED_EVICTED };
    struct Step { Kind kind; uint32_t id; uint32_t gen; int64_t slot; };
    ClassState &c;
    std::vector<Step> steps;
    bool armed = true;
    explicit Undo(ClassState &cls) : c(cls) {}
    void add(Kind k, uint32_t id = 0, int64_t slot = -1, uint32_t gen = 0) { steps.push_back({ k, id, gen, slot }); }
    void commit() { armed = false; }
    ~Undo()
    {
        if (!armed) return;
        for (auto it = steps.rbegin(); it != steps.rend(); ++it) {
            switch (it->kind) {
            case PLACED:               // the object took cache slot `slot`: back to the host entry of generation `gen`
                c.cache_release(it->slot);
                c.tier[it->id] = T_HOST; c.slot[it->id] = -1; c.gen[it->id] = it->gen; c.n_placed--;
                break;
            case REVOKED:              // the object left cache slot `slot`
                c.tier[it->id] = T_CACHE; c.slot[it->id] = it->slot; c.gen[it->id] = it->gen; c.n_revoked--;
                break;
            case DEMOTED:              // the object left local slot `slot`
                c.local_free.erase((uint32_t)it->slot);
                c.tier[it->id] = T_LOCAL; c.slot[it->id] = it->slot; c.gen[it->id] = it->gen; c.n_demoted--;
                break;
            case TOOK_CACHE_SLOT: c.cache_release(it->slot); break;
            case COUNTED_ENOSPC: c.n_enospc--; break;
            case COUNTED_EVICTED: c.n_evicted--; break;
            }
        }
    }
};

struct Staging {
    void *h = nullptr;
    size_t cap = 0;
    hipEvent_t done = nullptr;
    bool busy = false;      // the device may still read it: free again once `done` has passed
    bool held = false;      // a call has taken it and not yet handed it to the device (or given it back)
};

// Gives a staging block back if the call ends before the device got it.
struct Hold {
    Staging *st = nullptr;
    ~Hold() { if (st && st->held) st->held = false; }
};

struct ProfPair { hipEvent_t a, b; int which; };

// What a fetch leaves behind for its gathers and for harvest_fetch_info: the two request lists, the miss list and the
// counters.  Each class has its own set on every stream, so an expert fetch never touches what a KV fetch left (a
// decode step walks its layers with KV and expert fetches in turn, and harvest_fetch_kv_again reads the KV lists
// layers later).
struct Lists {
    Rec *hbm = nullptr, *host = nullptr;
    uint32_t *miss = nullptr;
    uint32_t *cnt = nullptr;                // [C_N] counters of the class's last fetch; every fetch overwrites all of them
    uint32_t cap = 0;                       // requests the three lists have room for
};

// Intermediate arrays of the KV resolve (classify_kv -> scan_groups -> compact_kv), one entry or row per table cell.
struct KvWork {
    Rec *tmp = nullptr;
    uint8_t *kind = nullptr;
    uint32_t *blk_counts = nullptr;
    uint32_t *grp_totals = nullptr, *row_prefix = nullptr;     // large tables: the middle pass of the compaction
};

struct StreamState {
    hipStream_t s = nullptr;
    hipStream_t side = nullptr;
    hipEvent_t fork = nullptr, join = nullptr, last = nullptr;
    bool last_valid = false;
    // fetch scratch
    Lists lists[HARVEST_N_CLASSES];
    KvWork work;
    uint32_t *cnt_block = nullptr;          // the counters of both classes: one allocation
    uint32_t *mark = nullptr;               // [MAX_EXPERTS / 32 + 1] routed-set bitmap and invalid-id count of large batches;
                                            // zero between fetches
    int last_cls = -1;                      // class of the latest fetch enqueued on this stream, -1: none yet
    bool counted[HARVEST_N_CLASSES] = { false, false };   // the class's latest fetch ran kernels, so its counters are its own
                                            // (an empty block table runs none: that fetch reports zeros)
    bool fixed = false;                     // the lists are borrowed, of a fixed size, and there is no side stream: the
                                            // state of a stream that harvest_fetch_kv_static serves
    // the latest single-layer KV fetch, for harvest_fetch_kv_again
    struct {
        bool valid = false, lists = false;  // lists: the general path ran, so the compacted lists describe it
        uint32_t layer = 0, n_seq = 0, max_blocks = 0, n_heads = 0, block_tokens = 0;
        const int32_t *table = nullptr, *n_blocks = nullptr;
        const uint64_t *seq_dst_block = nullptr;
        const uint32_t *seq_cap_blocks = nullptr;
        uint64_t dst_cap = 0, edit_seq = 0;
    } last_kv;
    uint64_t seen_seq[HARVEST_N_CLASSES] = { 0, 0 };   // per class: directory edits this stream has been ordered after
    // control scratch (host-built lists)
    void *ctl_buf = nullptr;
    size_t ctl_cap = 0;
    // pinned words the HBM-tier gather reports its request count to, per class: a hint for the next grid size
    uint32_t *h_feedback = nullptr;
    uint32_t *d_feedback = nullptr;
    bool feedback_valid[HARVEST_N_CLASSES] = { false, false };
};

// ---- fixed scratch of harvest_fetch_kv_static -------------------------------------------------------------------
// Everything a KV fetch of up to HARVEST_STATIC_MAX_CELLS table cells needs beyond its inputs and outputs - the arrays
// of the resolve, the two request lists, the miss list, the counters - in one file-scope device array, so that the
// call allocates nothing.  Each GPU the library runs on holds its own copy, at its own address, until the process
// ends; the address is asked for once per device (scratch_of_device), with that device current, and only that
// address is ever handed to a kernel - the array's name is a host-side stand-in, not a device address.
constexpr uint32_t STATIC_CELLS = HARVEST_STATIC_MAX_CELLS;
constexpr size_t STATIC_ROWS = (STATIC_CELLS + WG - 1) / WG;
constexpr size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
constexpr size_t SO_TMP = 0;
constexpr size_t SO_HBM = SO_TMP + align256((size_t)STATIC_CELLS * sizeof(Rec));
constexpr size_t SO_HOST = SO_HBM + align256((size_t)STATIC_CELLS * sizeof(Rec));
constexpr size_t SO_MISS = SO_HOST + align256((size_t)STATIC_CELLS * sizeof(Rec));
constexpr size_t SO_KIND = SO_MISS + align256((size_t)STATIC_CELLS * sizeof(uint32_t));
constexpr size_t SO_BLK = SO_KIND + align256((size_t)STATIC_CELLS);
constexpr size_t SO_CNT = SO_BLK + align256(STATIC_ROWS * BC_N * sizeof(uint32_t));
constexpr size_t STATIC_BYTES = SO_CNT + align256(C_N * sizeof(uint32_t));
static_assert(STATIC_ROWS <= 1024, "the fixed scratch has no room for the grouped compaction of very large tables");

static __device__ __align__(256) unsigned char scratch[STATIC_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
unsigned char *g_scratch_ptr[MAX_DEVICES];          // per device: where that GPU's copy of `scratch` lives

// The device address of `scratch` on device `dev`, which must be the current device.
int scratch_of_device(int dev, unsigned char **out)
{
    if (dev < 0 || dev >= MAX_DEVICES) return HARVEST_EINVAL;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        unsigned char *ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return HARVEST_EHIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return HARVEST_OK;
}

constexpr int STATIC_STREAMS = 4;                   // caller streams one context serves through harvest_fetch_kv_static

}  // namespace

struct harvest_prefetcher;

struct harvest_ctx {
    harvest_config cfg{};
    bool no_device = false, poison = false, profile = false, general_fetch = false;
    int n_cu = 256;
    uint32_t gather_grid = 0, host_grid = 0, ctl_grid = 0, pcie_grid = 0;
    uint32_t gather_threads = HBM_WG;     // threads per workgroup of the HBM-tier gather (64, 128 or 256)
    uint64_t small_cells = 0;             // block tables up to this many cells are fetched by one kernel
    ClassState cls[HARVEST_N_CLASSES];
    hipStream_t ctl = nullptr;            // directory edits that have no caller stream (register, restore, revoke)
    hipStream_t drain = nullptr;          // the poisoning of revoked slots (hundreds of MiB at times): kept off `ctl`, so that no
                                          // directory edit queues up behind it
    unsigned long long *d_totals = nullptr;  // [HARVEST_N_CLASSES][C_N]
    unsigned long long *d_lease = nullptr;   // until when (device clock) a fetch expects to need the PCIe link: see link_announce
    std::map<hipStream_t, std::unique_ptr<StreamState>> streams;
    std::deque<Staging> staging;          // deque: references stay valid when it grows
    std::vector<ProfPair> prof;
    std::vector<hipEvent_t> prof_pool;
    std::vector<hipEvent_t> evt_pool;     // events (no timing) of finished revocations, for the next ones
    // Latest-work events that revocations have taken out of their streams' states and are waiting for right now, with the
    // number of revocations waiting on each.  A second revocation that starts meanwhile no longer finds those events in
    // the stream states, yet the work they stand for is as much in flight for it: it waits for everything listed here too.
    struct DrainEvt { hipEvent_t e; int refs; };
    std::list<DrainEvt> draining;
    bool captured_work = false;           // a fetch was recorded into a HIP graph: replays are invisible to the events
    SegAlloc shared;                      // free space of cfg.d_shared_cache
    std::vector<harvest_prefetcher *> prefetchers;   // live ones: destroyed with the context if the caller did not
    // harvest_fetch_kv_static: stream states made when the context is created (events, a pinned feedback word each), their
    // lists inside the device's fixed scratch; a caller stream takes the first unused one
    StreamState fixed_streams[STATIC_STREAMS];
    int n_fixed_streams = 0;                         // how many have a caller stream
    std::mutex mu;
};

struct harvest_prefetcher {
    harvest_ctx *ctx = nullptr;
    hipStream_t fetch = nullptr;                 // library-owned, default priority
    void *staging[2] = { nullptr, nullptr };
    void **ptrs[2] = { nullptr, nullptr };
    uint32_t n_slots = 0;
    hipEvent_t ready[2] = { nullptr, nullptr };  // the fetch into buffer b has finished
    hipEvent_t freed[2] = { nullptr, nullptr };  // the consumer of buffer b has finished
    hipEvent_t dep = nullptr;                    // the routing ids of the next fetch exist
    bool freed_valid[2] = { false, false };
    uint64_t n_issued = 0, n_acquired = 0, n_released = 0;
};

namespace {

int device_guard(harvest_ctx *ctx)
{
    if (ctx->no_device) return HARVEST_OK;
    HIP_TRY(hipSetDevice(ctx->cfg.device));
    return HARVEST_OK;
}

bool is_capturing(hipStream_t s)
{
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &st) != hipSuccess) return false;
    return st != hipStreamCaptureStatusNone;
}

// Releases what a caller stream's state owns (any part of it may be missing); the stream's work must have finished.
void free_stream_state(StreamState *ss)
{
    if (ss->side) (void)hipStreamDestroy(ss->side);
    for (hipEvent_t e : { ss->fork, ss->join, ss->last }) if (e) (void)hipEventDestroy(e);
    if (ss->fixed) {
        if (ss->h_feedback) (void)hipHostFree(ss->h_feedback);
        return;
    }
    for (Lists &l : ss->lists) { (void)hipFree(l.hbm); (void)hipFree(l.host); (void)hipFree(l.miss); }
    (void)hipFree(ss->work.tmp); (void)hipFree(ss->work.kind); (void)hipFree(ss->work.blk_counts);
    (void)hipFree(ss->work.grp_totals); (void)hipFree(ss->work.row_prefix);
    (void)hipFree(ss->cnt_block); (void)hipFree(ss->mark);
    (void)hipFree(ss->ctl_buf);
    if (ss->h_feedback) (void)hipHostFree(ss->h_feedback);
}

int init_stream_state(StreamState *ss)
{
    HIP_TRY(hipStreamCreateWithFlags(&ss->side, hipStreamNonBlocking));
    for (hipEvent_t *e : { &ss->fork, &ss->join, &ss->last })
        HIP_TRY(hipEventCreateWithFlags(e, hipEventDisableTiming));
    HIP_TRY(hipMalloc(&ss->cnt_block, HARVEST_N_CLASSES * C_N * sizeof(uint32_t)));
    HIP_TRY(hipMemset(ss->cnt_block, 0, HARVEST_N_CLASSES * C_N * sizeof(uint32_t)));
    for (int k = 0; k < HARVEST_N_CLASSES; ++k) ss->lists[k].cnt = ss->cnt_block + k * C_N;
    HIP_TRY(hipMalloc(&ss->mark, (MAX_EXPERTS / 32 + 1) * sizeof(uint32_t)));
    HIP_TRY(hipMemset(ss->mark, 0, (MAX_EXPERTS / 32 + 1) * sizeof(uint32_t)));
    HIP_TRY(hipHostMalloc((void **)&ss->h_feedback, 64, hipHostMallocDefault));
    memset(ss->h_feedback, 0, 64);
    HIP_TRY(hipHostGetDevicePointer((void **)&ss->d_feedback, ss->h_feedback, 0));
    return HARVEST_OK;
}

int get_stream(harvest_ctx *ctx, void *stream, StreamState **out)
{
    hipStream_t s = (hipStream_t)stream;
    auto it = ctx->streams.find(s);
    if (it != ctx->streams.end()) { *out = it->second.get(); return HARVEST_OK; }
    if (is_capturing(s)) {
        fprintf(stderr, "libharvest: first use of a stream allocates its scratch - call once outside graph capture\n");
        return HARVEST_EINVAL;
    }
    auto ss = std::make_unique<StreamState>();
    ss->s = s;
    if (int rc = init_stream_state(ss.get())) {
        free_stream_state(ss.get());
        return rc;
    }
    *out = ss.get();
    ctx->streams[s] = std::move(ss);
    return HARVEST_OK;
}

// Room for n_req requests in the lists of class cls (and, for KV, in the arrays of the resolve).  Growing (not the
// first allocation) waits for the stream's earlier work, which may still read the old arrays; the new ones are all
// there before the old ones go, so a failed allocation leaves the stream as it was.
int ensure_req_cap(StreamState *ss, int cls, uint32_t n_req)
{
    Lists &l = ss->lists[cls];
    if (n_req <= l.cap) return HARVEST_OK;
    if (ss->fixed) {
        fprintf(stderr, "libharvest: a fetch of %u requests does not fit the fixed scratch (%u)\n", n_req, l.cap);
        return HARVEST_E2BIG;
    }
    if (is_capturing(ss->s)) {
        fprintf(stderr, "libharvest: this fetch needs larger scratch lists - run it once outside graph capture\n");
        return HARVEST_EINVAL;
    }
    if (l.cap) {                              // the stream's earlier work may still read the arrays that are about to go
        HIP_TRY(hipStreamSynchronize(ss->s));
        HIP_TRY(hipStreamSynchronize(ss->side));
    }
    uint32_t cap = std::max<uint32_t>(1024, n_req + n_req / 4);
    size_t n_rows = (cap + WG - 1) / WG;
    const bool kv = cls == HARVEST_KV;
    void *fresh[8] = { nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr };
    const size_t bytes[8] = { (size_t)cap * sizeof(Rec), (size_t)cap * sizeof(Rec), (size_t)cap * sizeof(uint32_t),
                              kv ? (size_t)cap * sizeof(Rec) : 0, kv ? (size_t)cap : 0,
                              kv ? n_rows * BC_N * sizeof(uint32_t) : 0,
                              kv ? ((n_rows + WG - 1) / WG) * BC_N * sizeof(uint32_t) : 0,
                              kv ? n_rows * 3 * sizeof(uint32_t) : 0 };
    for (int i = 0; i < 8; ++i) {
        if (!bytes[i]) continue;
        hipError_t e = hipMalloc(&fresh[i], bytes[i]);
        if (e != hipSuccess) {
            fprintf(stderr, "libharvest: hipMalloc(%zu) failed: %s\n", bytes[i], hipGetErrorString(e));
            for (int j = 0; j < i; ++j) (void)hipFree(fresh[j]);
            return HARVEST_EHIP;
        }
    }
    (void)hipFree(l.hbm); (void)hipFree(l.host); (void)hipFree(l.miss);
    l.hbm = (Rec *)fresh[0]; l.host = (Rec *)fresh[1]; l.miss = (uint32_t *)fresh[2];
    if (kv) {
        KvWork &w = ss->work;
        (void)hipFree(w.tmp); (void)hipFree(w.kind); (void)hipFree(w.blk_counts); (void)hipFree(w.grp_totals);
        (void)hipFree(w.row_prefix);
        w.tmp = (Rec *)fresh[3]; w.kind = (uint8_t *)fresh[4]; w.blk_counts = (uint32_t *)fresh[5];
        w.grp_totals = (uint32_t *)fresh[6]; w.row_prefix = (uint32_t *)fresh[7];
        ss->last_kv.valid = false;              // the lists that fetch left are gone
    }
    l.cap = cap;
    return HARVEST_OK;
}

int ensure_ctl_cap(harvest_ctx *ctx, StreamState *ss, size_t bytes)
{
    if (fault_due()) return HARVEST_EHIP;
    if (ctx->no_device || bytes <= ss->ctl_cap) return HARVEST_OK;
    if (ss->ctl_buf) {                        // the stream's earlier work may still read the list that is about to go
        HIP_TRY(hipStreamSynchronize(ss->s));
        HIP_TRY(hipFree(ss->ctl_buf));
    }
    ss->ctl_buf = nullptr; ss->ctl_cap = 0;
    size_t cap = std::max<size_t>(1 << 16, bytes + bytes / 4);
    HIP_TRY(hipMalloc(&ss->ctl_buf, cap));
    ss->ctl_cap = cap;
    return HARVEST_OK;
}

// A pinned block nobody on the device still reads.
int acquire_staging(harvest_ctx *ctx, size_t bytes, Staging **out)
{
    *out = nullptr;
    if (fault_due()) return HARVEST_EHIP;
    if (ctx->no_device) return HARVEST_OK;
    for (auto &st : ctx->staging) {
        if (st.cap < bytes || st.held) continue;
        if (st.busy) {
            hipError_t q = hipEventQuery(st.done);
            if (q == hipErrorNotReady) continue;
            if (q != hipSuccess) return HARVEST_EHIP;
            st.busy = false;
        }
        st.held = true;
        *out = &st;
        return HARVEST_OK;
    }
    Staging st;
    st.cap = std::max<size_t>(1 << 16, bytes);
    HIP_TRY(hipHostMalloc(&st.h, st.cap, hipHostMallocDefault));
    if (hipEventCreateWithFlags(&st.done, hipEventDisableTiming) != hipSuccess) {
        (void)hipHostFree(st.h);
        return HARVEST_EHIP;
    }
    st.held = true;
    ctx->staging.push_back(st);
    *out = &ctx->staging.back();
    return HARVEST_OK;
}

// The device reads the block in work enqueued on `s` so far: it is free again when that work has passed.
int release_after(harvest_ctx *ctx, Staging *st, hipStream_t s)
{
    if (fault_due()) return HARVEST_EHIP;
    if (ctx->no_device || !st) return HARVEST_OK;
    HIP_TRY(hipEventRecord(st->done, s));
    st->busy = true;
    st->held = false;
    return HARVEST_OK;
}

constexpr uint64_t SMALL_FETCH_CELLS = 4096;      // block tables up to this many cells are fetched by one kernel (measured:
                                                  // it wins up to 4 096 cells and loses from 8 192 on)
constexpr uint64_t SMALL_FETCH_TILES = 1u << 22;      // and never more workgroups than this in x
constexpr uint32_t MARKED_BATCH_IDS = 32768;      // routing-id batches beyond this take the two-kernel resolve
constexpr uint32_t GROUPED_SCAN_ROWS = 1024;      // block tables of more than 262 144 cells take the three-kernel compaction

uint32_t tiles_per_chunk(uint64_t chunk_bytes, uint32_t tile) { return (uint32_t)((chunk_bytes + tile - 1) / tile); }

// one workgroup per tile up to here; beyond, the kernels loop.  Kept below 2^32 threads per launch dimension.
constexpr uint32_t MAX_GRID = 0xFFFFFFFFu / WG;

uint32_t grid_for(uint64_t n_tiles, uint32_t max_grid)
{
    return (uint32_t)std::max<uint64_t>(1, std::min<uint64_t>(n_tiles, max_grid));
}

ClassDev class_dev(const ClassState &c)
{
    ClassDev d{};
    d.dir = c.d_dir;
    d.n_objects = c.n_objects;
    d.n_planes = c.cfg.n_planes;
    d.chunk_bytes = c.cfg.chunk_bytes;
    for (uint32_t p = 0; p < 2; ++p) {
        d.pool[T_HOST][p] = c.host_dev[p];
        d.pool[T_CACHE][p] = c.cache_base(p);
        d.pool[T_LOCAL][p] = (uint64_t)c.cfg.d_local_pool[p];
    }
    d.n_slots[T_HOST] = c.cfg.n_host_slots;
    d.n_slots[T_CACHE] = c.seg ? (uint32_t)c.n_granules : c.cfg.n_cache_slots;
    d.n_slots[T_LOCAL] = c.cfg.n_local_slots;
    for (int t = 0; t < 3; ++t) {
        d.slot_stride[t] = c.cfg.chunk_bytes;
        d.layer_stride[t] = (uint64_t)d.n_slots[t] * c.cfg.chunk_bytes;
    }
    if (c.seg) {
        d.slot_stride[T_CACHE] = c.granule;
        d.layer_stride[T_CACHE] = (uint64_t)c.cfg.n_planes * c.cfg.chunk_bytes;
    } else if (c.adjacent) {
        d.slot_stride[T_CACHE] = (uint64_t)c.cfg.n_planes * c.cfg.chunk_bytes;
        d.layer_stride[T_CACHE] = (uint64_t)c.cfg.n_cache_slots * c.cfg.n_planes * c.cfg.chunk_bytes;
    }
    return d;
}

// Publishes the mirror entries of `ids` to the device directory with a dir_write kernel on stream `on`, ordered after
// everything enqueued on `on` so far (for a placement: the copy that makes the new entry true) and after every earlier
// directory edit, wherever that ran.  pre: a staging block of n * 12 bytes taken earlier, so that this step cannot fail
// for want of one.  *committed (if given) says whether the dir_write was enqueued: from then on the device will apply
// the edit, and a failure reported by a later step no longer entitles the caller to roll its mirror back.
int publish(harvest_ctx *ctx, ClassState &c, const std::vector<uint32_t> &ids, hipStream_t on, bool must_see,
            Staging *pre = nullptr, bool *committed = nullptr)
{
    if (committed) *committed = ids.empty();
    if (ids.empty()) return HARVEST_OK;
    size_t n = ids.size();
    size_t bytes = n * (sizeof(uint64_t) + sizeof(uint32_t));
    Hold hold;
    Staging *st = pre;
    if (!st) {
        int rc = acquire_staging(ctx, bytes, &st);
        if (rc) return rc;
        hold.st = st;
    }
    // An edit that has no caller stream (register, restore, revoke: on == the control stream) whose predecessor is still
    // queued on a caller's stream goes onto that stream, right behind it, instead of making the control stream wait: a
    // wait parked on a library stream occupies one of the device's few hardware queues for as long as the awaited work
    // takes (a placement of some hundred MiB: milliseconds), and a caller stream that HIP happens to map to the same
    // queue stands still meanwhile.  (Not onto a stream that is being recorded into a graph: then the control stream waits.)
    if (on == ctx->ctl && c.edit_seq && c.edit_stream != ctx->ctl && !ctx->no_device && !is_capturing(c.edit_stream)) {
        hipError_t q = hipEventQuery(c.edit_evt);
        if (q == hipErrorNotReady) on = c.edit_stream;
        else if (q != hipSuccess) HIP_TRY(q);
    }
    if (c.edit_seq && c.edit_stream != on) DEV_TRY(hipStreamWaitEvent(on, c.edit_evt, 0));
    void *d_st = nullptr;
    DEV_TRY(hipHostGetDevicePointer(&d_st, st->h, 0));
    if (!ctx->no_device) {
        uint64_t *ent = (uint64_t *)st->h;
        uint32_t *idv = (uint32_t *)(ent + n);
        for (size_t i = 0; i < n; ++i) { ent[i] = c.packed(ids[i]); idv[i] = ids[i]; }
        uint64_t *d_ent = (uint64_t *)d_st;
        uint32_t *d_ids = (uint32_t *)(d_ent + n);
        hipLaunchKernelGGL(dir_write, dim3((uint32_t)((n + WG - 1) / WG)), dim3(WG), 0, on, c.d_dir, d_ids, d_ent,
                           (uint32_t)n);
    }
    DEV_TRY(hipGetLastError());
    if (committed) *committed = true;
    c.edit_seq++;
    c.edit_stream = on;
    if (must_see) c.must_seq = c.edit_seq;
    if (ctx->no_device) return HARVEST_OK;
    HIP_TRY(hipEventRecord(c.edit_evt, on));
    return release_after(ctx, st, on);
}

// Orders the caller's stream after the edits of the class's directory that a fetch enqueued now has to see - every
// registration, restore, revocation and demotion made so far - without the host ever waiting.  Placements alone are
// not waited for: a fetch is on the critical path and a placement is best effort (it may sit behind hundreds of MiB of
// copies on another stream), and until its entry is seen the older one names the host copy, which holds the same bytes.
// Nothing to do either when the latest edit ran on this very stream: the chain put every earlier one before it.
int order_after_directory_edits(harvest_ctx *ctx, StreamState *ss, int cls)
{
    const ClassState &c = ctx->cls[cls];
    if (ss->seen_seq[cls] >= c.must_seq || is_capturing(ss->s)) return HARVEST_OK;
    if (c.edit_stream != ss->s) HIP_TRY(hipStreamWaitEvent(ss->s, c.edit_evt, 0));
    ss->seen_seq[cls] = c.edit_seq;
    return HARVEST_OK;
}

// Remembers the end of this call's work on the stream for the revocation drain.  Work recorded into a HIP graph runs
// whenever the caller replays the graph, which no event of ours can see: the drain then waits for the whole device.
int mark_last(harvest_ctx *ctx, StreamState *ss)
{
    if (is_capturing(ss->s)) {
        ctx->captured_work = true;
        return HARVEST_OK;
    }
    HIP_TRY(hipEventRecord(ss->last, ss->s));
    ss->last_valid = true;
    return HARVEST_OK;
}

hipEvent_t prof_event(harvest_ctx *ctx)
{
    if (!ctx->prof_pool.empty()) { hipEvent_t e = ctx->prof_pool.back(); ctx->prof_pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

// Launches the HBM-tier gather on the caller's stream and the host-tier gather on the side stream, joined back.
// max_req bounds the number of requests either list can hold; dst_base: where plane p of the working layout starts.
// n_rep > 1 gathers n_rep consecutive layers from the same two lists (they name slots, and an object has the same slot
// in every layer): repetition r reads layer_stride(tier) * r further into every pool and writes dst_step * r further
// into the destination.  The host-tier gathers of all repetitions queue up behind each other on one stream, so
// the link never waits for a join between layers.
int launch_gathers(harvest_ctx *ctx, StreamState *ss, ClassState &c, int cls, const Lists &lists, uint64_t max_req,
                   uint64_t dst_base0, uint64_t dst_base1, const HmArgs *hm = nullptr, uint32_t n_rep = 1,
                   uint64_t dst_step = 0, int64_t layer_delta = 0, bool repeat = false)
{
    // layer_delta: the lists were made for another layer; an object has the same slot in every layer, so adding that many
    // layer strides to every pool base retargets them.  repeat: these requests have been counted for the lists' first
    // use only - add them to the running totals again.
    const ClassDev cd = class_dev(c);
    GatherArgs ga{};
    ga.chunk_bytes = c.cfg.chunk_bytes;
    // the head-major gather and the host tier walk 4 KiB tiles, the token-major HBM-tier gather gather_threads * 16 bytes
    const uint32_t tile_hbm = hm ? TILE_4K : ctx->gather_threads * 16;
    uint32_t tpc_hbm = tiles_per_chunk(c.cfg.chunk_bytes, tile_hbm);
    uint32_t planes = c.cfg.n_planes;
    ga.n_planes = planes;
    // timing events cannot be recorded into a graph, and taking one from the pool may allocate
    const bool profile = ctx->profile && !ss->fixed && !is_capturing(ss->s);
    const bool host_tier = c.cfg.n_host_slots != 0;
    // one pass over both planes of each request where the cache tier keeps them side by side (see gather; not the
    // head-major gather, see gather_hm)
    const bool fold = !hm && c.cache_planes_adjacent() && !ctx->gather_grid;
    // Grid of the HBM-tier gather: about one workgroup per tile.  The request count lives on the device, so the grid is
    // sized from what the previous gather of this class on this stream reported, never below a floor that still fills the
    // chip, never above the bound; the kernel loops where the grid is short, so any size is correct.  The guess is
    // biased low on purpose: surplus workgroups at the end of the grid cost time (6 % of them 1 %, 23 % of them 3.5 %),
    // a grid 10 to 25 % short costs nothing (the first workgroups take a second tile while the rest still run).
    uint64_t max_tiles = max_req * tpc_hbm;
    uint64_t want = max_tiles;
    // Which of the two gathers stays on the caller's stream: crossing to the side stream and back costs some 15 us each
    // way, so the one that takes longer - by the same report: host bytes at PCIe rate against HBM bytes at HBM rate,
    // about 1 : 48 per request - stays, and the short one takes the detour inside the long one's shadow.
    // And whether there is a detour at all: when even the longer of the two is expected to be over in less time than the
    // two crossings take (a small fetch: a few dozen blocks from the host, or some tens of MiB from HBM), both run on the
    // caller's stream one after the other, and so they do when the class has no host tier.
    bool host_stays = host_tier, serial = !host_tier || !ss->side;
    if (ss->feedback_valid[cls]) {
        uint64_t seen = *(volatile uint32_t *)&ss->h_feedback[cls];
        uint64_t seen_host = *(volatile uint32_t *)&ss->h_feedback[HARVEST_N_CLASSES + cls];
        // (the head-major kernel, whose tiles cost more address arithmetic, does best on an exact grid: +0.8 %)
        uint64_t guess = std::max<uint64_t>(1, hm ? seen : seen - seen / 8) * tpc_hbm;
        want = std::min(max_tiles, std::max<uint64_t>(guess, 16ull * ctx->n_cu));
        host_stays = host_tier && seen_host * 48 > seen;
        double bytes = (double)planes * c.cfg.chunk_bytes * n_rep;
        double us_hbm = 2.0 * seen * bytes / 6.0e6, us_host = seen_host * bytes / 57.0e3;     // at 6 TB/s and 57 GB/s
        // ... or when the shorter one is next to nothing (a fetch served by one tier alone): waiting for the other
        // stream costs the caller's stream more than running a few microseconds of kernel itself
        serial = serial || std::max(us_hbm, us_host) < 35.0 || std::min(us_hbm, us_host) < 8.0;
    }
    if (!serial) {
        HIP_TRY(hipEventRecord(ss->fork, ss->s));
        HIP_TRY(hipStreamWaitEvent(ss->side, ss->fork, 0));
    }
    hipStream_t s_host = (host_stays || serial) ? ss->s : ss->side, s_hbm = (host_stays && !serial) ? ss->side : ss->s;
    uint32_t grid = ctx->gather_grid ? grid_for(want, ctx->gather_grid) : grid_for(want, MAX_GRID);
    for (uint32_t r = 0; r < n_rep; ++r) {
        for (uint32_t p = 0; p < 2; ++p) {
            const uint64_t k = (uint64_t)((int64_t)r + layer_delta);          // may be "negative": the sums wrap back
            ga.src_base[T_HOST][p] = c.host_dev[p] + k * cd.layer_stride[T_HOST];
            ga.src_base[T_CACHE][p] = c.cache_base(p) + k * cd.layer_stride[T_CACHE];
            ga.src_base[T_LOCAL][p] = (uint64_t)c.cfg.d_local_pool[p] + k * cd.layer_stride[T_LOCAL];
        }
        ga.dst_base[0] = dst_base0 + r * dst_step;
        ga.dst_base[1] = dst_base1 + r * dst_step;
        // With profiling on, the events are attached to the dispatch itself and read the kernel's own begin and end.
        hipEvent_t pa = nullptr, pb = nullptr, pc = nullptr, pd = nullptr;
        if (profile) { pa = prof_event(ctx); pb = prof_event(ctx); }
        if (profile && host_tier) { pc = prof_event(ctx); pd = prof_event(ctx); }
        if (host_tier) {             // first, so that the long PCIe transfer starts before the CUs fill up
            ga.tiles_per_chunk = tiles_per_chunk(c.cfg.chunk_bytes, TILE_4K);
            const Rec *recs = (const Rec *)lists.host;
            const uint32_t *n_req = (const uint32_t *)(lists.cnt + C_HOST_REQ);
            uint32_t *fb = ss->d_feedback + HARVEST_N_CLASSES + cls;
            dim3 g(ctx->host_grid);
            if (hm) {
                auto kernel = planes == 2 ? gather_hm_host<2> : gather_hm_host<1>;
                if (pc)
                    hipExtLaunchKernelGGL(kernel, g, dim3(WG), 0, s_host, pc, pd, 0, recs, n_req, ga, *hm, fb, ctx->d_lease);
                else
                    hipLaunchKernelGGL(kernel, g, dim3(WG), 0, s_host, recs, n_req, ga, *hm, fb, ctx->d_lease);
            } else {
                auto kernel = planes == 2 ? gather_host<2> : gather_host<1>;
                if (pc)
                    hipExtLaunchKernelGGL(kernel, g, dim3(WG), 0, s_host, pc, pd, 0, recs, n_req, ga, fb, ctx->d_lease);
                else
                    hipLaunchKernelGGL(kernel, g, dim3(WG), 0, s_host, recs, n_req, ga, fb, ctx->d_lease);
            }
            HIP_TRY(hipGetLastError());
        }
        ga.tiles_per_chunk = tpc_hbm;
        const Rec *recs = (const Rec *)lists.hbm;
        const uint32_t *n_req = (const uint32_t *)(lists.cnt + C_HBM_REQ);
        if (hm) {
            auto kernel = gather_hm<1, true>;
            const dim3 g(grid, planes);
            if (pa)
                hipExtLaunchKernelGGL(kernel, g, dim3(WG), 0, s_hbm, pa, pb, 0, recs, n_req, ga, *hm, ss->d_feedback + cls);
            else
                hipLaunchKernelGGL(kernel, g, dim3(WG), 0, s_hbm, recs, n_req, ga, *hm, ss->d_feedback + cls);
        } else {
            const uint32_t nthr = ctx->gather_threads;
            auto kernel = fold ? (nthr == 64 ? gather<64, true, true> : (nthr == 128 ? gather<128, true, true> : gather<256, true, true>))
                               : (nthr == 64 ? gather<64, true, false> : (nthr == 128 ? gather<128, true, false> : gather<256, true, false>));
            const dim3 g = fold ? dim3(grid_for(want * planes, MAX_GRID)) : dim3(grid, planes);
            if (pa)
                hipExtLaunchKernelGGL(kernel, g, dim3(nthr), 0, s_hbm, pa, pb, 0, recs, n_req, ga, ss->d_feedback + cls);
            else
                hipLaunchKernelGGL(kernel, g, dim3(nthr), 0, s_hbm, recs, n_req, ga, ss->d_feedback + cls);
        }
        HIP_TRY(hipGetLastError());
        if (profile) {
            ctx->prof.push_back({ pa, pb, 0 });
            if (host_tier) ctx->prof.push_back({ pc, pd, 1 });
        }
    }
    ss->feedback_valid[cls] = true;
    if (repeat) {                                   // off the longer gather's stream where there are two
        hipLaunchKernelGGL(repeat_totals, dim3(1), dim3(64), 0, serial ? ss->s : ss->side, (const uint32_t *)lists.cnt,
                           ctx->d_totals + cls * C_N);
        HIP_TRY(hipGetLastError());
    }
    if (!serial) {
        HIP_TRY(hipEventRecord(ss->join, ss->side));
        HIP_TRY(hipStreamWaitEvent(ss->s, ss->join, 0));
    }
    return mark_last(ctx, ss);
}

int check_class(harvest_ctx *ctx, int cls)
{
    if (!ctx) return HARVEST_EINVAL;
    if (cls < 0 || cls >= HARVEST_N_CLASSES || !ctx->cls[cls].used) return HARVEST_ENOENT;
    return HARVEST_OK;
}

// Device-side set-up of a context; on failure the caller destroys the half-built context, which frees whatever exists.
int init_device(harvest_ctx *ctx, const harvest_config *cfg)
{
    HIP_TRY(hipSetDevice(cfg->device));
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDeviceProperties(&prop, cfg->device));
    ctx->n_cu = prop.multiProcessorCount;
    ctx->gather_grid = cfg->gather_wg_per_cu * ctx->n_cu;         // 0: one workgroup per tile
    ctx->host_grid = cfg->host_wgs ? cfg->host_wgs : 24;
    ctx->gather_threads = cfg->gather_threads ? cfg->gather_threads : HBM_WG;
    ctx->ctl_grid = 8 * ctx->n_cu;                 // HBM-bound fills
    // Copies that cross PCIe outside a fetch (place, write-back): persistent workgroups with one 32 KiB tile in flight
    // each, the tiles counted out to them one at a time; they stand back while a fetch says it needs the link (see
    // link_announce).  Alone, 8 of them already fill the link (a 906 MB placement: 15.9 ms = 57 GB/s with 8, 12, 16 or
    // 64; 24 ms with 4); what the number decides is who gets the link when a fetch on another stream wants it too - the
    // link serves its clients by what they have in flight.  Beside a stream of PCIe-bound KV fetches of 1.04 ms each, a
    // placement with 64 workgroups makes a fetch take 8.1 ms, with 32 or 16: 1.3 ms, with 12: 1.2 ms, with 8: 1.1 ms
    // (without the standing back: 16.8, 4.4, 1.8, 1.5, 1.3 ms).  A miss waits on the link, where its transfer contends
    // with whatever else crosses it (paper Section 2.2), and a placement is best effort (Section 3.1), so the copies
    // run narrow.
    ctx->pcie_grid = cfg->pcie_wgs ? cfg->pcie_wgs : 12;
    HIP_TRY(hipStreamCreateWithFlags(&ctx->ctl, hipStreamNonBlocking));
    HIP_TRY(hipStreamCreateWithFlags(&ctx->drain, hipStreamNonBlocking));
    HIP_TRY(hipMalloc(&ctx->d_totals, HARVEST_N_CLASSES * C_N * sizeof(unsigned long long)));
    HIP_TRY(hipMemset(ctx->d_totals, 0, HARVEST_N_CLASSES * C_N * sizeof(unsigned long long)));
    HIP_TRY(hipMalloc(&ctx->d_lease, 256));
    HIP_TRY(hipMemset(ctx->d_lease, 0, 256));
    for (int k = 0; k < HARVEST_N_CLASSES; ++k) {
        ClassState &c = ctx->cls[k];
        if (!c.used) continue;
        HIP_TRY(hipEventCreateWithFlags(&c.edit_evt, hipEventDisableTiming));
        HIP_TRY(hipMalloc(&c.d_dir, (size_t)c.cfg.max_objects * sizeof(uint64_t)));
        HIP_TRY(hipMemset(c.d_dir, 0xFF, (size_t)c.cfg.max_objects * sizeof(uint64_t)));   // tier NONE everywhere
        for (uint32_t p = 0; p < c.cfg.n_planes; ++p) {
            if (!c.cfg.n_host_slots) continue;
            void *d = nullptr;
            if (hipHostGetDevicePointer(&d, c.cfg.host_pool[p], 0) != hipSuccess) {
                fprintf(stderr, "libharvest: host pool plane %u of class %d is not pinned, mapped host memory\n", p, k);
                return HARVEST_EINVAL;
            }
            c.host_dev[p] = (uint64_t)d;
        }
    }
    if (ctx->cls[HARVEST_KV].used) {
        unsigned char *base = nullptr;
        int rc = scratch_of_device(cfg->device, &base);
        if (rc) return rc;
        for (StreamState &ss : ctx->fixed_streams) {
            ss.fixed = true;
            HIP_TRY(hipEventCreateWithFlags(&ss.last, hipEventDisableTiming));
            HIP_TRY(hipHostMalloc((void **)&ss.h_feedback, 64, hipHostMallocDefault));
            memset(ss.h_feedback, 0, 64);
            HIP_TRY(hipHostGetDevicePointer((void **)&ss.d_feedback, ss.h_feedback, 0));
            Lists &l = ss.lists[HARVEST_KV];
            l.hbm = (Rec *)(base + SO_HBM); l.host = (Rec *)(base + SO_HOST); l.miss = (uint32_t *)(base + SO_MISS);
            l.cnt = (uint32_t *)(base + SO_CNT); l.cap = STATIC_CELLS;
            ss.work.tmp = (Rec *)(base + SO_TMP); ss.work.kind = base + SO_KIND;
            ss.work.blk_counts = (uint32_t *)(base + SO_BLK);
        }
    }
    HIP_TRY(hipDeviceSynchronize());
    return HARVEST_OK;
}

}  // namespace

// =============================================================================================================
extern "C" {

const char *harvest_strerror(int status)
{
    switch (status) {
    case HARVEST_OK: return "ok";
    case HARVEST_EINVAL: return "invalid argument";
    case HARVEST_ENOSPC: return "no free slot";
    case HARVEST_ENOENT: return "unknown object or class";
    case HARVEST_EHIP: return "HIP runtime error";
    case HARVEST_ELOST: return "lossy object was revoked";
    case HARVEST_ENODEV: return "context has no device";
    case HARVEST_EBUSY: return "both prefetch buffers are in use, or none is ready; or no fixed stream state is left";
    case HARVEST_E2BIG: return "the request does not fit the fixed scratch of an entry point that allocates nothing";
    }
    return "unknown status";
}

void *harvest_pinned_alloc(size_t bytes)
{
    void *p = nullptr;
    hipError_t e = hipHostMalloc(&p, bytes ? bytes : 1, hipHostMallocDefault);
    if (e != hipSuccess) {
        fprintf(stderr, "libharvest: hipHostMalloc(%zu) failed: %s\n", bytes, hipGetErrorString(e));
        return nullptr;
    }
    return p;
}

int harvest_pinned_free(void *p)
{
    if (!p) return HARVEST_OK;
    HIP_TRY(hipHostFree(p));
    return HARVEST_OK;
}

int harvest_create(const harvest_config *cfg, harvest_ctx **out)
{
    if (!cfg || !out) return HARVEST_EINVAL;
    *out = nullptr;
    for (uint32_t r : cfg->reserved) if (r) return HARVEST_EINVAL;
    if (cfg->gather_threads != 0 && cfg->gather_threads != 64 && cfg->gather_threads != 128 && cfg->gather_threads != 256)
        return HARVEST_EINVAL;
    auto ctx = std::make_unique<harvest_ctx>();
    ctx->cfg = *cfg;
    ctx->no_device = cfg->flags & HARVEST_FLAG_NO_DEVICE;
    ctx->poison = cfg->flags & HARVEST_FLAG_POISON;
    ctx->profile = cfg->flags & HARVEST_FLAG_PROFILE;
    ctx->general_fetch = cfg->flags & HARVEST_FLAG_GENERAL_FETCH;
    ctx->small_cells = cfg->small_fetch_cells ? cfg->small_fetch_cells : SMALL_FETCH_CELLS;
    const uint64_t granule = cfg->shared_granule ? cfg->shared_granule : 4096;
    const bool shared = cfg->d_shared_cache != nullptr || ((cfg->flags & HARVEST_FLAG_NO_DEVICE) && cfg->shared_cache_bytes);
    if (shared) {
        if (granule < 256 || (granule & (granule - 1)) || cfg->shared_cache_bytes % granule ||
            cfg->shared_cache_bytes / granule > 0x3FFFFFFFull || cfg->shared_cache_bytes >= (1ull << 47) ||
            ((uint64_t)cfg->d_shared_cache & 255))
            return HARVEST_EINVAL;
        ctx->shared.reset(cfg->shared_cache_bytes / granule);
    } else if (cfg->shared_cache_bytes || cfg->shared_granule) return HARVEST_EINVAL;
    bool any = false;
    for (int k = 0; k < HARVEST_N_CLASSES; ++k) {
        const harvest_class_config &cc = cfg->cls[k];
        if (cc.n_layers == 0) continue;
        if (cc.n_planes < 1 || cc.n_planes > 2 || cc.chunk_bytes == 0 || cc.chunk_bytes % 16 || cc.max_objects == 0)
            return HARVEST_EINVAL;
        if (cc.max_objects > 0x3FFFFFFFu || cc.n_host_slots > 0x3FFFFFFFu || cc.n_cache_slots > 0x3FFFFFFFu ||
            cc.n_local_slots > 0x3FFFFFFFu)
            return HARVEST_EINVAL;
        if (k == HARVEST_EXPERT && (cc.n_layers != 1 || cc.n_planes != 1 || cc.n_experts == 0 ||
                                    cc.n_experts > MAX_EXPERTS))
            return HARVEST_EINVAL;
        if (!ctx->no_device) {
            for (uint32_t p = 0; p < cc.n_planes; ++p) {
                if (cc.n_host_slots && !cc.host_pool[p]) return HARVEST_EINVAL;
                if (cc.n_cache_slots && !cc.d_cache_pool[p] && !(p == 1 && (cfg->flags & HARVEST_FLAG_CACHE_PLANES_ADJACENT)))
                    return HARVEST_EINVAL;
                if (cc.n_local_slots && !cc.d_local_pool[p]) return HARVEST_EINVAL;
                if (((uint64_t)cc.host_pool[p] | (uint64_t)cc.d_cache_pool[p] | (uint64_t)cc.d_local_pool[p]) & 15)
                    return HARVEST_EINVAL;
            }
        }
        ClassState &c = ctx->cls[k];
        c.cfg = cc;
        c.used = true;
        c.adjacent = (cfg->flags & HARVEST_FLAG_CACHE_PLANES_ADJACENT) && cc.n_planes == 2 && cc.n_cache_slots;
        any = true;
        c.host_used.assign(cc.n_host_slots, 0);
        if (shared && cc.n_cache_slots == 0) {
            c.seg = &ctx->shared;
            c.seg_base = (uint64_t)cfg->d_shared_cache;
            c.granule = granule;
            c.n_granules = cfg->shared_cache_bytes / granule;
            c.obj_granules = ((uint64_t)cc.n_layers * cc.n_planes * cc.chunk_bytes + granule - 1) / granule;
        }
        for (uint32_t s = 0; s < cc.n_cache_slots; ++s) c.cache_free.insert(c.cache_free.end(), s);
        for (uint32_t s = 0; s < cc.n_local_slots; ++s) c.local_free.insert(c.local_free.end(), s);
    }
    if (!any) return HARVEST_EINVAL;
    if (!ctx->no_device) {
        int rc = init_device(ctx.get(), cfg);
        if (rc) {
            harvest_destroy(ctx.release());
            return rc;
        }
    }
    *out = ctx.release();
    return HARVEST_OK;
}

int harvest_destroy(harvest_ctx *ctx)
{
    if (!ctx) return HARVEST_OK;
    if (!ctx->no_device) {
        int rc = device_guard(ctx);
        if (rc) return rc;
        while (!ctx->prefetchers.empty()) (void)harvest_prefetcher_destroy(ctx->prefetchers.back());
        for (auto &kv : ctx->streams) {
            StreamState *ss = kv.second.get();
            (void)hipStreamSynchronize(ss->s);
            (void)hipStreamSynchronize(ss->side);
        }
        (void)hipStreamSynchronize(ctx->ctl);
        if (ctx->drain) (void)hipStreamSynchronize(ctx->drain);
        for (auto &kv : ctx->streams) free_stream_state(kv.second.get());
        for (int i = 0; i < ctx->n_fixed_streams; ++i) (void)hipStreamSynchronize(ctx->fixed_streams[i].s);
        for (StreamState &ss : ctx->fixed_streams) free_stream_state(&ss);
        for (auto &st : ctx->staging) { (void)hipEventDestroy(st.done); (void)hipHostFree(st.h); }
        for (auto &pp : ctx->prof) { (void)hipEventDestroy(pp.a); (void)hipEventDestroy(pp.b); }
        for (auto e : ctx->prof_pool) (void)hipEventDestroy(e);
        for (auto e : ctx->evt_pool) (void)hipEventDestroy(e);
        for (auto &d : ctx->draining) (void)hipEventDestroy(d.e);
        for (auto &c : ctx->cls) if (c.d_dir) (void)hipFree(c.d_dir);
        (void)hipFree(ctx->d_totals);
        (void)hipFree(ctx->d_lease);
        for (auto &c : ctx->cls) if (c.edit_evt) (void)hipEventDestroy(c.edit_evt);
        if (ctx->ctl) (void)hipStreamDestroy(ctx->ctl);
        if (ctx->drain) (void)hipStreamDestroy(ctx->drain);
    }
    delete ctx;
    return HARVEST_OK;
}

int harvest_register(harvest_ctx *ctx, int cls, uint32_t n, const int64_t *host_slot, int tier, harvest_revoke_cb cb,
                     void *user, harvest_obj *out_ids)
{
    int rc = check_class(ctx, cls);
    if (rc) return rc;
    std::lock_guard<std::mutex> lk(ctx->mu);
    ClassState &c = ctx->cls[cls];
    if (tier != HARVEST_HOST && tier != HARVEST_LOCAL) return HARVEST_EINVAL;
    if (!host_slot && tier != HARVEST_LOCAL) return HARVEST_EINVAL;
    if ((uint64_t)c.n_objects + n > c.cfg.max_objects) return HARVEST_ENOSPC;
    if (host_slot) {
        std::unordered_set<int64_t> seen;
        for (uint32_t i = 0; i < n; ++i) {
            if (host_slot[i] < 0 || host_slot[i] >= (int64_t)c.cfg.n_host_slots) return HARVEST_EINVAL;
            if (c.host_used[host_slot[i]] || !seen.insert(host_slot[i]).second) return HARVEST_EINVAL;
        }
    }
    if (tier == HARVEST_LOCAL && c.local_free.size() < n) return HARVEST_ENOSPC;
    if ((rc = device_guard(ctx))) return rc;
    std::vector<uint32_t> ids(n);
    for (uint32_t i = 0; i < n; ++i) {
        uint32_t id = c.n_objects++;
        ids[i] = id;
        c.tier.push_back((uint8_t)tier);
        c.gen.push_back(0);
        c.host_slot.push_back(host_slot ? host_slot[i] : -1);
        if (host_slot) c.host_used[host_slot[i]] = 1;
        c.cb.push_back(cb);
        c.cb_user.push_back(user);
        int64_t s = -1;
        if (tier == HARVEST_LOCAL) { s = *c.local_free.begin(); c.local_free.erase(c.local_free.begin()); }
        c.slot.push_back(s);
        if (out_ids) out_ids[i] = id;
    }
    if ((rc = publish(ctx, c, ids, ctx->ctl, true))) return rc;
    // Later fetches are ordered after this edit on their own streams; only replays of recorded graphs, which the library
    // does not see, need the entry to be there before this call returns.
    if (!ctx->no_device && ctx->captured_work) HIP_TRY(hipEventSynchronize(c.edit_evt));
    return HARVEST_OK;
}

int harvest_restore(harvest_ctx *ctx, int cls, const harvest_obj *ids, uint32_t n)
{
    int rc = check_class(ctx, cls);
    if (rc) return rc;
    if (n && !ids) return HARVEST_EINVAL;
    std::lock_guard<std::mutex> lk(ctx->mu);
    ClassState &c = ctx->cls[cls];
    c.new_call();
    for (uint32_t i = 0; i < n; ++i) {
        if (ids[i] >= c.n_objects) return HARVEST_ENOENT;
        if (c.tier[ids[i]] != T_NONE || !c.first_time(ids[i])) return HARVEST_EINVAL;
    }
    if (c.local_free.size() < n) return HARVEST_ENOSPC;
    if ((rc = device_guard(ctx))) return rc;
    std::vector<uint32_t> changed(ids, ids + n);
    for (uint32_t id : changed) {
        c.slot[id] = *c.local_free.begin();
        c.local_free.erase(c.local_free.begin());
        c.tier[id] = T_LOCAL;
        c.gen[id] += 1;
    }
    if ((rc = publish(ctx, c, changed, ctx->ctl, true))) return rc;
    if (!ctx->no_device && ctx->captured_work) HIP_TRY(hipEventSynchronize(c.edit_evt));
    return HARVEST_OK;
}

int harvest_lookup(harvest_ctx *ctx, int cls, harvest_obj id, int *tier, int64_t *slot, uint32_t *gen,
                   int64_t *host_slot)
{
    int rc = check_class(ctx, cls);
    if (rc) return rc;
    std::lock_guard<std::mutex> lk(ctx->mu);
    ClassState &c = ctx->cls[cls];
    if (id >= c.n_objects) return HARVEST_ENOENT;
    if (tier) *tier = c.tier[id];
    if (slot) *slot = c.slot[id];
    if (gen) *gen = c.gen[id];
    if (host_slot) *host_slot = c.host_slot[id];
    return HARVEST_OK;
}

// Source of a placement that does not read the host copies: planes laid out [layer][stride][chunk], object i at block[i].
struct PlaceSource { uint64_t plane[2]; const uint64_t *block; uint64_t stride; };

static int place_impl(harvest_ctx *ctx, int cls, const harvest_obj *ids, uint32_t n, const PlaceSource *from, void *stream,
                      int *status)
{
    int rc = check_class(ctx, cls);
    if (rc) return rc;
    if (n && !ids) return HARVEST_EINVAL;
    std::lock_guard<std::mutex> lk(ctx->mu);
    ClassState &c = ctx->cls[cls];
    for (uint32_t i = 0; i < n; ++i) {
        if (ids[i] >= c.n_objects) return HARVEST_ENOENT;
        if (from && from->block[i] >= from->stride) return HARVEST_EINVAL;
    }
    if (from && n && !ctx->no_device) {
        if (!from->plane[0] || (c.cfg.n_planes == 2 && !from->plane[1])) return HARVEST_EINVAL;
        if ((from->plane[0] | from->plane[1]) & 15) return HARVEST_EINVAL;
    }
    if ((rc = device_guard(ctx))) return rc;
    // directory edits go through pinned staging: they cannot be recorded into a graph
    if (!ctx->no_device && is_capturing((hipStream_t)stream)) return HARVEST_EINVAL;
    // Everything the call may have to create or allocate comes first - the stream's state, room for the copy list on the
    // device, the two staging blocks - so that nothing has changed yet when one of them fails; what can still fail
    // afterwards (enqueueing on a broken stream) is undone below.
    StreamState *ss = nullptr;
    if (!ctx->no_device && (rc = get_stream(ctx, stream, &ss))) return rc;
    hipStream_t s = ss ? ss->s : nullptr;
    const size_t max_items = (size_t)n * c.cfg.n_planes * c.cfg.n_layers;
    Hold h_items, h_dir;
    if (n) {
        if ((rc = ensure_ctl_cap(ctx, ss, LIST_HEADER + max_items * sizeof(Item)))) return rc;
        if ((rc = acquire_staging(ctx, LIST_HEADER + max_items * sizeof(Item), &h_items.st))) return rc;
        if ((rc = acquire_staging(ctx, (size_t)n * (sizeof(uint64_t) + sizeof(uint32_t)), &h_dir.st))) return rc;
    }
    Undo undo(c);
    std::vector<uint32_t> moved;
    std::vector<Item> items;
    std::vector<int> st_all(n, HARVEST_OK);
    for (uint32_t i = 0; i < n; ++i) {
        uint32_t id = ids[i];
        int st = HARVEST_OK;
        if (c.tier[id] == T_NONE) st = HARVEST_ELOST;
        else if (c.tier[id] != T_HOST) st = HARVEST_OK;
        else if (c.host_slot[id] < 0) st = HARVEST_EINVAL;
        else if (int64_t slot = c.cache_take(); slot < 0) {
            st = HARVEST_ENOSPC;
            c.n_enospc++;
            undo.add(Undo::COUNTED_ENOSPC);
        } else {
            for (uint32_t p = 0; p < c.cfg.n_planes; ++p)
                for (uint32_t l = 0; l < c.cfg.n_layers; ++l) {
                    uint64_t src = from ? from->plane[p] + ((uint64_t)l * from->stride + from->block[i]) * c.cfg.chunk_bytes
                                        : c.addr(T_HOST, p, l, (uint64_t)c.host_slot[id]);
                    items.push_back({ src, c.addr(T_CACHE, p, l, (uint64_t)slot) });
                }
            const uint32_t old_gen = c.gen[id];
            c.tier[id] = T_CACHE; c.slot[id] = slot; c.gen[id] += 1;
            c.n_placed++;
            undo.add(Undo::PLACED, id, slot, old_gen);
            moved.push_back(id);
        }
        st_all[i] = st;
    }
    if (!moved.empty()) {
        size_t bytes = LIST_HEADER + items.size() * sizeof(Item);
        if (!ctx->no_device) {
            memset(h_items.st->h, 0, LIST_HEADER);         // the copy kernel's tile counter
            memcpy((char *)h_items.st->h + LIST_HEADER, items.data(), items.size() * sizeof(Item));
        }
        DEV_TRY(hipMemcpyAsync(ss->ctl_buf, h_items.st->h, bytes, hipMemcpyHostToDevice, s));
        if ((rc = release_after(ctx, h_items.st, s))) return rc;
        if (!ctx->no_device) {
            const Item *d_items = (const Item *)((char *)ss->ctl_buf + LIST_HEADER);
            const uint64_t tiles_hbm = (uint64_t)items.size() * tiles_per_chunk(c.cfg.chunk_bytes, HBM_WG * 16);
            if (from && tiles_hbm < (1ull << 32)) {        // HBM to HBM: a workgroup per 1 KiB tile, as in the gather
                hipLaunchKernelGGL(copy_items_hbm<HBM_WG>, dim3(grid_for(tiles_hbm, MAX_GRID)), dim3(HBM_WG), 0, s,
                                   d_items, (uint32_t)items.size(), c.cfg.chunk_bytes,
                                   tiles_per_chunk(c.cfg.chunk_bytes, HBM_WG * 16));
            } else {                                       // over PCIe: a dozen persistent workgroups, tiles counted out
                uint32_t tpc = tiles_per_chunk(c.cfg.chunk_bytes, TILE_HOST);
                uint32_t grid = grid_for((uint64_t)items.size() * tpc, from ? ctx->ctl_grid : ctx->pcie_grid);
                hipLaunchKernelGGL(copy_items, dim3(grid), dim3(WG), 0, s, d_items, (uint32_t)items.size(),
                                   c.cfg.chunk_bytes, tpc, from ? (unsigned long long *)nullptr : (unsigned long long *)ss->ctl_buf,
                                   from ? (const unsigned long long *)nullptr : (const unsigned long long *)ctx->d_lease);
            }
        }
        DEV_TRY(hipGetLastError());
        // the new entries are written on the same stream, behind the copy: visible only once the bytes are in the slot,
        // and before anything enqueued on `stream` later
        bool committed = false;
        rc = publish(ctx, c, moved, s, false, h_dir.st, &committed);
        if (committed) undo.commit();
        if (rc) return rc;
        if (!ctx->no_device && (rc = mark_last(ctx, ss))) return rc;
    }
    undo.commit();
    if (status) memcpy(status, st_all.data(), n * sizeof(int));
    return HARVEST_OK;
}

int harvest_place(harvest_ctx *ctx, int cls, const harvest_obj *ids, uint32_t n, void *stream, int *status)
{
    return place_impl(ctx, cls, ids, n, nullptr, stream, status);
}

int harvest_place_from(harvest_ctx *ctx, int cls, const harvest_obj *ids, uint32_t n, const void *d_src0, const void *d_src1,
                       const uint64_t *src_block, uint64_t src_layer_stride, void *stream, int *status)
{
    if (n && !src_block) return HARVEST_EINVAL;
    PlaceSource from{ { (uint64_t)d_src0, (uint64_t)d_src1 }, src_block, src_layer_stride };
    return place_impl(ctx, cls, ids, n, &from, stream, status);
}

// Enqueues the poisoning of the given cache slots on the drain stream (the list travels through `st`).
static int enqueue_poison(harvest_ctx *ctx, ClassState &c, const std::vector<uint32_t> &slots, Staging *st)
{
    std::vector<Item> items;
    for (uint32_t s : slots)
        for (uint32_t p = 0; p < c.cfg.n_planes; ++p)
            for (uint32_t l = 0; l < c.cfg.n_layers; ++l) items.push_back({ 0, c.addr(T_CACHE, p, l, s) });
    memcpy(st->h, items.data(), items.size() * sizeof(Item));
    void *d_items = nullptr;
    HIP_TRY(hipHostGetDevicePointer(&d_items, st->h, 0));
    const uint64_t tiles_hbm = (uint64_t)items.size() * tiles_per_chunk(c.cfg.chunk_bytes, HBM_WG * 16);
    if (tiles_hbm < (1ull << 32)) {
        hipLaunchKernelGGL(fill_items_hbm<HBM_WG>, dim3(grid_for(tiles_hbm, MAX_GRID)), dim3(HBM_WG), 0, ctx->drain,
                           (const Item *)d_items, (uint32_t)items.size(), c.cfg.chunk_bytes,
                           tiles_per_chunk(c.cfg.chunk_bytes, HBM_WG * 16), 0xA5A5A5A5u);
    } else {
        uint32_t tpc = tiles_per_chunk(c.cfg.chunk_bytes, TILE_HOST);
        uint32_t grid = grid_for((uint64_t)items.size() * tpc, ctx->ctl_grid);
        hipLaunchKernelGGL(fill_items, dim3(grid), dim3(WG), 0, ctx->drain, (const Item *)d_items, (uint32_t)items.size(),
                           c.cfg.chunk_bytes, tpc, 0xA5A5A5A5u);
    }
    HIP_TRY(hipGetLastError());
    return release_after(ctx, st, ctx->drain);
}

// Revocation (paper Section 3.2).  The context's lock is held while the directory changes and while work is enqueued, and
// released while the host waits for the drain: the thread that drives another stream keeps enqueuing meanwhile.  What
// keeps that safe: the revoked objects already read HOST (mirror and, in stream order, device), so nothing new is pointed
// at their slots, and the slots return to the allocator only after the wait, so nobody else is given them.
//
// The drain is a wait of the host, not of a stream: this call blocks anyway, and a wait parked on a library stream
// would occupy one of the device's few hardware queues until the slowest caller stream has caught up - long enough for
// a caller stream that HIP maps to the same queue to stand still behind it (seen: KV fetches on one stream held up for
// the 7 ms of a placement queued on another).  Each stream's "latest work" event is taken out of the stream's state and
// replaced by a fresh one, so the event the host then waits on is nobody else's: later calls on that stream record the
// new event, and destroying a prefetcher's stream state meanwhile does not touch the one being waited on.  The events
// taken are listed in the context while the wait lasts: a revocation that another thread starts meanwhile finds the
// stream states without them, and waits for the listed ones as well.
static int revoke_impl(harvest_ctx *ctx, int cls, const harvest_obj *ids, uint32_t n, bool notify)
{
    int rc = check_class(ctx, cls);
    if (rc) return rc;
    if (n && !ids) return HARVEST_EINVAL;
    std::vector<uint32_t> hit;
    std::vector<uint32_t> old_slot;
    std::vector<std::pair<harvest_revoke_cb, void *>> cbs;
    ClassState &c = ctx->cls[cls];
    std::vector<harvest_ctx::DrainEvt *> waits;   // the latest work of every stream, as of the invalidation
    bool whole_device = false;
    Staging *st_fill = nullptr;
    {
        std::lock_guard<std::mutex> lk(ctx->mu);
        for (uint32_t i = 0; i < n; ++i) if (ids[i] >= c.n_objects) return HARVEST_ENOENT;
        if ((rc = device_guard(ctx))) return rc;
        // the drain waits for streams: impossible while one of them is being recorded into a graph
        std::vector<StreamState *> busy;       // the streams with work the drain has to wait for
        if (!ctx->no_device) {
            for (auto &kv : ctx->streams) {
                if (is_capturing(kv.first)) return HARVEST_EINVAL;
                if (kv.second->last_valid) busy.push_back(kv.second.get());
            }
            for (int i = 0; i < ctx->n_fixed_streams; ++i) {
                if (is_capturing(ctx->fixed_streams[i].s)) return HARVEST_EINVAL;
                if (ctx->fixed_streams[i].last_valid) busy.push_back(&ctx->fixed_streams[i]);
            }
        }
        size_t n_hit = 0;
        c.new_call();
        for (uint32_t i = 0; i < n; ++i) n_hit += c.tier[ids[i]] == T_CACHE && c.first_time(ids[i]);
        if (n_hit == 0) return HARVEST_OK;
        // what the call may have to allocate comes before any change: staging for the new entries and for the poison
        // list, one fresh event per stream that has work in flight
        Hold h_dir, h_fill;
        if ((rc = acquire_staging(ctx, n_hit * (sizeof(uint64_t) + sizeof(uint32_t)), &h_dir.st))) return rc;
        if (ctx->poison &&
            (rc = acquire_staging(ctx, n_hit * c.cfg.n_planes * c.cfg.n_layers * sizeof(Item), &h_fill.st)))
            return rc;
        if (fault_due()) return HARVEST_EHIP;
        whole_device = ctx->captured_work;
        std::vector<hipEvent_t> fresh;
        struct PutBack {                       // unused events go back to the pool on every return
            harvest_ctx *ctx; std::vector<hipEvent_t> &v;
            ~PutBack() { for (hipEvent_t e : v) ctx->evt_pool.push_back(e); }
        } put_back{ ctx, fresh };
        if (!whole_device)
            for (size_t i = 0; i < busy.size(); ++i) {
                hipEvent_t e = nullptr;
                if (!ctx->evt_pool.empty()) { e = ctx->evt_pool.back(); ctx->evt_pool.pop_back(); }
                else HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
                fresh.push_back(e);
            }
        // 1. invalidate
        Undo undo(c);
        for (uint32_t i = 0; i < n; ++i) {
            uint32_t id = ids[i];
            if (c.tier[id] != T_CACHE) continue;
            const uint32_t slot = (uint32_t)c.slot[id], old_gen = c.gen[id];
            hit.push_back(id);
            old_slot.push_back(slot);
            c.tier[id] = c.host_slot[id] >= 0 ? T_HOST : T_NONE;
            c.slot[id] = -1;
            c.gen[id] += 1;
            c.n_revoked++;
            undo.add(Undo::REVOKED, id, slot, old_gen);
            cbs.push_back({ c.cb[id], c.cb_user[id] });
        }
        bool committed = false;
        rc = publish(ctx, c, hit, ctx->ctl, true, h_dir.st, &committed);
        if (committed) undo.commit();
        if (rc) return rc;
        // 2. the drain, first half: everything the library has enqueued so far on every stream that could still read the
        // slots is what each stream's latest-work event stands for; those events are taken now (later calls on the
        // streams get the fresh ones) and waited for below, with the lock released.  Fetches enqueued from now on need no
        // waiting for: they are ordered after the invalidation above by the class's edit chain.  Work recorded into
        // graphs is invisible to those events: then the host waits for the whole device.
        if (!whole_device) {
            for (auto &d : ctx->draining) {        // what other revocations took before this one is in flight for it too
                d.refs++;
                waits.push_back(&d);
            }
            for (StreamState *ss : busy) {
                ctx->draining.push_back({ ss->last, 1 });
                waits.push_back(&ctx->draining.back());
                ss->last = fresh.back();
                fresh.pop_back();
                ss->last_valid = false;
            }
        }
        if (ctx->poison && !ctx->no_device) {      // stays held until the slots are poisoned, after the wait
            st_fill = h_fill.st;
            h_fill.st = nullptr;
        }
    }
    if (!ctx->no_device) {
        hipError_t e = whole_device ? hipDeviceSynchronize() : hipSuccess;
        for (harvest_ctx::DrainEvt *w : waits)
            if (e == hipSuccess) e = hipEventSynchronize(w->e);    // (the list's entries stay put while anyone refers to them)
        std::unique_lock<std::mutex> lk(ctx->mu);
        for (harvest_ctx::DrainEvt *w : waits)
            if (--w->refs == 0) {
                ctx->evt_pool.push_back(w->e);
                ctx->draining.remove_if([w](const harvest_ctx::DrainEvt &d) { return &d == w; });
            }
        if (e != hipSuccess) {                     // the slots stay out of the allocator: nobody may be given them
            if (st_fill) st_fill->held = false;
            fprintf(stderr, "libharvest: the revocation drain failed: %s\n", hipGetErrorString(e));
            return HARVEST_EHIP;
        }
        if (st_fill) {                             // debug aid: overwrite the slots, now that nothing reads them
            rc = enqueue_poison(ctx, c, old_slot, st_fill);
            if (st_fill->held) st_fill->held = false;
            if (rc) return rc;
            lk.unlock();
            HIP_TRY(hipStreamSynchronize(ctx->drain));
            lk.lock();
        }
        // 3. free
        for (uint32_t s : old_slot) c.cache_release(s);
    } else {
        std::lock_guard<std::mutex> lk(ctx->mu);
        for (uint32_t s : old_slot) c.cache_release(s);
    }
    // 4. notify (outside the lock: a callback may call back into the library)
    for (size_t i = 0; i < hit.size(); ++i)
        if (notify && cbs[i].first) cbs[i].first(cls, hit[i], cbs[i].second);
    return HARVEST_OK;
}

int harvest_revoke(harvest_ctx *ctx, int cls, const harvest_obj *ids, uint32_t n)
{
    return revoke_impl(ctx, cls, ids, n, true);
}

// The three calls of the paper's API (Section 3.2), one object each, on top of the calls above.
int harvest_alloc(harvest_ctx *ctx, int cls, harvest_obj id, void *stream)
{
    int status = HARVEST_OK;
    int rc = harvest_place(ctx, cls, &id, 1, stream, &status);
    return rc ? rc : status;
}

int harvest_free(harvest_ctx *ctx, int cls, harvest_obj id)
{
    return revoke_impl(ctx, cls, &id, 1, false);       // the application's own decision: nobody to notify
}

int harvest_register_cb(harvest_ctx *ctx, int cls, harvest_obj id, harvest_revoke_cb cb, void *user)
{
    int rc = check_class(ctx, cls);
    if (rc) return rc;
    std::lock_guard<std::mutex> lk(ctx->mu);
    ClassState &c = ctx->cls[cls];
    if (id >= c.n_objects) return HARVEST_ENOENT;
    c.cb[id] = cb;
    c.cb_user[id] = user;
    return HARVEST_OK;
}

static int fetch_kv_locked(harvest_ctx *ctx, uint32_t layer, const int32_t *d_block_table, const int32_t *d_n_blocks,
                           uint32_t n_seq, uint32_t max_blocks, void *d_dst_k, void *d_dst_v,
                           const uint64_t *d_seq_dst_block, const uint32_t *d_seq_cap_blocks, uint64_t dst_capacity_blocks,
                           uint32_t n_heads, uint32_t block_tokens, void *stream, uint32_t n_layers,
                           uint64_t dst_layer_stride, StreamState *fixed_ss = nullptr, uint32_t *miss_out = nullptr);

static int fetch_kv_impl(harvest_ctx *ctx, uint32_t layer, const int32_t *d_block_table, const int32_t *d_n_blocks,
                         uint32_t n_seq, uint32_t max_blocks, void *d_dst_k, void *d_dst_v,
                         const uint64_t *d_seq_dst_block, const uint32_t *d_seq_cap_blocks, uint64_t dst_capacity_blocks,
                         uint32_t n_heads, uint32_t block_tokens, void *stream, uint32_t n_layers = 1,
                         uint64_t dst_layer_stride = 0)
{
    int rc = check_class(ctx, HARVEST_KV);
    if (rc) return rc == HARVEST_ENOENT ? HARVEST_EINVAL : rc;
    if (ctx->no_device) return HARVEST_ENODEV;
    std::lock_guard<std::mutex> lk(ctx->mu);
    return fetch_kv_locked(ctx, layer, d_block_table, d_n_blocks, n_seq, max_blocks, d_dst_k, d_dst_v, d_seq_dst_block,
                           d_seq_cap_blocks, dst_capacity_blocks, n_heads, block_tokens, stream, n_layers, dst_layer_stride);
}

// The body of every KV fetch; the context's lock is held.  fixed_ss: the stream's state when it is not one of
// ctx->streams (harvest_fetch_kv_static); miss_out: where the miss list goes instead of the stream's own array.
static int fetch_kv_locked(harvest_ctx *ctx, uint32_t layer, const int32_t *d_block_table, const int32_t *d_n_blocks,
                           uint32_t n_seq, uint32_t max_blocks, void *d_dst_k, void *d_dst_v,
                           const uint64_t *d_seq_dst_block, const uint32_t *d_seq_cap_blocks, uint64_t dst_capacity_blocks,
                           uint32_t n_heads, uint32_t block_tokens, void *stream, uint32_t n_layers,
                           uint64_t dst_layer_stride, StreamState *fixed_ss, uint32_t *miss_out)
{
    int rc;
    ClassState &c = ctx->cls[HARVEST_KV];
    if (n_layers == 0 || (uint64_t)layer + n_layers > c.cfg.n_layers) return HARVEST_EINVAL;
    if (n_layers > 1 && (dst_layer_stride % 16 || dst_layer_stride < dst_capacity_blocks * c.cfg.chunk_bytes))
        return HARVEST_EINVAL;
    uint64_t total = (uint64_t)n_seq * max_blocks;
    if (total >= (1ull << 31)) return HARVEST_EINVAL;
    HmArgs hm{};
    bool head_major = d_seq_cap_blocks != nullptr || n_heads != 0;
    if (head_major) {
        if (!n_heads || !block_tokens || c.cfg.chunk_bytes % ((uint64_t)n_heads * block_tokens)) return HARVEST_EINVAL;
        uint64_t head_bytes = c.cfg.chunk_bytes / ((uint64_t)n_heads * block_tokens);
        if (head_bytes % 16 || (total && !d_seq_cap_blocks)) return HARVEST_EINVAL;
        hm.n_heads = n_heads;
        hm.upr = (uint32_t)(head_bytes / 16);
        hm.ups = hm.upr * block_tokens;
    }
    if ((rc = device_guard(ctx))) return rc;
    StreamState *ss = fixed_ss;
    if (!ss && (rc = get_stream(ctx, stream, &ss))) return rc;
    if ((rc = order_after_directory_edits(ctx, ss, HARVEST_KV))) return rc;
    ss->last_kv.valid = false;
    if (total == 0) { ss->last_cls = HARVEST_KV; ss->counted[HARVEST_KV] = false; return HARVEST_OK; }
    auto remember = [&](bool lists) {
        if (n_layers != 1) return;
        auto &k = ss->last_kv;
        k.valid = true; k.lists = lists; k.layer = layer; k.n_seq = n_seq; k.max_blocks = max_blocks;
        k.n_heads = n_heads; k.block_tokens = block_tokens; k.table = d_block_table; k.n_blocks = d_n_blocks;
        k.seq_dst_block = d_seq_dst_block; k.seq_cap_blocks = d_seq_cap_blocks; k.dst_cap = dst_capacity_blocks;
        k.edit_seq = c.edit_seq;
    };
    if (!d_block_table || !d_n_blocks || !d_seq_dst_block || !d_dst_k || (c.cfg.n_planes == 2 && !d_dst_v))
        return HARVEST_EINVAL;
    if (((uint64_t)d_dst_k | (uint64_t)d_dst_v) & 15) return HARVEST_EINVAL;
    if (total * tiles_per_chunk(c.cfg.chunk_bytes, HBM_WG * 16) * c.cfg.n_planes >= (1ull << 32)) return HARVEST_EINVAL;
    if ((rc = ensure_req_cap(ss, HARVEST_KV, (uint32_t)total))) return rc;
    Lists lists = ss->lists[HARVEST_KV];
    if (miss_out) lists.miss = miss_out;
    const KvWork &work = ss->work;
    uint32_t *cnt = lists.cnt;
    const uint32_t tpc = tiles_per_chunk(c.cfg.chunk_bytes, TILE_4K);
    if (!ctx->general_fetch && !head_major && n_layers <= 65535 && total <= ctx->small_cells && total * tpc <= SMALL_FETCH_TILES) {
        // a small table: the whole fetch is one kernel (no compaction, no second stream) - see fetch_kv_small
        GatherArgs ga{};
        const ClassDev cd = class_dev(c);
        for (uint32_t p = 0; p < 2; ++p) {
            ga.src_base[T_HOST][p] = cd.pool[T_HOST][p];
            ga.src_base[T_CACHE][p] = cd.pool[T_CACHE][p];
            ga.src_base[T_LOCAL][p] = cd.pool[T_LOCAL][p];
        }
        ga.dst_base[0] = (uint64_t)d_dst_k; ga.dst_base[1] = (uint64_t)d_dst_v;
        ga.chunk_bytes = c.cfg.chunk_bytes; ga.tiles_per_chunk = tpc; ga.n_planes = c.cfg.n_planes;
        hipLaunchKernelGGL(fetch_kv_small, dim3((uint32_t)(total * tpc), c.cfg.n_planes, n_layers), dim3(WG), 0, ss->s, cd,
                           layer, d_block_table, d_n_blocks, n_seq, max_blocks, d_seq_dst_block, dst_capacity_blocks, ga,
                           dst_layer_stride, lists.miss, cnt, ctx->d_totals + HARVEST_KV * C_N,
                           ss->d_feedback + HARVEST_KV, ss->d_feedback + HARVEST_N_CLASSES + HARVEST_KV,
                           c.cfg.n_host_slots ? ctx->d_lease : (unsigned long long *)nullptr);
        HIP_TRY(hipGetLastError());
        ss->last_cls = HARVEST_KV; ss->counted[HARVEST_KV] = true;
        ss->feedback_valid[HARVEST_KV] = true;
        remember(false);
        return mark_last(ctx, ss);
    }
    uint32_t n_wg = (uint32_t)((total + WG - 1) / WG);
    hipLaunchKernelGGL(classify_kv, dim3(n_wg), dim3(WG), 0, ss->s, class_dev(c), layer, d_block_table, d_n_blocks, n_seq,
                       max_blocks, d_seq_dst_block, dst_capacity_blocks, work.tmp, work.kind, work.blk_counts,
                       d_seq_cap_blocks, (uint64_t)hm.ups * 16);
    HIP_TRY(hipGetLastError());
    // Beyond this many rows of workgroup totals the compaction's own adding-up of all earlier rows (quadratic) costs more
    // than one more small kernel that groups them first (2 M cells: 70 us against about 10).
    const bool grouped = n_wg > GROUPED_SCAN_ROWS;
    if (grouped) {
        hipLaunchKernelGGL(scan_groups, dim3((n_wg + WG - 1) / WG), dim3(WG), 0, ss->s, (const uint32_t *)work.blk_counts, n_wg,
                           work.grp_totals, work.row_prefix);
        HIP_TRY(hipGetLastError());
    }
    hipLaunchKernelGGL(compact_kv, dim3(n_wg), dim3(WG), 0, ss->s, (uint32_t)total, (const Rec *)work.tmp,
                       (const uint8_t *)work.kind, (const uint32_t *)work.blk_counts, lists.hbm, lists.host,
                       lists.miss, cnt, ctx->d_totals + HARVEST_KV * C_N,
                       grouped ? (const uint32_t *)work.grp_totals : (const uint32_t *)nullptr,
                       grouped ? (const uint32_t *)work.row_prefix : (const uint32_t *)nullptr);
    HIP_TRY(hipGetLastError());
    ss->last_cls = HARVEST_KV; ss->counted[HARVEST_KV] = true;
    // lists recorded into a graph exist only once the graph has been replayed: nothing to use again
    remember(!is_capturing(ss->s));
    return launch_gathers(ctx, ss, c, HARVEST_KV, lists, total, (uint64_t)d_dst_k, (uint64_t)d_dst_v,
                          head_major ? &hm : nullptr, n_layers, dst_layer_stride);
}

int harvest_fetch_kv_again(harvest_ctx *ctx, uint32_t layer, void *d_dst_k, void *d_dst_v, void *stream)
{
    int rc = check_class(ctx, HARVEST_KV);
    if (rc) return rc == HARVEST_ENOENT ? HARVEST_EINVAL : rc;
    if (ctx->no_device) return HARVEST_ENODEV;
    std::lock_guard<std::mutex> lk(ctx->mu);
    ClassState &c = ctx->cls[HARVEST_KV];
    if (layer >= c.cfg.n_layers) return HARVEST_EINVAL;
    auto it = ctx->streams.find((hipStream_t)stream);
    if (it == ctx->streams.end() || !it->second->last_kv.valid) return HARVEST_EINVAL;
    StreamState *ss = it->second.get();
    const auto k = ss->last_kv;
    // The lists of that fetch still describe this one when nothing has edited the directory since (and that fetch made
    // lists at all: small tables are fetched without); otherwise the table is resolved again.
    // A recorded fetch resolves for itself too: by the time its graph is replayed, residency may be another.
    if (!k.lists || k.edit_seq != c.edit_seq || is_capturing((hipStream_t)stream))
        return fetch_kv_locked(ctx, layer, k.table, k.n_blocks, k.n_seq, k.max_blocks, d_dst_k, d_dst_v, k.seq_dst_block,
                               k.seq_cap_blocks, k.dst_cap, k.n_heads, k.block_tokens, stream, 1, 0);
    if (!d_dst_k || (c.cfg.n_planes == 2 && !d_dst_v) || (((uint64_t)d_dst_k | (uint64_t)d_dst_v) & 15)) return HARVEST_EINVAL;
    if ((rc = device_guard(ctx))) return rc;
    HmArgs hm{};
    const bool head_major = k.n_heads != 0;
    if (head_major) {
        hm.n_heads = k.n_heads;
        hm.upr = (uint32_t)(c.cfg.chunk_bytes / ((uint64_t)k.n_heads * k.block_tokens) / 16);
        hm.ups = hm.upr * k.block_tokens;
    }
    ss->last_cls = HARVEST_KV; ss->counted[HARVEST_KV] = true;
    return launch_gathers(ctx, ss, c, HARVEST_KV, ss->lists[HARVEST_KV], (uint64_t)k.n_seq * k.max_blocks, (uint64_t)d_dst_k, (uint64_t)d_dst_v,
                          head_major ? &hm : nullptr, 1, 0, (int64_t)layer - (int64_t)k.layer, true);
}

int harvest_fetch_kv_static(harvest_ctx *ctx, uint32_t layer, const int32_t *d_block_table, const int32_t *d_n_blocks,
                            uint32_t n_seq, uint32_t max_blocks, void *d_dst_k, void *d_dst_v,
                            const uint64_t *d_seq_dst_block, uint64_t dst_capacity_blocks, uint32_t *d_info,
                            uint32_t *d_miss_idx, void *stream)
{
    int rc = check_class(ctx, HARVEST_KV);
    if (rc) return rc == HARVEST_ENOENT ? HARVEST_EINVAL : rc;
    if (ctx->no_device) return HARVEST_ENODEV;
    const uint64_t total = (uint64_t)n_seq * max_blocks;
    if (total > STATIC_CELLS) {
        fprintf(stderr, "libharvest: harvest_fetch_kv_static serves block tables of up to %u cells, this one has %llu\n",
                STATIC_CELLS, (unsigned long long)total);
        return HARVEST_E2BIG;
    }
    std::lock_guard<std::mutex> lk(ctx->mu);
    StreamState *ss = nullptr;
    for (int i = 0; i < ctx->n_fixed_streams && !ss; ++i)
        if (ctx->fixed_streams[i].s == (hipStream_t)stream) ss = &ctx->fixed_streams[i];
    if (!ss) {
        if (ctx->n_fixed_streams == STATIC_STREAMS) {
            fprintf(stderr, "libharvest: harvest_fetch_kv_static serves %d streams per context\n", STATIC_STREAMS);
            return HARVEST_EBUSY;
        }
        ss = &ctx->fixed_streams[ctx->n_fixed_streams++];
        ss->s = (hipStream_t)stream;
    }
    rc = fetch_kv_locked(ctx, layer, d_block_table, d_n_blocks, n_seq, max_blocks, d_dst_k, d_dst_v, d_seq_dst_block, nullptr,
                         dst_capacity_blocks, 0, 0, stream, 1, 0, ss, d_miss_idx);
    if (rc || !d_info) return rc;
    hipLaunchKernelGGL(export_info, dim3(1), dim3(64), 0, ss->s, (const uint32_t *)ss->lists[HARVEST_KV].cnt, d_info,
                       total ? 1u : 0u);
    HIP_TRY(hipGetLastError());
    return mark_last(ctx, ss);
}

int harvest_fetch_kv(harvest_ctx *ctx, uint32_t layer, const int32_t *d_block_table, const int32_t *d_n_blocks,
                     uint32_t n_seq, uint32_t max_blocks, void *d_dst_k, void *d_dst_v,
                     const uint64_t *d_seq_dst_block, uint64_t dst_capacity_blocks, void *stream)
{
    return fetch_kv_impl(ctx, layer, d_block_table, d_n_blocks, n_seq, max_blocks, d_dst_k, d_dst_v, d_seq_dst_block,
                         nullptr, dst_capacity_blocks, 0, 0, stream);
}

int harvest_fetch_kv_layers(harvest_ctx *ctx, uint32_t layer_first, uint32_t n_layers, const int32_t *d_block_table,
                            const int32_t *d_n_blocks, uint32_t n_seq, uint32_t max_blocks, void *d_dst_k, void *d_dst_v,
                            uint64_t dst_layer_stride_bytes, const uint64_t *d_seq_dst_block,
                            uint64_t dst_capacity_blocks, void *stream)
{
    return fetch_kv_impl(ctx, layer_first, d_block_table, d_n_blocks, n_seq, max_blocks, d_dst_k, d_dst_v,
                         d_seq_dst_block, nullptr, dst_capacity_blocks, 0, 0, stream, n_layers, dst_layer_stride_bytes);
}

int harvest_fetch_kv_head_major(harvest_ctx *ctx, uint32_t layer, const int32_t *d_block_table, const int32_t *d_n_blocks,
                                uint32_t n_seq, uint32_t max_blocks, void *d_dst_k, void *d_dst_v,
                                const uint64_t *d_seq_dst_block, const uint32_t *d_seq_cap_blocks,
                                uint64_t dst_capacity_blocks, uint32_t n_heads, uint32_t block_tokens, void *stream)
{
    if (!n_heads || !block_tokens) return HARVEST_EINVAL;
    return fetch_kv_impl(ctx, layer, d_block_table, d_n_blocks, n_seq, max_blocks, d_dst_k, d_dst_v, d_seq_dst_block,
                         d_seq_cap_blocks, dst_capacity_blocks, n_heads, block_tokens, stream);
}

int harvest_fetch_experts(harvest_ctx *ctx, uint32_t layer, const int32_t *d_topk_ids, uint32_t n_tokens, uint32_t k,
                          void *d_staging, uint32_t n_staging_slots, void **d_expert_ptr, void *stream)
{
    int rc = check_class(ctx, HARVEST_EXPERT);
    if (rc) return rc == HARVEST_ENOENT ? HARVEST_EINVAL : rc;
    if (ctx->no_device) return HARVEST_ENODEV;
    std::lock_guard<std::mutex> lk(ctx->mu);
    ClassState &c = ctx->cls[HARVEST_EXPERT];
    uint32_t E = c.cfg.n_experts;
    if ((uint64_t)(layer + 1) * E > c.cfg.max_objects) return HARVEST_EINVAL;
    uint64_t n_ids = (uint64_t)n_tokens * k;
    if (n_ids >= (1ull << 31) || !d_expert_ptr || (n_ids && !d_topk_ids)) return HARVEST_EINVAL;
    if (n_staging_slots && (!d_staging || ((uint64_t)d_staging & 15))) return HARVEST_EINVAL;
    if ((rc = device_guard(ctx))) return rc;
    StreamState *ss;
    if ((rc = get_stream(ctx, stream, &ss))) return rc;
    if ((uint64_t)E * tiles_per_chunk(c.cfg.chunk_bytes, HBM_WG * 16) >= (1ull << 32)) return HARVEST_EINVAL;
    if ((rc = ensure_req_cap(ss, HARVEST_EXPERT, E))) return rc;
    if ((rc = order_after_directory_edits(ctx, ss, HARVEST_EXPERT))) return rc;
    const Lists &lists = ss->lists[HARVEST_EXPERT];
    uint32_t *cnt = lists.cnt;
    // a large batch of routing ids is marked by many workgroups first; the single resolving workgroup reads the bitmap
    const bool marked = n_ids > MARKED_BATCH_IDS;
    if (marked) {
        uint32_t grid = (uint32_t)std::min<uint64_t>(1024, (n_ids + WG * 8 - 1) / (WG * 8));
        hipLaunchKernelGGL(mark_experts, dim3(grid), dim3(WG), 0, ss->s, d_topk_ids, (uint32_t)n_ids, E, ss->mark,
                           ss->mark + MAX_EXPERTS / 32);
        HIP_TRY(hipGetLastError());
    }
    hipLaunchKernelGGL(resolve_experts, dim3(1), dim3(WG), 0, ss->s, class_dev(c), layer, E, d_topk_ids, (uint32_t)n_ids,
                       (uint64_t)d_staging, n_staging_slots, (uint64_t *)d_expert_ptr, lists.hbm, lists.host,
                       lists.miss, cnt, ctx->d_totals + HARVEST_EXPERT * C_N, marked ? ss->mark : (uint32_t *)nullptr,
                       marked ? ss->mark + MAX_EXPERTS / 32 : (uint32_t *)nullptr);
    HIP_TRY(hipGetLastError());
    ss->last_cls = HARVEST_EXPERT; ss->counted[HARVEST_EXPERT] = true;
    return launch_gathers(ctx, ss, c, HARVEST_EXPERT, lists, std::min<uint64_t>(E, n_staging_slots), (uint64_t)d_staging, 0);
}

int harvest_prefetcher_create(harvest_ctx *ctx, void *const d_staging[2], uint32_t n_staging_slots,
                              void **const d_expert_ptr[2], harvest_prefetcher **out)
{
    if (!out) return HARVEST_EINVAL;
    *out = nullptr;
    int rc = check_class(ctx, HARVEST_EXPERT);
    if (rc) return rc == HARVEST_ENOENT ? HARVEST_EINVAL : rc;
    if (ctx->no_device) return HARVEST_ENODEV;
    if (!d_staging || !d_expert_ptr) return HARVEST_EINVAL;
    for (int b = 0; b < 2; ++b) {
        if (!d_expert_ptr[b] || (n_staging_slots && (!d_staging[b] || ((uint64_t)d_staging[b] & 15)))) return HARVEST_EINVAL;
    }
    if (d_staging[0] == d_staging[1] && n_staging_slots) return HARVEST_EINVAL;
    if (d_expert_ptr[0] == d_expert_ptr[1]) return HARVEST_EINVAL;
    if ((rc = device_guard(ctx))) return rc;
    auto pf = std::make_unique<harvest_prefetcher>();
    pf->ctx = ctx;
    pf->n_slots = n_staging_slots;
    for (int b = 0; b < 2; ++b) { pf->staging[b] = d_staging[b]; pf->ptrs[b] = d_expert_ptr[b]; }
    auto fail = [&](void) {
        for (hipEvent_t e : { pf->ready[0], pf->ready[1], pf->freed[0], pf->freed[1], pf->dep }) if (e) (void)hipEventDestroy(e);
        if (pf->fetch) (void)hipStreamDestroy(pf->fetch);
        return HARVEST_EHIP;
    };
    if (hipStreamCreateWithFlags(&pf->fetch, hipStreamNonBlocking) != hipSuccess) return fail();
    for (hipEvent_t *e : { &pf->ready[0], &pf->ready[1], &pf->freed[0], &pf->freed[1], &pf->dep })
        if (hipEventCreateWithFlags(e, hipEventDisableTiming) != hipSuccess) return fail();
    {
        std::lock_guard<std::mutex> lk(ctx->mu);
        ctx->prefetchers.push_back(pf.get());
    }
    *out = pf.release();
    return HARVEST_OK;
}

int harvest_prefetcher_destroy(harvest_prefetcher *pf)
{
    if (!pf) return HARVEST_OK;
    harvest_ctx *ctx = pf->ctx;
    int rc = device_guard(ctx);
    if (rc) return rc;
    {
        std::lock_guard<std::mutex> lk(ctx->mu);
        (void)hipStreamSynchronize(pf->fetch);
        ctx->prefetchers.erase(std::remove(ctx->prefetchers.begin(), ctx->prefetchers.end(), pf), ctx->prefetchers.end());
        auto it = ctx->streams.find(pf->fetch);
        if (it != ctx->streams.end()) {
            (void)hipStreamSynchronize(it->second->side);
            free_stream_state(it->second.get());
            ctx->streams.erase(it);
        }
    }
    for (hipEvent_t e : { pf->ready[0], pf->ready[1], pf->freed[0], pf->freed[1], pf->dep }) (void)hipEventDestroy(e);
    (void)hipStreamDestroy(pf->fetch);
    delete pf;
    return HARVEST_OK;
}

void *harvest_prefetcher_stream(harvest_prefetcher *pf) { return pf ? (void *)pf->fetch : nullptr; }

int harvest_prefetch_issue(harvest_prefetcher *pf, uint32_t layer, const int32_t *d_topk_ids, uint32_t n_tokens,
                           uint32_t k, void *topk_stream)
{
    if (!pf) return HARVEST_EINVAL;
    if (pf->n_issued - pf->n_released >= 2) return HARVEST_EBUSY;
    int rc = device_guard(pf->ctx);
    if (rc) return rc;
    int b = (int)(pf->n_issued & 1);
    // the fetch starts once the routing ids exist and the last consumer of this buffer is done with it
    HIP_TRY(hipEventRecord(pf->dep, (hipStream_t)topk_stream));
    HIP_TRY(hipStreamWaitEvent(pf->fetch, pf->dep, 0));
    if (pf->freed_valid[b]) HIP_TRY(hipStreamWaitEvent(pf->fetch, pf->freed[b], 0));
    rc = harvest_fetch_experts(pf->ctx, layer, d_topk_ids, n_tokens, k, pf->staging[b], pf->n_slots, pf->ptrs[b], pf->fetch);
    if (rc) return rc;
    HIP_TRY(hipEventRecord(pf->ready[b], pf->fetch));
    pf->n_issued++;
    return HARVEST_OK;
}

int harvest_prefetch_acquire(harvest_prefetcher *pf, void *compute_stream, void **d_staging, void ***d_expert_ptr)
{
    if (!pf) return HARVEST_EINVAL;
    if (pf->n_acquired >= pf->n_issued) return HARVEST_EBUSY;
    int rc = device_guard(pf->ctx);
    if (rc) return rc;
    int b = (int)(pf->n_acquired & 1);
    HIP_TRY(hipStreamWaitEvent((hipStream_t)compute_stream, pf->ready[b], 0));
    if (d_staging) *d_staging = pf->staging[b];
    if (d_expert_ptr) *d_expert_ptr = pf->ptrs[b];
    pf->n_acquired++;
    return HARVEST_OK;
}

int harvest_prefetch_release(harvest_prefetcher *pf, void *compute_stream)
{
    if (!pf) return HARVEST_EINVAL;
    if (pf->n_released >= pf->n_acquired) return HARVEST_EINVAL;
    int rc = device_guard(pf->ctx);
    if (rc) return rc;
    int b = (int)(pf->n_released & 1);
    HIP_TRY(hipEventRecord(pf->freed[b], (hipStream_t)compute_stream));
    pf->freed_valid[b] = true;
    pf->n_released++;
    return HARVEST_OK;
}

int harvest_release_stream(harvest_ctx *ctx, void *stream)
{
    if (!ctx) return HARVEST_EINVAL;
    if (ctx->no_device) return HARVEST_ENODEV;
    int rc = device_guard(ctx);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    if (is_capturing(s)) return HARVEST_EINVAL;
    std::unique_ptr<StreamState> gone;
    bool found = false;
    {
        std::lock_guard<std::mutex> lk(ctx->mu);
        for (harvest_prefetcher *pf : ctx->prefetchers)
            if (pf->fetch == s) return HARVEST_EINVAL;
        auto it = ctx->streams.find(s);
        if (it != ctx->streams.end()) {
            gone = std::move(it->second);          // out of the map: no later call, no revocation sees it any more
            ctx->streams.erase(it);
            found = true;
        }
        for (int i = 0; i < ctx->n_fixed_streams; ++i) {
            StreamState &f = ctx->fixed_streams[i];
            if (f.s != s) continue;
            // the fixed state keeps its event, its feedback words and its place in the device's fixed scratch; only what
            // ties it to this stream is reset, and the last state in use moves into the gap
            HIP_TRY(hipStreamSynchronize(s));
            f.s = nullptr;
            f.last_valid = false; f.last_cls = -1; f.last_kv.valid = false;
            for (int k = 0; k < HARVEST_N_CLASSES; ++k) { f.counted[k] = false; f.feedback_valid[k] = false; f.seen_seq[k] = 0; }
            std::swap(f, ctx->fixed_streams[ctx->n_fixed_streams - 1]);
            ctx->n_fixed_streams--;
            found = true;
            break;
        }
    }
    if (!found) return HARVEST_ENOENT;
    if (gone) {                                    // the waits run with the lock released
        hipError_t e = hipStreamSynchronize(gone->s);
        if (e == hipSuccess) e = hipStreamSynchronize(gone->side);
        free_stream_state(gone.get());
        if (e != hipSuccess) return HARVEST_EHIP;
    }
    return HARVEST_OK;
}

int harvest_fetch_info_of(harvest_ctx *ctx, void *stream, int cls, harvest_fetch_counts *counts, uint32_t *miss_idx,
                          uint32_t miss_cap, uint32_t *n_miss)
{
    if (!ctx) return HARVEST_EINVAL;
    if (ctx->no_device) return HARVEST_ENODEV;
    if (cls >= HARVEST_N_CLASSES) return HARVEST_EINVAL;
    int rc = device_guard(ctx);
    if (rc) return rc;
    StreamState *ss = nullptr;
    {
        std::lock_guard<std::mutex> lk(ctx->mu);
        auto it = ctx->streams.find((hipStream_t)stream);
        if (it == ctx->streams.end()) return HARVEST_ENOENT;
        ss = it->second.get();
    }
    // the wait runs outside the lock, so that another thread can enqueue on its own stream meanwhile (it waits for the
    // stream, whose handle it has, and touches the stream's state only once it holds the lock again and has found it
    // still in place)
    HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    std::lock_guard<std::mutex> lk(ctx->mu);
    {
        auto it = ctx->streams.find((hipStream_t)stream);
        if (it == ctx->streams.end() || it->second.get() != ss) return HARVEST_ENOENT;
    }
    if (cls < 0) cls = ss->last_cls;                       // the latest fetch, whichever class it was
    uint32_t h[C_N] = { 0 };
    const Lists *l = cls >= 0 && ss->counted[cls] ? &ss->lists[cls] : nullptr;
    if (l) HIP_TRY(hipMemcpy(h, l->cnt, sizeof h, hipMemcpyDeviceToHost));
    if (counts) {
        counts->n_requests = h[C_REQ]; counts->n_local = h[C_LOCAL]; counts->n_cache = h[C_CACHE];
        counts->n_host = h[C_HOST]; counts->n_lost = h[C_LOST]; counts->n_invalid = h[C_INVALID];
    }
    if (n_miss) *n_miss = h[C_MISS];
    uint32_t m = std::min(h[C_MISS], miss_cap);
    if (miss_idx && m) HIP_TRY(hipMemcpy(miss_idx, l->miss, m * sizeof(uint32_t), hipMemcpyDeviceToHost));
    return HARVEST_OK;
}

int harvest_fetch_info(harvest_ctx *ctx, void *stream, harvest_fetch_counts *counts, uint32_t *miss_idx,
                       uint32_t miss_cap, uint32_t *n_miss)
{
    return harvest_fetch_info_of(ctx, stream, -1, counts, miss_idx, miss_cap, n_miss);
}

int harvest_evict(harvest_ctx *ctx, int cls, int layer, const harvest_obj *ids, uint32_t n, const void *d_src0,
                  const void *d_src1, const uint64_t *src_block, uint64_t src_layer_stride, int flags, void *stream)
{
    int rc = check_class(ctx, cls);
    if (rc) return rc;
    if (n && (!ids || !src_block)) return HARVEST_EINVAL;
    std::lock_guard<std::mutex> lk(ctx->mu);
    ClassState &c = ctx->cls[cls];
    if (layer >= (int)c.cfg.n_layers) return HARVEST_EINVAL;
    bool demote_flag = flags & HARVEST_EVICT_DEMOTE;
    if (demote_flag && layer >= 0 && c.cfg.n_layers != 1) return HARVEST_EINVAL;
    size_t n_demote = 0;
    {
        c.new_call();
        size_t need_cache = 0;
        for (uint32_t i = 0; i < n; ++i) {
            if (ids[i] >= c.n_objects) return HARVEST_ENOENT;
            if (src_block[i] >= src_layer_stride) return HARVEST_EINVAL;
            if (c.tier[ids[i]] == T_NONE) return HARVEST_ELOST;
            if (demote_flag && c.tier[ids[i]] == T_LOCAL) n_demote++;
            if (demote_flag && c.tier[ids[i]] == T_LOCAL && c.host_slot[ids[i]] < 0) need_cache++;
            if (!c.first_time(ids[i])) return HARVEST_EINVAL;
        }
        if (!c.seg && need_cache > c.cache_free.size()) return HARVEST_ENOSPC;
    }
    if (n == 0) return HARVEST_OK;
    if (!ctx->no_device) {
        if (!d_src0 || (c.cfg.n_planes == 2 && !d_src1)) return HARVEST_EINVAL;
        if (((uint64_t)d_src0 | (uint64_t)d_src1) & 15) return HARVEST_EINVAL;
    }
    if ((rc = device_guard(ctx))) return rc;
    if (!ctx->no_device && is_capturing((hipStream_t)stream)) return HARVEST_EINVAL;     // as for harvest_place
    // as in harvest_place: what may have to be created or allocated comes before any change
    StreamState *ss = nullptr;
    if (!ctx->no_device && (rc = get_stream(ctx, stream, &ss))) return rc;
    hipStream_t s = ss ? ss->s : nullptr;
    const uint32_t l0 = layer < 0 ? 0 : (uint32_t)layer, l1 = layer < 0 ? c.cfg.n_layers : (uint32_t)layer + 1;
    const size_t max_items = (size_t)n * c.cfg.n_planes * (l1 - l0);
    Hold h_items, h_dir;
    if ((rc = ensure_ctl_cap(ctx, ss, LIST_HEADER + max_items * sizeof(Item2)))) return rc;
    if ((rc = acquire_staging(ctx, LIST_HEADER + max_items * sizeof(Item2), &h_items.st))) return rc;
    if (n_demote && (rc = acquire_staging(ctx, n_demote * (sizeof(uint64_t) + sizeof(uint32_t)), &h_dir.st))) return rc;
    const uint64_t src[2] = { (uint64_t)d_src0, (uint64_t)d_src1 };
    std::vector<Item2> items;
    items.reserve(max_items);
    std::vector<uint32_t> demoted;
    Undo undo(c);
    // room for every lossy object that leaves local HBM, taken in request order before anything changes: all or nothing
    std::vector<int64_t> room;
    if (demote_flag)
        for (uint32_t i = 0; i < n; ++i)
            if (c.tier[ids[i]] == T_LOCAL && c.host_slot[ids[i]] < 0) {
                int64_t slot = c.cache_take();
                if (slot < 0) return HARVEST_ENOSPC;           // (the slots taken so far go back: undo)
                room.push_back(slot);
                undo.add(Undo::TOOK_CACHE_SLOT, 0, slot);
            }
    size_t n_room = 0;
    for (uint32_t i = 0; i < n; ++i) {
        uint32_t id = ids[i];
        bool demote = demote_flag && c.tier[id] == T_LOCAL;
        int64_t to_cache = -1;                  // a lossy object leaves local HBM for the cache tier: it has no host copy
        if (demote && c.host_slot[id] < 0) to_cache = room[n_room++];
        for (uint32_t p = 0; p < c.cfg.n_planes; ++p)
            for (uint32_t l = l0; l < l1; ++l) {
                uint64_t li = layer < 0 ? l : 0;
                Item2 it{};
                it.src = src[p] + (li * src_layer_stride + src_block[i]) * c.cfg.chunk_bytes;
                if (c.host_slot[id] >= 0) it.dst0 = c.addr(T_HOST, p, l, (uint64_t)c.host_slot[id]);
                if (c.tier[id] == T_CACHE) it.dst1 = c.addr(T_CACHE, p, l, (uint64_t)c.slot[id]);
                if (to_cache >= 0) it.dst1 = c.addr(T_CACHE, p, l, (uint64_t)to_cache);
                if (c.tier[id] == T_LOCAL && !demote) {
                    uint64_t d = c.addr(T_LOCAL, p, l, (uint64_t)c.slot[id]);
                    if (d != it.src) it.dst1 = d;       // a source that already is the slot needs no copy
                }
                if (it.dst0 || it.dst1) items.push_back(it);
            }
        c.n_evicted++;
        undo.add(Undo::COUNTED_EVICTED);
        if (demote) {
            const int64_t old_slot = c.slot[id];
            const uint32_t old_gen = c.gen[id];
            c.local_free.insert((uint32_t)old_slot);
            if (to_cache >= 0) { c.tier[id] = T_CACHE; c.slot[id] = to_cache; }
            else { c.tier[id] = T_HOST; c.slot[id] = -1; }
            c.gen[id] += 1;
            c.n_demoted++;
            undo.add(Undo::DEMOTED, id, old_slot, old_gen);
            demoted.push_back(id);
        }
    }
    if (!items.empty()) {
        size_t bytes = LIST_HEADER + items.size() * sizeof(Item2);
        if (!ctx->no_device) {
            memset(h_items.st->h, 0, LIST_HEADER);         // the copy kernel's tile counter
            memcpy((char *)h_items.st->h + LIST_HEADER, items.data(), items.size() * sizeof(Item2));
        }
        DEV_TRY(hipMemcpyAsync(ss->ctl_buf, h_items.st->h, bytes, hipMemcpyHostToDevice, s));
        if ((rc = release_after(ctx, h_items.st, s))) return rc;
        if (!ctx->no_device) {
            const Item2 *d_items = (const Item2 *)((char *)ss->ctl_buf + LIST_HEADER);
            bool to_host = false;                          // lossy objects move between HBM pools only
            for (const Item2 &it : items) to_host |= it.dst0 != 0;
            const uint64_t tiles_hbm = (uint64_t)items.size() * tiles_per_chunk(c.cfg.chunk_bytes, HBM_WG * 16);
            if (!to_host && tiles_hbm < (1ull << 32)) {
                hipLaunchKernelGGL(copy_items2_hbm<HBM_WG>, dim3(grid_for(tiles_hbm, MAX_GRID)), dim3(HBM_WG), 0, s,
                                   d_items, (uint32_t)items.size(), c.cfg.chunk_bytes,
                                   tiles_per_chunk(c.cfg.chunk_bytes, HBM_WG * 16));
            } else {
                uint32_t tpc = tiles_per_chunk(c.cfg.chunk_bytes, TILE_HOST);
                uint32_t grid = grid_for((uint64_t)items.size() * tpc, to_host ? ctx->pcie_grid : ctx->ctl_grid);
                hipLaunchKernelGGL(copy_items2, dim3(grid), dim3(WG), 0, s, d_items, (uint32_t)items.size(),
                                   c.cfg.chunk_bytes, tpc, to_host ? (unsigned long long *)ss->ctl_buf : (unsigned long long *)nullptr,
                                   to_host ? (const unsigned long long *)ctx->d_lease : (const unsigned long long *)nullptr);
            }
        }
        DEV_TRY(hipGetLastError());
    }
    // Without demotions the write-back itself is the commit point: once the copy is enqueued the bytes will change.
    bool committed = demoted.empty();
    if (!demoted.empty()) rc = publish(ctx, c, demoted, s, true, h_dir.st, &committed);
    if (committed) undo.commit();
    if (rc) return rc;
    if (ctx->no_device) return HARVEST_OK;
    if ((rc = mark_last(ctx, ss))) return rc;
    // A freed local slot may be handed out by the very next harvest_register.  Fetches enqueued through the library are
    // ordered behind the new entry, replays of recorded graphs are not: with recorded work around, the entry has to be
    // on the device before this call returns.
    if (!demoted.empty() && ctx->captured_work) HIP_TRY(hipStreamSynchronize(s));
    return HARVEST_OK;
}

int harvest_stats(harvest_ctx *ctx, harvest_stats_t *out)
{
    if (!ctx || !out) return HARVEST_EINVAL;
    std::lock_guard<std::mutex> lk(ctx->mu);
    memset(out, 0, sizeof *out);
    unsigned long long h[HARVEST_N_CLASSES * C_N] = { 0 };
    if (!ctx->no_device) {
        int rc = device_guard(ctx);
        if (rc) return rc;
        for (auto &kv : ctx->streams) HIP_TRY(hipStreamSynchronize(kv.second->s));
        for (int i = 0; i < ctx->n_fixed_streams; ++i) HIP_TRY(hipStreamSynchronize(ctx->fixed_streams[i].s));
        HIP_TRY(hipMemcpy(h, ctx->d_totals, sizeof h, hipMemcpyDeviceToHost));
    }
    for (int k = 0; k < HARVEST_N_CLASSES; ++k) {
        const ClassState &c = ctx->cls[k];
        if (!c.used) continue;
        const unsigned long long *t = h + k * C_N;
        out->fetch[k].n_requests = t[C_REQ]; out->fetch[k].n_local = t[C_LOCAL]; out->fetch[k].n_cache = t[C_CACHE];
        out->fetch[k].n_host = t[C_HOST]; out->fetch[k].n_lost = t[C_LOST]; out->fetch[k].n_invalid = t[C_INVALID];
        out->n_placed[k] = c.n_placed; out->n_place_enospc[k] = c.n_enospc; out->n_revoked[k] = c.n_revoked;
        out->n_evicted[k] = c.n_evicted; out->n_demoted[k] = c.n_demoted;
        out->cache_slots_in_use[k] = c.cache_in_use;
        out->local_slots_in_use[k] = c.cfg.n_local_slots - c.local_free.size();
    }
    out->shared_granules_free = ctx->shared.n_free;
    out->shared_free_runs = ctx->shared.by_off.size();
    out->shared_longest_free_run = ctx->shared.by_len.empty() ? 0 : ctx->shared.by_len.rbegin()->first;
    return HARVEST_OK;
}

int harvest_profile(harvest_ctx *ctx, harvest_profile_t *out)
{
    if (!ctx || !out) return HARVEST_EINVAL;
    if (ctx->no_device) return HARVEST_ENODEV;
    std::lock_guard<std::mutex> lk(ctx->mu);
    memset(out, 0, sizeof *out);
    int rc = device_guard(ctx);
    if (rc) return rc;
    for (auto &kv : ctx->streams) {
        HIP_TRY(hipStreamSynchronize(kv.second->s));
        HIP_TRY(hipStreamSynchronize(kv.second->side));
    }
    for (auto &pp : ctx->prof) {
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, pp.a, pp.b));
        if (pp.which == 0) { out->hbm_launches++; out->hbm_ms += ms; }
        else { out->host_launches++; out->host_ms += ms; }
        ctx->prof_pool.push_back(pp.a);
        ctx->prof_pool.push_back(pp.b);
    }
    ctx->prof.clear();
    return HARVEST_OK;
}

int harvest_plain_copy(void *d_dst, const void *d_src, uint64_t bytes, void *stream)
{
    if (!d_dst || !d_src || bytes % 16 || (((uint64_t)d_dst | (uint64_t)d_src) & 15)) return HARVEST_EINVAL;
    if (bytes == 0) return HARVEST_OK;
    uint64_t n_tiles = (bytes + HBM_WG * 16 - 1) / (HBM_WG * 16);
    uint32_t grid = grid_for(n_tiles, MAX_GRID);
    hipLaunchKernelGGL(plain_copy<HBM_WG>, dim3(grid), dim3(HBM_WG), 0, (hipStream_t)stream, (uint64_t)d_dst, (uint64_t)d_src,
                       bytes);
    HIP_TRY(hipGetLastError());
    return HARVEST_OK;
}

int harvest_plain_read(const void *d_src, uint64_t bytes, void *d_sink, void *stream)
{
    constexpr int NTHR = 1024;
    if (!d_src || !d_sink || bytes % 16 || ((uint64_t)d_src & 15) || ((uint64_t)d_sink & 3)) return HARVEST_EINVAL;
    if (bytes == 0) return HARVEST_OK;
    uint64_t n_tiles = (bytes + NTHR * 16 - 1) / (NTHR * 16);
    hipLaunchKernelGGL(plain_read<NTHR>, dim3(grid_for(n_tiles, MAX_GRID)), dim3(NTHR), 0, (hipStream_t)stream,
                       (uint64_t)d_src, bytes, (uint32_t *)d_sink);
    HIP_TRY(hipGetLastError());
    return HARVEST_OK;
}

int harvest_plain_write(void *d_dst, uint64_t bytes, uint32_t pattern, void *stream)
{
    constexpr int NTHR = 256;
    if (!d_dst || bytes % 16 || ((uint64_t)d_dst & 15)) return HARVEST_EINVAL;
    if (bytes == 0) return HARVEST_OK;
    uint64_t n_tiles = (bytes + NTHR * 16 - 1) / (NTHR * 16);
    hipLaunchKernelGGL(plain_write<NTHR>, dim3(grid_for(n_tiles, MAX_GRID)), dim3(NTHR), 0, (hipStream_t)stream,
                       (uint64_t)d_dst, bytes, pattern);
    HIP_TRY(hipGetLastError());
    return HARVEST_OK;
}

}  // extern "C"
