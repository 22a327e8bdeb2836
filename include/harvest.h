/*
 * harvest.h - C ABI of the MI355X tiered cache fetch library (libharvest.so).
 *
 * The library implements the data path of Harvest (arxiv 2602.00328): objects
 * (paged KV-cache blocks, MoE expert weights) live in one of three tiers -
 * local HBM of the compute GPU, a cache tier in spare HBM that may be revoked
 * at any time, and an authoritative copy in pinned host DRAM (paper Section
 * 3.1).  A residency directory in device memory maps object -> (tier, slot,
 * generation) (the per-expert residency map of Section 4.3, the block table
 * extended with residency of Section 5.2), and fetches resolve every requested object through it inside
 * HIP kernels and gather the bytes into the caller's working layout.
 *
 * Conventions for every entry point
 *   - Plain C types only.  "d_" arguments are DEVICE pointers, "h_"/unprefixed
 *     pointer arguments are HOST pointers.  `stream` is a hipStream_t passed as
 *     void* (NULL = the null stream).
 *   - Ownership: all pools, destination / staging / source buffers and streams
 *     belong to the caller and are only borrowed; they must outlive the
 *     context (pools) or the enqueued work (buffers).  The library owns the
 *     device directory, its per-stream scratch lists and its events.
 *   - Data-moving calls are asynchronous: they enqueue on `stream` and return;
 *     results are valid in stream order.  The first call on a stream, and a
 *     call with more requests than any before it on that stream, allocates
 *     per-stream scratch (hipMalloc), the latter after waiting for that
 *     stream's earlier work and freeing the smaller scratch (hipFree waits for
 *     the whole device); steady-state calls allocate nothing.  harvest_fetch_kv and
 *     harvest_fetch_experts may be recorded into a HIP graph (stream capture)
 *     once such a call has run on that stream outside capture: they use no
 *     memset and read residency from device memory, so a replay follows every
 *     place / revoke made since.  harvest_place and harvest_evict refuse a
 *     capturing stream, harvest_revoke refuses while any stream the context
 *     knows is capturing (EINVAL, nothing changed).  While a context has recorded work,
 *     harvest_revoke drains by waiting for the whole device.  Directory edits made by place /
 *     revoke / evict(DEMOTE) / register are visible to every fetch enqueued
 *     after the call returns (place: on the same stream; other streams may
 *     still see the older, equally correct, host entry for a while).
 *     harvest_register / restore / revoke have no stream argument; their directory edit runs on a stream of the
 *     library - or, while the class's previous edit (a placement, say) is still queued on the caller stream it was
 *     made on, right behind it on that stream, so that no stream of the library ever waits for a caller's.  The
 *     host-side waits of harvest_revoke are waits of the calling thread only.
 *   - Return value: HARVEST_OK (0) or a negative harvest_status.  A fetch never
 *     fails because of residency (Section 3.1: what the cache tier holds or
 *     has lost changes no result).
 *   - No call mutates the directory except register / place / revoke /
 *     evict(DEMOTE).  In particular a fetch never promotes an object (Section
 *     4.3: a miss leaves the object where it is), and the library never writes
 *     back on its own (Section 3.1: which copies are stale is the application's
 *     business).
 *   - Calls on one context may come from several threads: each call runs under
 *     the context's lock.  A prefetcher belongs to one thread at a time.
 *     Operations that touch the same object from different streams must be
 *     ordered by the caller.
 *
 * Shared cache pool (Section 3.3: the controller allocates best-fit among free
 * segments).  When harvest_config.d_shared_cache is set, every class whose
 * n_cache_slots is 0 takes its cache-tier storage from that one pool instead
 * of from equal-size slots of its own, so objects of different sizes (KV
 * blocks, experts) compete for the same spare HBM.  An object then owns one
 * contiguous segment of ceil(n_layers * n_planes * chunk_bytes / granule)
 * granules laid out [layer][plane][chunk_bytes]; the cache "slot" that
 * harvest_lookup reports is the index of the segment's first granule.  A
 * segment is taken best-fit: from the free run that leaves the fewest granules
 * behind (the lowest of equally good runs), at the low end of that run; freed
 * segments merge with free neighbours.  HARVEST_ENOSPC therefore means "no free
 * run is long enough", which fragmentation can cause while enough granules are
 * free in total.
 *
 * Pool layout (per class, per plane):  [layer][slot][chunk_bytes]  - an object
 * occupies the same slot number in every layer and plane of its tier.  KV
 * objects are logical blocks with planes K and V and one chunk per model layer;
 * expert objects have one plane and one storage layer, and the object for
 * (model layer l, expert e) must be number l * n_experts + e.
 */
#ifndef HARVEST_H
#define HARVEST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct harvest_ctx harvest_ctx;   /* opaque, owned by the library */
typedef uint32_t harvest_obj;             /* dense per-class object number, assigned by harvest_register */

enum harvest_tier { HARVEST_HOST = 0, HARVEST_CACHE = 1, HARVEST_LOCAL = 2, HARVEST_NONE = 3 };

enum harvest_status {
    HARVEST_OK = 0,
    HARVEST_EINVAL = -1,   /* bad argument; nothing was enqueued or changed */
    HARVEST_ENOSPC = -2,   /* no free slot: NOT fatal for place - the object stays on the host (Figure 4) */
    HARVEST_ENOENT = -3,   /* unknown object / class */
    HARVEST_EHIP = -4,     /* a HIP runtime call failed */
    HARVEST_ELOST = -5,    /* lossy object whose cache copy was revoked (Section 3.1) */
    HARVEST_ENODEV = -6,   /* data-moving call on a context created with HARVEST_FLAG_NO_DEVICE */
    HARVEST_EBUSY = -7,    /* prefetcher: both buffers are in use (issue), or no issued fetch is left (acquire);
                              harvest_fetch_kv_static: the context already serves its 4 streams */
    HARVEST_E2BIG = -8     /* harvest_fetch_kv_static: the block table has more cells than its fixed scratch holds */
};

enum harvest_class { HARVEST_KV = 0, HARVEST_EXPERT = 1, HARVEST_N_CLASSES = 2 };

enum harvest_flags {
    HARVEST_FLAG_NO_DEVICE = 1,  /* directory bookkeeping only (no HIP call at all): for host-side tests */
    HARVEST_FLAG_POISON = 2,     /* revoke overwrites the freed cache slot with 0xA5 after the drain */
    HARVEST_FLAG_PROFILE = 4,    /* bracket the gather kernels with events; read them with harvest_profile
                                    (launches recorded into a graph are not timed) */
    HARVEST_FLAG_GENERAL_FETCH = 8, /* harvest_fetch_kv never takes its one-kernel form for small block tables (up to
                                    4096 cells): every fetch runs resolve, compaction and the two gathers - for
                                    measurements and tests of that path; results are the same either way */
    HARVEST_FLAG_CACHE_PLANES_ADJACENT = 16 /* two-plane classes with cache slots of their own keep them in ONE buffer,
                                    d_cache_pool[0], laid out [layer][slot][plane][chunk_bytes] (d_cache_pool[1] is ignored):
                                    the K and V chunk of a block are neighbours, as they are in a segment of the shared
                                    pool, and a fetch reads one run of 2 * chunk_bytes per block instead of two */
};

enum harvest_evict_flags {
    HARVEST_EVICT_DEMOTE = 1     /* local objects leave local HBM after the write-back: slot freed, directory -> HOST
                                    (backed objects) or -> CACHE (lossy objects) */
};

/* Invoked on the thread calling harvest_revoke, after the entry has been invalidated, in-flight work on the slot
 * has drained and the slot has been freed (Section 3.2). */
typedef void (*harvest_revoke_cb)(int cls, harvest_obj id, void *user);

typedef struct harvest_class_config {
    uint32_t n_layers;        /* chunks per object per plane; 0 = class unused */
    uint32_t n_planes;        /* 1 or 2 */
    uint64_t chunk_bytes;     /* multiple of 16 */
    uint32_t max_objects;
    uint32_t n_host_slots, n_cache_slots, n_local_slots;
    uint32_t n_experts;       /* HARVEST_EXPERT only: experts per model layer */
    void *host_pool[2];       /* pinned (hipHostMalloc) host memory, per plane; NULL iff n_host_slots == 0 */
    void *d_cache_pool[2];    /* device memory, per plane; 256-byte aligned */
    void *d_local_pool[2];    /* device memory, per plane; 256-byte aligned */
} harvest_class_config;

typedef struct harvest_config {
    uint32_t flags;                 /* harvest_flags */
    int32_t device;                 /* HIP device ordinal the pools live on */
    harvest_class_config cls[HARVEST_N_CLASSES];
    uint32_t gather_wg_per_cu;      /* tuning: cap the HBM-tier gather at this many workgroups per CU (they then loop
                                       over tiles, and take a request's planes one after the other); 0 = default, one workgroup
                                       per tile of gather_threads * 16 bytes */
    uint32_t host_wgs;              /* tuning: persistent workgroups of the host-tier (PCIe) gather; 0 = default (24) */
    uint32_t shared_granule;        /* segment granule of the shared cache pool in bytes: a power of two >= 256;
                                       0 = 4096 */
    uint32_t small_fetch_cells;     /* tuning: harvest_fetch_kv takes its one-kernel form for block tables of up to this
                                       many cells (n_seq * max_blocks); 0 = default (4096) */
    uint32_t gather_threads;        /* tuning: threads per workgroup of the HBM-tier gather, 64, 128 or 256; 0 = default
                                       (64: one wavefront per workgroup, 1 KiB tiles) */
    uint32_t pcie_wgs;              /* tuning: persistent workgroups of the copies that cross PCIe outside a fetch (place,
                                       write-back), each with one 32 KiB tile in flight; 0 = default (12: enough to fill the link
                                       when alone, few enough that a fetch on another stream keeps most of it) */
    uint32_t reserved[2];           /* must be 0 */
    void *d_shared_cache;           /* optional shared cache pool (device memory, 256-byte aligned), see below */
    uint64_t shared_cache_bytes;    /* its size: a multiple of the granule, at most 2^30 granules */
} harvest_config;

typedef struct harvest_fetch_counts {
    uint64_t n_requests;  /* requests examined (KV: sum of clamped n_blocks; experts: size of the distinct set) */
    uint64_t n_local;     /* served from local HBM (experts: used in place, no bytes moved) */
    uint64_t n_cache;     /* served from the cache tier */
    uint64_t n_host;      /* served from the host copy (the miss list) */
    uint64_t n_lost;      /* lossy and revoked: destination left untouched */
    uint64_t n_invalid;   /* skipped: unknown object, destination out of range, staging full */
} harvest_fetch_counts;

typedef struct harvest_stats_t {
    harvest_fetch_counts fetch[HARVEST_N_CLASSES];   /* running totals over all fetches */
    uint64_t n_placed[HARVEST_N_CLASSES], n_place_enospc[HARVEST_N_CLASSES];
    uint64_t n_revoked[HARVEST_N_CLASSES], n_evicted[HARVEST_N_CLASSES], n_demoted[HARVEST_N_CLASSES];
    uint64_t cache_slots_in_use[HARVEST_N_CLASSES], local_slots_in_use[HARVEST_N_CLASSES];
    /* shared cache pool (all 0 without one): free granules, number of free runs, length of the longest */
    uint64_t shared_granules_free, shared_free_runs, shared_longest_free_run;
} harvest_stats_t;

typedef struct harvest_profile_t {
    uint64_t hbm_launches;  double hbm_ms;    /* HBM-tier gather kernel: launches and summed event time */
    uint64_t host_launches; double host_ms;   /* host-tier gather kernel */
} harvest_profile_t;

/* ---- life cycle ------------------------------------------------------------------------------------------- */

/* Creates a context over caller-owned pools.  Allocates the device directory (8 bytes per object).  EINVAL on
 * misaligned / missing pools or chunk_bytes % 16 != 0; EHIP if the device cannot be used. */
int harvest_create(const harvest_config *cfg, harvest_ctx **out);

/* Waits for all work the library enqueued, frees everything the library owns. */
int harvest_destroy(harvest_ctx *ctx);

/* ---- directory (Sections 3.1, 3.2, 4.3) ------------------------------------------------------------------- */

/* Registers n new objects of class cls; they get consecutive numbers, written to out_ids (may be NULL).
 * tier = HARVEST_HOST: the object lives in its host slot (Section 4.3: at start every expert the user did not pick
 * for local HBM sits in host DRAM).  tier = HARVEST_LOCAL: the object takes the lowest free local slot (Section 4.3:
 * the experts the user picked are loaded into local HBM); the caller then fills that slot (see harvest_lookup).
 * host_slot[i] = slot of the authoritative host copy (backed mode, Section 3.1); host_slot == NULL registers lossy
 * objects, allowed for HARVEST_LOCAL only.  cb/user: revocation callback for these objects (may be NULL).
 * All-or-nothing: EINVAL (slot out of range / already owned / repeated), ENOSPC (max_objects or local pool
 * exhausted).  Synchronous. */
int harvest_register(harvest_ctx *ctx, int cls, uint32_t n, const int64_t *host_slot, int tier,
                     harvest_revoke_cb cb, void *user, harvest_obj *out_ids);

/* The paper's own three calls (Section 3.2: an allocation in the cache tier that may fail, its release, and a callback
 * per allocation), for one object each, expressed through the calls above:
 *   harvest_alloc       = harvest_place of one object; returns its status (ENOSPC: no room, the object stays on the
 *                         host; ELOST; OK also when the object already is in HBM).  The size is the class's object size;
 *                         there are no peers to choose between, so the paper's hints have no counterpart.
 *   harvest_free        = the application gives the object's cache-tier copy back: exactly harvest_revoke (invalidate,
 *                         drain, free), except that no callback is invoked - nobody needs telling.
 *   harvest_register_cb = sets (or, with cb == NULL, clears) the callback harvest_revoke invokes for this object. */
int harvest_alloc(harvest_ctx *ctx, int cls, harvest_obj id, void *stream);
int harvest_free(harvest_ctx *ctx, int cls, harvest_obj id);
int harvest_register_cb(harvest_ctx *ctx, int cls, harvest_obj id, harvest_revoke_cb cb, void *user);

/* Reconstruction of lost objects (Section 3.1: a lossy object that is revoked is lost and rebuilt later; Section 3.2:
 * the revocation callback is where the application starts that).  Each listed object must be lost (tier
 * HARVEST_NONE); it gets the lowest free local slot and a new generation, and the caller then writes the rebuilt
 * bytes into that slot (see harvest_lookup), as it does after registering a local object.  ids: host pointer.
 * All-or-nothing: ENOENT (unknown id), EINVAL (an object that is not lost, or a repeated id), ENOSPC (local pool
 * exhausted).  Synchronous like harvest_register. */
int harvest_restore(harvest_ctx *ctx, int cls, const harvest_obj *ids, uint32_t n);

/* Host-side copy of one directory entry.  slot = cache / local slot, or -1.  ENOENT for unknown ids. */
int harvest_lookup(harvest_ctx *ctx, int cls, harvest_obj id, int *tier, int64_t *slot, uint32_t *gen,
                   int64_t *host_slot);

/* Placement = the paper's harvest_alloc + explicit migration + placement-map update (Sections 3.2, 4.3): for each
 * id on the host, take the lowest free cache slot, copy host copy -> slot on `stream`, then publish
 * (CACHE, slot, gen+1).  per_obj_status[i] (may be NULL, written on success only): OK (also for objects already in HBM:
 * no-op), ENOSPC (cache pool full - object stays on the host), ELOST, EINVAL (lossy object).  The call fails as a
 * whole, changing nothing, for unknown ids (ENOENT) and when a HIP call fails before the new entries are enqueued
 * (EHIP: slots, directory and statistics are as before). */
int harvest_place(harvest_ctx *ctx, int cls, const harvest_obj *ids, uint32_t n, void *stream, int *per_obj_status);

/* Placement from a copy the application already holds in device memory (Section 3.2: the allocation only allocates
 * and every copy stays explicit, so a new cache-tier object may be filled from wherever its bytes are; Section 4.3:
 * after a miss the whole expert sits in local staging memory).  Exactly harvest_place, except that object i is read,
 * in every layer l and plane p, from d_src{p} + (l * src_layer_stride + src_block[i]) * chunk_bytes - the source
 * addressing of harvest_evict with layer < 0 - instead of from its host copy, so nothing crosses PCIe.  For experts
 * (one storage layer) d_src0 is the staging buffer of the fetch, src_block[i] the staging slot and src_layer_stride
 * the number of staging slots.  The host copy is neither read nor written: that the source holds the same bytes is
 * the caller's business (Section 3.1: the runtime keeps no tier coherent).  ids, src_block: host pointers.  The
 * copy is enqueued on `stream`; whatever wrote the source must precede it in stream order.  Statuses and errors as
 * for harvest_place, plus EINVAL (nothing changed) for src_block[i] >= src_layer_stride or a missing / misaligned
 * source plane.  Refuses a capturing stream like harvest_place. */
int harvest_place_from(harvest_ctx *ctx, int cls, const harvest_obj *ids, uint32_t n, const void *d_src0,
                       const void *d_src1, const uint64_t *src_block, uint64_t src_layer_stride, void *stream,
                       int *per_obj_status);

/* Revocation (Section 3.2: an explicit call whose steps come in a fixed order): for each id in the cache tier: publish (HOST, gen+1) - or
 * (NONE) for a lossy object -, wait until every fetch / evict / place enqueued so far on any stream this context
 * has seen has completed (the drain), free the slot (poison it if asked), then invoke the callback.  Ids not in the
 * cache tier are skipped.  Synchronous; ENOENT for unknown ids (nothing changed).
 * The context is locked while the directory changes and while work is enqueued, not while the host waits for the
 * drain: other threads may meanwhile call anything on their own streams.  They see the revoked objects on the host
 * already, and the slots being revoked are handed to nobody before the wait has ended.  EHIP before the new entries
 * were enqueued: nothing changed; EHIP afterwards (the wait itself failed): the objects are on the host and their
 * slots stay out of use. */
int harvest_revoke(harvest_ctx *ctx, int cls, const harvest_obj *ids, uint32_t n);

/* ---- fetch (Sections 4.3, 5.2) ---------------------------------------------------------------------------- */

/* KV fetch (Section 5.2: resolve each required block through the block table, reload what is not local).
 * Request r = s * max_blocks + j, for j < min(max(d_n_blocks[s], 0), max_blocks), asks for block
 * d_block_table[r]; its K chunk of `layer` is copied to d_dst_k + (d_seq_dst_block[s] + j) * chunk_bytes and its V
 * chunk likewise into d_dst_v.  d_dst_k / d_dst_v hold dst_capacity_blocks chunks each.  Requests naming an unknown
 * block or a destination >= dst_capacity_blocks are skipped and counted; lost blocks leave the destination
 * untouched.  HBM-tier requests run on `stream`, host-tier requests on a library-owned side stream that is joined
 * back before this call's work on `stream` ends.  EINVAL: layer out of range, class unused, n_seq * max_blocks
 * >= 2^31. */
int harvest_fetch_kv(harvest_ctx *ctx, uint32_t layer, const int32_t *d_block_table, const int32_t *d_n_blocks,
                     uint32_t n_seq, uint32_t max_blocks, void *d_dst_k, void *d_dst_v,
                     const uint64_t *d_seq_dst_block, uint64_t dst_capacity_blocks, void *stream);

/* The same fetch for n_layers consecutive layers in one call (Section 5.2 moves whole blocks; an engine that reloads a
 * block needs it in every layer).  The block table is resolved once - an object has the same slot in every layer -
 * and layer layer_first + r lands d_dst + r * dst_layer_stride_bytes (a multiple of 16, at least dst_capacity_blocks *
 * chunk_bytes).  The host-tier copies of all layers follow each other without a join in between.  Counts and miss
 * list are per request (block), not per layer.  Nothing can change residency inside one call, and a revocation made
 * after it returns drains all of its layers. */
int harvest_fetch_kv_layers(harvest_ctx *ctx, uint32_t layer_first, uint32_t n_layers, const int32_t *d_block_table,
                            const int32_t *d_n_blocks, uint32_t n_seq, uint32_t max_blocks, void *d_dst_k,
                            void *d_dst_v, uint64_t dst_layer_stride_bytes, const uint64_t *d_seq_dst_block,
                            uint64_t dst_capacity_blocks, void *stream);

/* Repeats the latest single-layer KV fetch enqueued on `stream` (harvest_fetch_kv or harvest_fetch_kv_head_major) for
 * another layer and another destination: same block table, lengths and destination map - the way a decode step walks its
 * layers (Section 5.2: the table says where every block of the step is; it does not change from layer to layer).  The
 * caller vouches that the table arrays of that call have not changed and are still valid device memory.  When no directory
 * edit has happened since that call, its request lists are used again (an object occupies the same slot in every layer),
 * which saves resolving and compacting the table; otherwise, and for the small tables that are fetched without lists, the
 * table is resolved again - the result is the same either way.  Counters and miss list are those of a fetch of this
 * layer; the running totals count the requests again.  EINVAL: no such earlier fetch on this stream (a multi-layer call
 * does not count), layer out of range, missing / misaligned destination. */
int harvest_fetch_kv_again(harvest_ctx *ctx, uint32_t layer, void *d_dst_k, void *d_dst_v, void *stream);

/* The same fetch into a head-major working layout (the paper leaves layouts open; attention kernels that walk one head at
 * a time want this one).  A pool block is [block_tokens][n_heads][head_bytes] with head_bytes = chunk_bytes /
 * (block_tokens * n_heads), a multiple of 16.  Sequence s owns d_seq_cap_blocks[s] (< 65536) destination blocks starting at
 * block d_seq_dst_block[s], laid out [n_heads][d_seq_cap_blocks[s] * block_tokens][head_bytes]; request (s, j) fills rows
 * j * block_tokens ... of every head strip.  Skipped and counted invalid: unknown block, j >= d_seq_cap_blocks[s], a
 * sequence region that ends beyond dst_capacity_blocks.  EINVAL additionally when chunk_bytes does not factor as
 * stated. */
int harvest_fetch_kv_head_major(harvest_ctx *ctx, uint32_t layer, const int32_t *d_block_table,
                                const int32_t *d_n_blocks, uint32_t n_seq, uint32_t max_blocks, void *d_dst_k,
                                void *d_dst_v, const uint64_t *d_seq_dst_block, const uint32_t *d_seq_cap_blocks,
                                uint64_t dst_capacity_blocks, uint32_t n_heads, uint32_t block_tokens, void *stream);

/* harvest_fetch_kv for callers that cannot allocate device memory when they call: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same requests, same bytes in d_dst_k / d_dst_v, but this call never
 * allocates (no hipMalloc / hipFree / hipHostMalloc, no event or stream creation, on any call including the first):
 * everything it needs beyond its arguments - the arrays of the resolve, the two request lists, the counters - lives in
 * a statically allocated device array of about 3.4 MiB, which every GPU the library has created a context on holds
 * until the process ends.  The limit that follows: n_seq * max_blocks <= HARVEST_STATIC_MAX_CELLS table cells,
 * HARVEST_E2BIG (and a message on stderr, nothing enqueued) beyond.  Both gathers run on `stream` one after the other
 * (there is no side stream to overlap the host tier on), so a fetch with a large host-tier share takes the sum of the
 * two, not the longer one.  The fetch may be recorded into a HIP graph without any earlier call.
 *   d_info     (device, 8 words, may be NULL) receives: requests, local, cache, host, lost, invalid, length of the miss
 *              list, 0 - what harvest_fetch_info reports for harvest_fetch_kv;
 *   d_miss_idx (device, n_seq * max_blocks words, may be NULL) receives the miss list in request order.
 * All calls on one GPU - any stream, any context - share that GPU's array and each call overwrites all of it that it
 * reads (nothing in it has to be zero): calls whose execution may overlap on one GPU race, so the caller orders them
 * (one stream, or events).  A context serves up to 4 different streams this way (HARVEST_EBUSY for a fifth).  Revocation
 * drains these fetches like any other.  harvest_fetch_kv_again and harvest_fetch_info do not see them. */
#define HARVEST_STATIC_MAX_CELLS 65536u
int harvest_fetch_kv_static(harvest_ctx *ctx, uint32_t layer, const int32_t *d_block_table, const int32_t *d_n_blocks,
                            uint32_t n_seq, uint32_t max_blocks, void *d_dst_k, void *d_dst_v,
                            const uint64_t *d_seq_dst_block, uint64_t dst_capacity_blocks, uint32_t *d_info,
                            uint32_t *d_miss_idx, void *stream);

/* Expert fetch (Section 4.3: experts are paged whole and must be resident before the FFN runs).  U = the distinct
 * valid expert numbers in d_topk_ids[n_tokens][k].  For e in U ascending: a local expert is used in place
 * (d_expert_ptr[e] = its address in the local pool, no bytes move); a cache- or host-tier expert is copied into
 * staging slot r = number of earlier staged members of U (d_expert_ptr[e] = d_staging + r * chunk_bytes), or, when
 * r >= n_staging_slots, skipped and counted invalid (pointer NULL); a lost expert gets NULL.  Experts not in U get
 * NULL.  d_expert_ptr has n_experts entries. */
int harvest_fetch_experts(harvest_ctx *ctx, uint32_t layer, const int32_t *d_topk_ids, uint32_t n_tokens, uint32_t k,
                          void *d_staging, uint32_t n_staging_slots, void **d_expert_ptr, void *stream);

/* Double-buffered expert prefetch (Section 4.3: the transfers of expert weights for the next micro-batch overlap the
 * computation of the current one).  A prefetcher owns a fetch stream (default priority) and borrows two staging
 * buffers (n_staging_slots * chunk_bytes each, device memory) and two pointer tables (n_experts entries each, device
 * memory) from the caller; they must outlive it.  The three calls form a ring of two:
 *   issue   - harvest_fetch_experts for `layer` into the next buffer, on the fetch stream, after (a) the work enqueued
 *             so far on topk_stream, which produces d_topk_ids, and (b) the release of that buffer's previous use.
 *             EBUSY when two issued fetches are not released yet.
 *   acquire - makes compute_stream wait for the oldest fetch not acquired yet and returns its staging buffer and
 *             pointer table.  EBUSY when every issued fetch has been acquired.
 *   release - the work enqueued so far on compute_stream is the last use of the oldest acquired buffer.  EINVAL when
 *             nothing is acquired.
 * All three only enqueue.  harvest_prefetcher_stream returns the fetch stream (for harvest_fetch_info); destroy waits
 * for it.  harvest_destroy destroys the prefetchers its context still has; their handles are dead afterwards. */
typedef struct harvest_prefetcher harvest_prefetcher;
int harvest_prefetcher_create(harvest_ctx *ctx, void *const d_staging[2], uint32_t n_staging_slots,
                              void **const d_expert_ptr[2], harvest_prefetcher **out);
int harvest_prefetcher_destroy(harvest_prefetcher *pf);
void *harvest_prefetcher_stream(harvest_prefetcher *pf);
int harvest_prefetch_issue(harvest_prefetcher *pf, uint32_t layer, const int32_t *d_topk_ids, uint32_t n_tokens,
                           uint32_t k, void *topk_stream);
int harvest_prefetch_acquire(harvest_prefetcher *pf, void *compute_stream, void **d_staging, void ***d_expert_ptr);
int harvest_prefetch_release(harvest_prefetcher *pf, void *compute_stream);

/* Forgets a caller stream: waits for what the library has enqueued on it, then frees the scratch lists, the side stream and
 * the events the context keeps for it - or, for a stream served by harvest_fetch_kv_static, gives its fixed state back,
 * so that another stream can take it.  For applications that create and destroy streams while a context lives: call it
 * before destroying the stream (a new stream that happens to get the same handle later simply starts afresh).  The next
 * call on the stream sets its state up again, with the allocations of a first call.  Freeing device memory waits for the
 * whole device, so this is no call for a latency-critical moment.  ENOENT: the context has no state for
 * this stream; EINVAL: the stream is being recorded into a graph, or belongs to a prefetcher (harvest_prefetcher_destroy
 * releases that one).  Must not run concurrently with another call that uses the same stream. */
int harvest_release_stream(harvest_ctx *ctx, void *stream);

/* Synchronises `stream` and reports the last fetch enqueued on it: its counts and its miss list (requests served
 * from host or lost: KV request numbers r, or expert numbers e; order unspecified).  miss_idx may be NULL; at most
 * miss_cap entries are written, *n_miss receives the full count. */
int harvest_fetch_info(harvest_ctx *ctx, void *stream, harvest_fetch_counts *counts, uint32_t *miss_idx,
                       uint32_t miss_cap, uint32_t *n_miss);

/* The same for the last fetch of class cls enqueued on `stream` (Sections 4.3 and 5.2: a decode step fetches KV blocks
 * and experts layer by layer, typically on one stream; each class keeps counters and a miss list of its own there, so a
 * later fetch of the other class does not hide them).  cls < 0: the latest fetch of either class, i.e.
 * harvest_fetch_info.  EINVAL: cls >= HARVEST_N_CLASSES. */
int harvest_fetch_info_of(harvest_ctx *ctx, void *stream, int cls, harvest_fetch_counts *counts, uint32_t *miss_idx,
                          uint32_t miss_cap, uint32_t *n_miss);

/* ---- write-back (Sections 5.1, 5.2) ----------------------------------------------------------------------- */

/* Eviction / write-back: the source bytes become the value of each object: they are written to its host slot (when
 * backed) and to the HBM slot the directory names, so every copy stays identical.  ids and src_block are HOST
 * arrays of n entries.  layer >= 0: that layer only, each source plane is [src_layer_stride][chunk_bytes];
 * layer < 0: all layers, each source plane is [n_layers][src_layer_stride][chunk_bytes].  Object i reads source
 * chunk src_block[i] (< src_layer_stride).  d_src1 is ignored for one-plane classes.  HARVEST_EVICT_DEMOTE (all
 * layers, or a one-layer class): local objects leave local HBM - slot freed, directory -> (HOST, gen+1) once the
 * copy is done; the source may be the local pool itself.  A lossy local object (no host slot; Section 5.2: KV state
 * need not be duplicated in a lower tier) moves into the lowest free cache slot instead -> (CACHE, slot, gen+1);
 * ENOSPC, with nothing changed, if the cache tier cannot take every lossy object of the call.  EINVAL: repeated id,
 * src_block out of range; ENOENT; ELOST (the object was revoked).  On error nothing is changed (EHIP included, as long as
 * the call had not yet enqueued its last step).
 * A demoted object's local slot is free the moment the call returns, and the next harvest_register / harvest_restore may
 * hand it out.  Fetches enqueued through this library afterwards see the new entry; a fetch of the same object that is
 * still queued on ANOTHER stream must have been ordered before this call by the caller (as for every operation on one
 * object from two streams), or it may read the slot after its new owner has written it.  While the context has fetches
 * recorded into graphs, a call that demotes waits until the new entries are on the device before it returns. */
int harvest_evict(harvest_ctx *ctx, int cls, int layer, const harvest_obj *ids, uint32_t n, const void *d_src0,
                  const void *d_src1, const uint64_t *src_block, uint64_t src_layer_stride, int flags, void *stream);

/* ---- introspection ---------------------------------------------------------------------------------------- */

/* Running totals.  Synchronises the streams the context has seen. */
int harvest_stats(harvest_ctx *ctx, harvest_stats_t *out);

/* With HARVEST_FLAG_PROFILE: synchronises, returns and resets the event timings of the gather kernels. */
int harvest_profile(harvest_ctx *ctx, harvest_profile_t *out);

/* A plain contiguous device copy with the gather kernel's inner loop (bytes % 16 == 0): the achievable ceiling the
 * gather is compared with, and the known-size kernel used to calibrate hardware byte counters. */
int harvest_plain_copy(void *d_dst, const void *d_src, uint64_t bytes, void *stream);

/* The two halves of that copy on their own, for the same purpose: a read-only stream over d_src (bytes % 16 == 0; d_sink: 4
 * bytes of device memory the kernel may write to - it does not for ordinary data - so that its loads cannot be dropped) and
 * a write-only stream that fills d_dst with a 32-bit pattern.  A copy moves half its bytes each way over the same memory
 * interface, so with r and w the rates of these two, no copy on the machine passes 2 / (1/r + 1/w). */
int harvest_plain_read(const void *d_src, uint64_t bytes, void *d_sink, void *stream);
int harvest_plain_write(void *d_dst, uint64_t bytes, uint32_t pattern, void *stream);

/* Pinned host memory of exactly `bytes` bytes (hipHostMalloc, mapped); NULL on failure. */
void *harvest_pinned_alloc(size_t bytes);
int harvest_pinned_free(void *p);

const char *harvest_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* HARVEST_H */
