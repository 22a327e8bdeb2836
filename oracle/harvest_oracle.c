/*
 * TEST INFRASTRUCTURE - not part of the product.
 *
 * A plain, slow CPU statement of what Harvest's tiered cache fetch computes,
 * written from the paper.  Only tests, the smoke check and the benchmark's
 * CPU-baseline leg may use it; it shares no code with the HIP library.
 *
 * Model (paper Section 3.1): three memory tiers - compute-GPU HBM ("local",
 * authoritative), spare HBM of a peer ("cache", may vanish at any time) and
 * host DRAM (backing store).  Each object is either backed (it owns a host
 * slot holding the authoritative copy) or lossy (no host copy; once revoked it
 * is gone until reconstructed).  A residency directory maps object -> (tier,
 * slot, generation) (the per-expert residency map of Section 4.3, the
 * block table extended with residency of Section 5.2).
 *
 * Storage of one class of objects: every tier is a set of planes (KV: K and
 * V; experts: one), each plane laid out [layer][slot][chunk_bytes].  An object
 * occupies the same slot number in every layer and plane of the tier it is in.
 *
 * Instead of equal-size cache slots a class may draw its cache-tier storage
 * from a segment pool shared with the other class (Section 3.3: the
 * controller allocates best-fit among free segments): an object then owns one
 * contiguous run of granules holding [layer][plane][chunk_bytes], and its
 * cache "slot" is the number of the run's first granule.
 *
 * Beside the tiers the oracle keeps `truth`: the tier-free value of every
 * object, [layer][object][chunk_bytes], written only by orc_set_object and
 * orc_evict.  The plain definition of a fetch ("deliver the current value of
 * each requested object") reads only `truth`; the tiered definition resolves
 * through the directory.  Section 3.1 demands that both always agree for
 * backed objects.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py
 * (closed forms, tier independence, round trips, brute-force enumeration,
 * numpy take / set cross-checks).  Nothing is "parity unpinned".
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { T_HOST = 0, T_CACHE = 1, T_LOCAL = 2, T_NONE = 3 };
enum { ORC_OK = 0, ORC_EINVAL = -1, ORC_ENOSPC = -2, ORC_ENOENT = -3, ORC_ELOST = -5 };
enum { ORC_EVICT_DEMOTE = 1 };
#define ORC_POISON 0xA5

/* Free space of a segment pool: maximal runs of free granules, sorted by offset, never adjacent. */
typedef struct {
    uint64_t n_granules, granule;
    uint8_t *mem;
    uint64_t n_runs, cap_runs;
    uint64_t *run_off, *run_len;
} orc_segpool;

typedef struct {
    uint32_t n_layers, n_planes;
    uint64_t chunk_bytes;
    uint32_t max_objects, n_host_slots, n_cache_slots, n_local_slots;
    int poison;
    orc_segpool *seg;    /* NULL: equal-size cache slots */
    uint8_t *host[2], *cache[2], *local[2], *truth[2];
    /* directory */
    uint32_t n_objects;
    int8_t *tier;
    int64_t *slot;       /* cache or local slot, -1 when tier is HOST/NONE */
    uint32_t *gen;
    int64_t *host_slot;  /* -1 = lossy */
    uint8_t *host_used, *cache_used, *local_used;
} orc_class;

typedef struct {
    uint64_t n_requests, n_local, n_cache, n_host, n_lost, n_invalid;
} orc_counts;

typedef void (*orc_revoke_cb)(uint32_t id, void *user);

static uint8_t *plane_alloc(uint64_t n_layers, uint64_t n_slots, uint64_t chunk)
{
    uint64_t n = n_layers * n_slots * chunk;
    return (uint8_t *)calloc(n ? n : 1, 1);
}

static uint8_t *at(uint8_t *plane, const orc_class *c, uint64_t n_slots, uint32_t layer, uint64_t slot)
{
    return plane + ((uint64_t)layer * n_slots + slot) * c->chunk_bytes;
}

orc_segpool *orc_segpool_create(uint64_t bytes, uint64_t granule)
{
    if (!granule || bytes % granule) return NULL;
    orc_segpool *g = (orc_segpool *)calloc(1, sizeof *g);
    g->n_granules = bytes / granule; g->granule = granule;
    g->mem = (uint8_t *)calloc(bytes ? bytes : 1, 1);
    g->cap_runs = g->n_granules / 2 + 2;
    g->run_off = (uint64_t *)calloc(g->cap_runs, sizeof(uint64_t));
    g->run_len = (uint64_t *)calloc(g->cap_runs, sizeof(uint64_t));
    if (g->n_granules) { g->n_runs = 1; g->run_off[0] = 0; g->run_len[0] = g->n_granules; }
    return g;
}

void orc_segpool_destroy(orc_segpool *g)
{
    if (!g) return;
    free(g->mem); free(g->run_off); free(g->run_len); free(g);
}

uint8_t *orc_segpool_mem(orc_segpool *g) { return g->mem; }

/* free runs as (offset, length) pairs in granules, ascending; returns how many there are */
uint64_t orc_segpool_free_runs(const orc_segpool *g, uint64_t *off, uint64_t *len, uint64_t cap)
{
    for (uint64_t i = 0; i < g->n_runs && i < cap; ++i) { off[i] = g->run_off[i]; len[i] = g->run_len[i]; }
    return g->n_runs;
}

/*
 * Best-fit (Section 3.3): among the free runs that can hold `need` granules
 * take the one that leaves the least behind; of equally good ones the lowest.
 * The allocation sits at the low end of the run.  -1: no run is long enough.
 */
int64_t orc_segpool_alloc(orc_segpool *g, uint64_t need)
{
    if (!need) return -1;
    int64_t best = -1;
    for (uint64_t i = 0; i < g->n_runs; ++i)
        if (g->run_len[i] >= need && (best < 0 || g->run_len[i] < g->run_len[best])) best = (int64_t)i;
    if (best < 0) return -1;
    uint64_t off = g->run_off[best];
    if (g->run_len[best] == need) {
        for (uint64_t i = (uint64_t)best; i + 1 < g->n_runs; ++i) { g->run_off[i] = g->run_off[i + 1]; g->run_len[i] = g->run_len[i + 1]; }
        g->n_runs--;
    } else { g->run_off[best] += need; g->run_len[best] -= need; }
    return (int64_t)off;
}

/* Returns [off, off + len) to the pool, merging with a free neighbour on either side. */
void orc_segpool_free(orc_segpool *g, uint64_t off, uint64_t len)
{
    uint64_t i = 0;
    while (i < g->n_runs && g->run_off[i] < off) ++i;                    /* the new run goes before run i */
    int joins_prev = i > 0 && g->run_off[i - 1] + g->run_len[i - 1] == off;
    int joins_next = i < g->n_runs && off + len == g->run_off[i];
    if (joins_prev && joins_next) {
        g->run_len[i - 1] += len + g->run_len[i];
        for (uint64_t k = i; k + 1 < g->n_runs; ++k) { g->run_off[k] = g->run_off[k + 1]; g->run_len[k] = g->run_len[k + 1]; }
        g->n_runs--;
    } else if (joins_prev) g->run_len[i - 1] += len;
    else if (joins_next) { g->run_off[i] = off; g->run_len[i] += len; }
    else {
        for (uint64_t k = g->n_runs; k > i; --k) { g->run_off[k] = g->run_off[k - 1]; g->run_len[k] = g->run_len[k - 1]; }
        g->run_off[i] = off; g->run_len[i] = len; g->n_runs++;
    }
}

orc_class *orc_create(uint32_t n_layers, uint32_t n_planes, uint64_t chunk_bytes, uint32_t max_objects,
                      uint32_t n_host_slots, uint32_t n_cache_slots, uint32_t n_local_slots, int poison)
{
    if (n_planes < 1 || n_planes > 2 || n_layers < 1 || chunk_bytes == 0)
        return NULL;
    orc_class *c = (orc_class *)calloc(1, sizeof *c);
    c->n_layers = n_layers; c->n_planes = n_planes; c->chunk_bytes = chunk_bytes;
    c->max_objects = max_objects; c->n_host_slots = n_host_slots;
    c->n_cache_slots = n_cache_slots; c->n_local_slots = n_local_slots; c->poison = poison;
    for (uint32_t p = 0; p < n_planes; ++p) {
        c->host[p] = plane_alloc(n_layers, n_host_slots, chunk_bytes);
        c->cache[p] = plane_alloc(n_layers, n_cache_slots, chunk_bytes);
        c->local[p] = plane_alloc(n_layers, n_local_slots, chunk_bytes);
        c->truth[p] = plane_alloc(n_layers, max_objects, chunk_bytes);
    }
    c->tier = (int8_t *)calloc(max_objects + 1, 1);
    c->slot = (int64_t *)calloc(max_objects + 1, sizeof(int64_t));
    c->gen = (uint32_t *)calloc(max_objects + 1, sizeof(uint32_t));
    c->host_slot = (int64_t *)calloc(max_objects + 1, sizeof(int64_t));
    c->host_used = (uint8_t *)calloc(n_host_slots + 1, 1);
    c->cache_used = (uint8_t *)calloc(n_cache_slots + 1, 1);
    c->local_used = (uint8_t *)calloc(n_local_slots + 1, 1);
    return c;
}

void orc_destroy(orc_class *c)
{
    if (!c) return;
    for (int p = 0; p < 2; ++p) { free(c->host[p]); free(c->cache[p]); free(c->local[p]); free(c->truth[p]); }
    free(c->tier); free(c->slot); free(c->gen); free(c->host_slot);
    free(c->host_used); free(c->cache_used); free(c->local_used);
    free(c);
}

/* From now on the class takes its cache-tier storage from segment pool g (it must have no cache slots of its own). */
int orc_attach_segpool(orc_class *c, orc_segpool *g)
{
    if (c->n_cache_slots || c->n_objects || !g) return ORC_EINVAL;
    c->seg = g;
    return ORC_OK;
}

static uint64_t object_bytes(const orc_class *c) { return (uint64_t)c->n_layers * c->n_planes * c->chunk_bytes; }
static uint64_t object_granules(const orc_class *c) { return (object_bytes(c) + c->seg->granule - 1) / c->seg->granule; }

/* Where the cache tier keeps (plane, layer) of the object in cache slot `slot`. */
static uint8_t *cache_at(orc_class *c, uint32_t plane, uint32_t layer, uint64_t slot)
{
    if (c->seg)
        return c->seg->mem + slot * c->seg->granule + ((uint64_t)layer * c->n_planes + plane) * c->chunk_bytes;
    return at(c->cache[plane], c, c->n_cache_slots, layer, slot);
}

/* raw plane pointers, so the harness can look at (or, for the local pool it owns, write) tier contents.
 * which: 0 host, 1 cache, 2 local, 3 truth */
uint8_t *orc_plane(orc_class *c, int which, uint32_t plane)
{
    if (plane >= c->n_planes) return NULL;
    switch (which) {
    case 0: return c->host[plane];
    case 1: return c->cache[plane];
    case 2: return c->local[plane];
    case 3: return c->truth[plane];
    }
    return NULL;
}

uint32_t orc_n_objects(const orc_class *c) { return c->n_objects; }

static int64_t lowest_free(const uint8_t *used, uint32_t n)
{
    for (uint32_t s = 0; s < n; ++s)
        if (!used[s]) return s;
    return -1;
}

/* Room in the cache tier for one object: the lowest free slot, or a best-fit segment.  -1: none. */
static int64_t cache_take(orc_class *c)
{
    if (c->seg) return orc_segpool_alloc(c->seg, object_granules(c));
    int64_t s = lowest_free(c->cache_used, c->n_cache_slots);
    if (s >= 0) c->cache_used[s] = 1;
    return s;
}

static void cache_release(orc_class *c, int64_t slot)
{
    if (c->seg) orc_segpool_free(c->seg, (uint64_t)slot, object_granules(c));
    else c->cache_used[slot] = 0;
}

/*
 * Section 3.1 / 4.3: objects enter the system either in local HBM (at start
 * the user picks the experts that are loaded there) or in host DRAM (all the
 * others).
 * host_slot == NULL registers lossy objects (local tier only: a lossy object
 * with no copy anywhere would be meaningless).  All-or-nothing.
 */
int orc_register(orc_class *c, uint32_t n, const int64_t *host_slot, int tier, uint32_t *out_ids)
{
    if (tier != T_HOST && tier != T_LOCAL) return ORC_EINVAL;
    if (!host_slot && tier != T_LOCAL) return ORC_EINVAL;
    if ((uint64_t)c->n_objects + n > c->max_objects) return ORC_ENOSPC;
    if (host_slot) {
        for (uint32_t i = 0; i < n; ++i) {
            if (host_slot[i] < 0 || host_slot[i] >= (int64_t)c->n_host_slots) return ORC_EINVAL;
            if (c->host_used[host_slot[i]]) return ORC_EINVAL;
            for (uint32_t j = 0; j < i; ++j)
                if (host_slot[j] == host_slot[i]) return ORC_EINVAL;
        }
    }
    if (tier == T_LOCAL) {
        uint32_t free_local = 0;
        for (uint32_t s = 0; s < c->n_local_slots; ++s) free_local += !c->local_used[s];
        if (free_local < n) return ORC_ENOSPC;
    }
    for (uint32_t i = 0; i < n; ++i) {
        uint32_t id = c->n_objects++;
        c->host_slot[id] = host_slot ? host_slot[i] : -1;
        if (host_slot) c->host_used[host_slot[i]] = 1;
        c->gen[id] = 0;
        c->tier[id] = (int8_t)tier;
        c->slot[id] = -1;
        if (tier == T_LOCAL) {
            int64_t s = lowest_free(c->local_used, c->n_local_slots);
            c->local_used[s] = 1;
            c->slot[id] = s;
        }
        if (out_ids) out_ids[i] = id;
    }
    return ORC_OK;
}

/*
 * Reconstruction (Section 3.1: a lossy object that was revoked is lost and
 * the application rebuilds it later; Section 3.2: the callback starts that).
 * Every listed object must be lost; each gets the lowest free local slot and a
 * new generation, and the harness then writes the rebuilt bytes there.
 * All or nothing.
 */
int orc_restore(orc_class *c, const uint32_t *ids, uint32_t n)
{
    uint32_t free_local = 0;
    for (uint32_t s = 0; s < c->n_local_slots; ++s) free_local += !c->local_used[s];
    for (uint32_t i = 0; i < n; ++i) {
        if (ids[i] >= c->n_objects) return ORC_ENOENT;
        if (c->tier[ids[i]] != T_NONE) return ORC_EINVAL;
        for (uint32_t j = 0; j < i; ++j)
            if (ids[j] == ids[i]) return ORC_EINVAL;
    }
    if (free_local < n) return ORC_ENOSPC;
    for (uint32_t i = 0; i < n; ++i) {
        int64_t s = lowest_free(c->local_used, c->n_local_slots);
        c->local_used[s] = 1;
        c->tier[ids[i]] = T_LOCAL; c->slot[ids[i]] = s; c->gen[ids[i]] += 1;
    }
    return ORC_OK;
}

int orc_lookup(const orc_class *c, uint32_t id, int *tier, int64_t *slot, uint32_t *gen, int64_t *host_slot)
{
    if (id >= c->n_objects) return ORC_ENOENT;
    *tier = c->tier[id]; *slot = c->slot[id]; *gen = c->gen[id]; *host_slot = c->host_slot[id];
    return ORC_OK;
}

/* The bytes of object id in (plane, layer) as the directory resolves them; NULL when lost. */
static uint8_t *resolve(orc_class *c, uint32_t id, uint32_t plane, uint32_t layer)
{
    switch (c->tier[id]) {
    case T_LOCAL: return at(c->local[plane], c, c->n_local_slots, layer, (uint64_t)c->slot[id]);
    case T_CACHE: return cache_at(c, plane, layer, (uint64_t)c->slot[id]);
    case T_HOST:  return at(c->host[plane], c, c->n_host_slots, layer, (uint64_t)c->host_slot[id]);
    default:      return NULL;
    }
}

/*
 * Harness initialisation of one object's value (all layers): the bytes land
 * wherever the object currently lives - its host slot when backed, and its
 * local slot when local - and in `truth`.  src planes are
 * [n_layers][chunk_bytes].
 */
int orc_set_object(orc_class *c, uint32_t id, const uint8_t *src0, const uint8_t *src1)
{
    if (id >= c->n_objects) return ORC_ENOENT;
    if (c->tier[id] == T_CACHE || c->tier[id] == T_NONE) return ORC_EINVAL;
    const uint8_t *src[2] = { src0, src1 };
    for (uint32_t p = 0; p < c->n_planes; ++p)
        for (uint32_t l = 0; l < c->n_layers; ++l) {
            const uint8_t *s = src[p] + (uint64_t)l * c->chunk_bytes;
            memcpy(at(c->truth[p], c, c->max_objects, l, id), s, c->chunk_bytes);
            if (c->host_slot[id] >= 0)
                memcpy(at(c->host[p], c, c->n_host_slots, l, (uint64_t)c->host_slot[id]), s, c->chunk_bytes);
            if (c->tier[id] == T_LOCAL)
                memcpy(at(c->local[p], c, c->n_local_slots, l, (uint64_t)c->slot[id]), s, c->chunk_bytes);
        }
    return ORC_OK;
}

/*
 * Harness write into an object that lives in local HBM (a decode step
 * appending a token's rows to the open tail block): the application owns local
 * HBM (Section 3.1 names the compute GPU's HBM the authoritative tier), so this is not a
 * library call; `truth` follows because the local copy IS the value.
 */
int orc_write_local(orc_class *c, uint32_t id, uint32_t plane, uint32_t layer, uint64_t offset,
                    const uint8_t *src, uint64_t n)
{
    if (id >= c->n_objects) return ORC_ENOENT;
    if (c->tier[id] != T_LOCAL || plane >= c->n_planes || layer >= c->n_layers || offset + n > c->chunk_bytes)
        return ORC_EINVAL;
    memcpy(at(c->local[plane], c, c->n_local_slots, layer, (uint64_t)c->slot[id]) + offset, src, n);
    memcpy(at(c->truth[plane], c, c->max_objects, layer, id) + offset, src, n);
    return ORC_OK;
}

/*
 * Placement (Section 3.2: harvest_alloc + explicit copy + record in the
 * placement map; Section 4.3: the rebalancer moves chosen experts into peer
 * HBM as room appears).  With equal-size slots best-fit degenerates and the lowest
 * free slot is taken; with a segment pool the allocation is best-fit.  A failed allocation leaves the object on the host
 * (Figure 4 caption).  status[i] per object; the call itself fails only on an
 * unknown id.
 */
int orc_place(orc_class *c, const uint32_t *ids, uint32_t n, int *status)
{
    for (uint32_t i = 0; i < n; ++i)
        if (ids[i] >= c->n_objects) return ORC_ENOENT;
    for (uint32_t i = 0; i < n; ++i) {
        uint32_t id = ids[i];
        int st = ORC_OK;
        if (c->tier[id] == T_NONE) st = ORC_ELOST;
        else if (c->tier[id] != T_HOST) st = ORC_OK;          /* already in HBM: nothing to do */
        else {
            int64_t s = cache_take(c);
            if (s < 0) st = ORC_ENOSPC;
            else {
                for (uint32_t p = 0; p < c->n_planes; ++p)
                    for (uint32_t l = 0; l < c->n_layers; ++l)
                        memcpy(cache_at(c, p, l, (uint64_t)s),
                               at(c->host[p], c, c->n_host_slots, l, (uint64_t)c->host_slot[id]), c->chunk_bytes);
                c->tier[id] = T_CACHE; c->slot[id] = s; c->gen[id] += 1;
            }
        }
        if (status) status[i] = st;
    }
    return ORC_OK;
}

/*
 * Placement from a copy the application already holds in GPU memory.  Section
 * 3.2: the allocation call only allocates and every copy stays explicit, so
 * the bytes of a new cache-tier object may come from wherever the application
 * has them - after a miss an expert sits complete in local staging memory
 * (Section 4.3), and moving it to the cache tier from there saves the second
 * trip over PCIe.  Object i is read from plane p at
 * src[p] + (layer * src_layer_stride + src_block[i]) * chunk_bytes, all
 * layers, as orc_evict reads its source.  Everything else is orc_place: only
 * an object on the host moves, the lowest free slot (or a best-fit segment)
 * is taken, a failed allocation leaves the object where it is.  The host copy
 * is neither read nor written; that the source equals it is the
 * application's business (Section 3.1: the runtime keeps no tier coherent).
 */
int orc_place_from(orc_class *c, const uint32_t *ids, uint32_t n, const uint8_t *src0, const uint8_t *src1,
                   const uint64_t *src_block, uint64_t src_layer_stride, int *status)
{
    const uint8_t *src[2] = { src0, src1 };
    for (uint32_t i = 0; i < n; ++i) {
        if (ids[i] >= c->n_objects) return ORC_ENOENT;
        if (src_block[i] >= src_layer_stride) return ORC_EINVAL;
    }
    for (uint32_t i = 0; i < n; ++i) {
        uint32_t id = ids[i];
        int st = ORC_OK;
        if (c->tier[id] == T_NONE) st = ORC_ELOST;
        else if (c->tier[id] == T_CACHE || c->tier[id] == T_LOCAL) st = ORC_OK;      /* in HBM already: not written */
        else {
            int64_t room = cache_take(c);
            if (room < 0) st = ORC_ENOSPC;
            else {
                for (uint32_t p = 0; p < c->n_planes; ++p)
                    for (uint32_t l = 0; l < c->n_layers; ++l) {
                        const uint8_t *from = src[p] + ((uint64_t)l * src_layer_stride + src_block[i]) * c->chunk_bytes;
                        memcpy(cache_at(c, p, l, (uint64_t)room), from, c->chunk_bytes);
                    }
                c->tier[id] = T_CACHE; c->slot[id] = room; c->gen[id] = c->gen[id] + 1;
            }
        }
        if (status) status[i] = st;
    }
    return ORC_OK;
}

/*
 * Revocation (Section 3.2: an explicit call whose steps come in a fixed
 * order): invalidate the entry, (drain - nothing is in flight on a CPU),
 * free the slot, then invoke the callback.  Backed objects fall back to their
 * host copy (Sections 4.3, 5.2); lossy ones are gone (Section 3.1).  With
 * poison on, the freed slot is overwritten so that a stale read cannot pass
 * for correct data.
 */
int orc_revoke(orc_class *c, const uint32_t *ids, uint32_t n, orc_revoke_cb cb, void *user)
{
    for (uint32_t i = 0; i < n; ++i)
        if (ids[i] >= c->n_objects) return ORC_ENOENT;
    uint8_t *hit = (uint8_t *)calloc(n ? n : 1, 1);
    int64_t *old = (int64_t *)calloc(n ? n : 1, sizeof(int64_t));
    for (uint32_t i = 0; i < n; ++i) {               /* invalidate */
        uint32_t id = ids[i];
        if (c->tier[id] != T_CACHE) continue;
        hit[i] = 1; old[i] = c->slot[id];
        c->tier[id] = c->host_slot[id] >= 0 ? T_HOST : T_NONE;
        c->slot[id] = -1; c->gen[id] += 1;
    }
    for (uint32_t i = 0; i < n; ++i) {               /* free (+ poison) */
        if (!hit[i]) continue;
        if (c->poison)
            for (uint32_t p = 0; p < c->n_planes; ++p)
                for (uint32_t l = 0; l < c->n_layers; ++l)
                    memset(cache_at(c, p, l, (uint64_t)old[i]), ORC_POISON, c->chunk_bytes);
        cache_release(c, old[i]);
    }
    for (uint32_t i = 0; i < n; ++i)                 /* notify */
        if (hit[i] && cb) cb(ids[i], user);
    free(hit); free(old);
    return ORC_OK;
}

/*
 * KV fetch, tiered definition (Section 5.2: the decode worker looks every
 * block it needs up in the block table, which says where the block lives;
 * non-local blocks are reloaded; after revocation the entry falls back
 * to host DRAM).  Request r = s * max_blocks + j asks for block table[r] of
 * sequence s and lands in dst block seq_dst_block[s] + j of dst_k / dst_v.
 * Invalid requests (unknown block, dst index beyond dst_capacity_blocks) are
 * skipped and counted.  Lost blocks leave dst untouched.  miss_idx receives
 * the requests served from host or lost, in ascending r.
 */
int orc_fetch_kv(orc_class *c, uint32_t layer, const int32_t *table, const int32_t *n_blocks, uint32_t n_seq,
                 uint32_t max_blocks, uint8_t *dst_k, uint8_t *dst_v, const uint64_t *seq_dst_block,
                 uint64_t dst_capacity_blocks, uint32_t *miss_idx, uint32_t *n_miss, orc_counts *counts, int threads)
{
    if (layer >= c->n_layers) return ORC_EINVAL;
    uint8_t *dst[2] = { dst_k, dst_v };
    orc_counts k = { 0, 0, 0, 0, 0, 0 };
    uint32_t nm = 0;
    /* pass 1: classify, in request order */
    for (uint32_t s = 0; s < n_seq; ++s) {
        int64_t nb = n_blocks[s] < 0 ? 0 : n_blocks[s];
        if (nb > (int64_t)max_blocks) nb = max_blocks;
        for (int64_t j = 0; j < nb; ++j) {
            uint32_t r = s * max_blocks + (uint32_t)j;
            int32_t b = table[r];
            k.n_requests++;
            if (b < 0 || (uint32_t)b >= c->n_objects || seq_dst_block[s] + (uint64_t)j >= dst_capacity_blocks) {
                k.n_invalid++;
                continue;
            }
            switch (c->tier[b]) {
            case T_LOCAL: k.n_local++; break;
            case T_CACHE: k.n_cache++; break;
            case T_HOST:  k.n_host++; if (miss_idx) miss_idx[nm] = r; nm++; break;
            default:      k.n_lost++; if (miss_idx) miss_idx[nm] = r; nm++; break;
            }
        }
    }
    /* pass 2: move the bytes; requests are independent */
    long total = (long)n_seq * (long)max_blocks;
#pragma omp parallel for schedule(static) num_threads(threads > 0 ? threads : 1)
    for (long r = 0; r < total; ++r) {
        uint32_t s = (uint32_t)(r / max_blocks), j = (uint32_t)(r % max_blocks);
        int64_t nb = n_blocks[s] < 0 ? 0 : n_blocks[s];
        if ((int64_t)j >= nb) continue;
        int32_t b = table[r];
        if (b < 0 || (uint32_t)b >= c->n_objects || seq_dst_block[s] + j >= dst_capacity_blocks) continue;
        for (uint32_t p = 0; p < c->n_planes; ++p) {
            const uint8_t *src = resolve(c, (uint32_t)b, p, layer);
            if (src) memcpy(dst[p] + (seq_dst_block[s] + j) * c->chunk_bytes, src, c->chunk_bytes);
        }
    }
    if (n_miss) *n_miss = nm;
    if (counts) *counts = k;
    return ORC_OK;
}

/*
 * KV fetch into a head-major working layout (the layout attention kernels that
 * walk one head at a time want; the paper leaves layouts open).  A block in a
 * pool is token-major: [block_tokens][n_heads][head_bytes].  Sequence s owns
 * seq_cap_blocks[s] destination blocks starting at block seq_dst_block[s], laid
 * out [n_heads][seq_cap_blocks[s] * block_tokens][head_bytes]; request (s, j)
 * fills rows j * block_tokens ... of every head strip.  Invalid (skipped and
 * counted): unknown block, j >= seq_cap_blocks[s], or a sequence region that
 * does not fit dst_capacity_blocks.  Everything else as orc_fetch_kv.
 */
int orc_fetch_kv_head_major(orc_class *c, uint32_t layer, const int32_t *table, const int32_t *n_blocks,
                            uint32_t n_seq, uint32_t max_blocks, uint8_t *dst_k, uint8_t *dst_v,
                            const uint64_t *seq_dst_block, const uint32_t *seq_cap_blocks,
                            uint64_t dst_capacity_blocks, uint32_t n_heads, uint32_t block_tokens, uint32_t *miss_idx,
                            uint32_t *n_miss, orc_counts *counts)
{
    if (layer >= c->n_layers || n_heads == 0 || block_tokens == 0) return ORC_EINVAL;
    if (c->chunk_bytes % ((uint64_t)n_heads * block_tokens)) return ORC_EINVAL;
    uint64_t head_bytes = c->chunk_bytes / ((uint64_t)n_heads * block_tokens);
    uint8_t *dst[2] = { dst_k, dst_v };
    orc_counts k = { 0, 0, 0, 0, 0, 0 };
    uint32_t nm = 0;
    for (uint32_t s = 0; s < n_seq; ++s) {
        int64_t nb = n_blocks[s] < 0 ? 0 : n_blocks[s];
        if (nb > (int64_t)max_blocks) nb = max_blocks;
        int fits = seq_dst_block[s] + seq_cap_blocks[s] <= dst_capacity_blocks;
        uint64_t strip = (uint64_t)seq_cap_blocks[s] * block_tokens * head_bytes;       /* one head of this sequence */
        for (int64_t j = 0; j < nb; ++j) {
            uint32_t r = s * max_blocks + (uint32_t)j;
            int32_t b = table[r];
            k.n_requests++;
            if (b < 0 || (uint32_t)b >= c->n_objects || !fits || (uint64_t)j >= seq_cap_blocks[s]) { k.n_invalid++; continue; }
            int t = c->tier[b];
            if (t == T_LOCAL) k.n_local++;
            else if (t == T_CACHE) k.n_cache++;
            else if (t == T_HOST) k.n_host++;
            else k.n_lost++;
            if (t == T_HOST || t == T_NONE) { if (miss_idx) miss_idx[nm] = r; nm++; }
            if (t == T_NONE) continue;
            for (uint32_t p = 0; p < c->n_planes; ++p) {
                const uint8_t *src = resolve(c, (uint32_t)b, p, layer);
                uint8_t *seq_base = dst[p] + seq_dst_block[s] * c->chunk_bytes;
                for (uint32_t tok = 0; tok < block_tokens; ++tok)
                    for (uint32_t h = 0; h < n_heads; ++h)
                        memcpy(seq_base + h * strip + ((uint64_t)j * block_tokens + tok) * head_bytes,
                               src + ((uint64_t)tok * n_heads + h) * head_bytes, head_bytes);
            }
        }
    }
    if (n_miss) *n_miss = nm;
    if (counts) *counts = k;
    return ORC_OK;
}

/* KV fetch, plain definition: every valid request receives the current value of its block. */
int orc_fetch_kv_plain(orc_class *c, uint32_t layer, const int32_t *table, const int32_t *n_blocks, uint32_t n_seq,
                       uint32_t max_blocks, uint8_t *dst_k, uint8_t *dst_v, const uint64_t *seq_dst_block,
                       uint64_t dst_capacity_blocks)
{
    if (layer >= c->n_layers) return ORC_EINVAL;
    uint8_t *dst[2] = { dst_k, dst_v };
    for (uint32_t s = 0; s < n_seq; ++s) {
        int64_t nb = n_blocks[s] < 0 ? 0 : n_blocks[s];
        if (nb > (int64_t)max_blocks) nb = max_blocks;
        for (int64_t j = 0; j < nb; ++j) {
            int32_t b = table[s * max_blocks + j];
            if (b < 0 || (uint32_t)b >= c->n_objects || seq_dst_block[s] + (uint64_t)j >= dst_capacity_blocks) continue;
            if (c->tier[b] == T_NONE) continue;
            for (uint32_t p = 0; p < c->n_planes; ++p)
                memcpy(dst[p] + (seq_dst_block[s] + (uint64_t)j) * c->chunk_bytes,
                       at(c->truth[p], c, c->max_objects, layer, (uint32_t)b), c->chunk_bytes);
        }
    }
    return ORC_OK;
}

/*
 * Expert fetch (Section 4.3: experts are paged whole - the FFN of an expert
 * cannot start before all of its weights are in GPU memory; the residency map
 * says local HBM / peer HBM / host DRAM).
 * Objects of this class are numbered layer * n_experts + e and have one plane
 * and one storage layer.  U = distinct valid ids in topk.  For e in U,
 * ascending: local -> used in place (kind 1, where = local slot, no bytes
 * move); cache/host -> copied into staging slot `rank` = number of earlier
 * staged members (kind 2, where = rank), or kind 3 when staging is full; lost
 * -> kind 4.  Unselected experts: kind 0.  miss_idx lists the experts served
 * from host or lost, ascending.
 */
int orc_fetch_experts(orc_class *c, uint32_t layer, uint32_t n_experts, const int32_t *topk, uint32_t n_tokens,
                      uint32_t k, uint8_t *staging, uint32_t n_staging_slots, int32_t *kind, int64_t *where,
                      uint32_t *miss_idx, uint32_t *n_miss, orc_counts *counts)
{
    if ((uint64_t)(layer + 1) * n_experts > c->n_objects || c->n_planes != 1 || c->n_layers != 1) return ORC_EINVAL;
    orc_counts kc = { 0, 0, 0, 0, 0, 0 };
    uint8_t *sel = (uint8_t *)calloc(n_experts ? n_experts : 1, 1);
    for (uint64_t i = 0; i < (uint64_t)n_tokens * k; ++i) {
        int32_t e = topk[i];
        if (e < 0 || (uint32_t)e >= n_experts) { kc.n_invalid++; continue; }
        sel[e] = 1;
    }
    uint32_t rank = 0, nm = 0;
    for (uint32_t e = 0; e < n_experts; ++e) {
        kind[e] = 0; where[e] = -1;
        if (!sel[e]) continue;
        uint32_t id = layer * n_experts + e;
        kc.n_requests++;
        switch (c->tier[id]) {
        case T_LOCAL:
            kind[e] = 1; where[e] = c->slot[id]; kc.n_local++;
            break;
        case T_CACHE:
        case T_HOST:
            if (rank >= n_staging_slots) { kind[e] = 3; kc.n_invalid++; break; }
            if (c->tier[id] == T_HOST) { kc.n_host++; if (miss_idx) miss_idx[nm] = e; nm++; }
            else kc.n_cache++;
            memcpy(staging + (uint64_t)rank * c->chunk_bytes, resolve(c, id, 0, 0), c->chunk_bytes);
            kind[e] = 2; where[e] = rank++;
            break;
        default:
            kind[e] = 4; kc.n_lost++; if (miss_idx) miss_idx[nm] = e; nm++;
            break;
        }
    }
    free(sel);
    if (n_miss) *n_miss = nm;
    if (counts) *counts = kc;
    return ORC_OK;
}

/*
 * Eviction / write-back (Section 5.2: under memory pressure a worker asks for
 * blocks to be moved out of local HBM; Section 5.1: the copy that counts for
 * spilled KV is the one in host DRAM; Section 3.1: the runtime
 * never writes back on its own, so this explicit call is the only way bytes
 * reach a lower tier).  For each id the source bytes become the object's
 * value: written to its host slot (when backed) and to whichever HBM slot the
 * directory names, so that every copy of the object stays identical.
 *
 * layer >= 0: only that layer; each src plane is [src_layer_stride][chunk].
 * layer  < 0: all layers; each src plane is [n_layers][src_layer_stride][chunk].
 * ORC_EVICT_DEMOTE (all layers only): a local object leaves local HBM - its
 * slot is released.  A backed object then lives on the host; a lossy one
 * (Section 5.2: KV state need not be duplicated in a lower tier)
 * moves into the cache tier instead (lowest free slot, or a best-fit segment)
 * and has no other copy - if the cache tier cannot take all lossy objects of
 * the call, ORC_ENOSPC and nothing changes.
 * Duplicate ids make the write order undefined: rejected, nothing written.
 */
int orc_evict(orc_class *c, int layer, const uint32_t *ids, uint32_t n, const uint8_t *src_k, const uint8_t *src_v,
              const uint64_t *src_block, uint64_t src_layer_stride, int flags)
{
    const uint8_t *src[2] = { src_k, src_v };
    if (layer >= (int)c->n_layers) return ORC_EINVAL;
    if ((flags & ORC_EVICT_DEMOTE) && layer >= 0 && c->n_layers != 1) return ORC_EINVAL;
    uint32_t need_cache = 0;
    for (uint32_t i = 0; i < n; ++i) {
        if (ids[i] >= c->n_objects) return ORC_ENOENT;
        if (src_block[i] >= src_layer_stride) return ORC_EINVAL;
        if (c->tier[ids[i]] == T_NONE) return ORC_ELOST;
        if ((flags & ORC_EVICT_DEMOTE) && c->tier[ids[i]] == T_LOCAL && c->host_slot[ids[i]] < 0) need_cache++;
        for (uint32_t j = 0; j < i; ++j)
            if (ids[j] == ids[i]) return ORC_EINVAL;
    }
    /* room for every lossy object that leaves local HBM, taken in request order; all or nothing */
    int64_t *room = (int64_t *)calloc(need_cache ? need_cache : 1, sizeof(int64_t));
    for (uint32_t k = 0; k < need_cache; ++k) {
        room[k] = cache_take(c);
        if (room[k] < 0) {
            while (k > 0) cache_release(c, room[--k]);
            free(room);
            return ORC_ENOSPC;
        }
    }
    uint32_t n_room = 0;
    uint32_t l0 = layer < 0 ? 0 : (uint32_t)layer, l1 = layer < 0 ? c->n_layers : (uint32_t)layer + 1;
    for (uint32_t i = 0; i < n; ++i) {
        uint32_t id = ids[i];
        int demote = (flags & ORC_EVICT_DEMOTE) && c->tier[id] == T_LOCAL;
        int64_t to_cache = -1;
        if (demote && c->host_slot[id] < 0) to_cache = room[n_room++];
        for (uint32_t p = 0; p < c->n_planes; ++p)
            for (uint32_t l = l0; l < l1; ++l) {
                uint64_t li = layer < 0 ? l : 0;
                const uint8_t *s = src[p] + (li * src_layer_stride + src_block[i]) * c->chunk_bytes;
                /* a source that already is the object's own local slot needs no copy onto itself */
                if (c->host_slot[id] >= 0)
                    memcpy(at(c->host[p], c, c->n_host_slots, l, (uint64_t)c->host_slot[id]), s, c->chunk_bytes);
                if (c->tier[id] == T_CACHE)
                    memcpy(cache_at(c, p, l, (uint64_t)c->slot[id]), s, c->chunk_bytes);
                if (to_cache >= 0)
                    memcpy(cache_at(c, p, l, (uint64_t)to_cache), s, c->chunk_bytes);
                if (c->tier[id] == T_LOCAL && !demote) {
                    uint8_t *d = at(c->local[p], c, c->n_local_slots, l, (uint64_t)c->slot[id]);
                    if (d != s) memmove(d, s, c->chunk_bytes);
                }
                memmove(at(c->truth[p], c, c->max_objects, l, id), s, c->chunk_bytes);
            }
        if (demote) {
            c->local_used[c->slot[id]] = 0;
            if (to_cache >= 0) { c->tier[id] = T_CACHE; c->slot[id] = to_cache; }
            else { c->tier[id] = T_HOST; c->slot[id] = -1; }
            c->gen[id] += 1;
        }
    }
    free(room);
    return ORC_OK;
}

/*
 * Harness initialisation after a bulk fill of the pools: declares the bytes
 * now stored where the directory points (host slot, or local slot) to be the
 * object's value.
 */
int orc_adopt(orc_class *c, uint32_t id)
{
    if (id >= c->n_objects) return ORC_ENOENT;
    if (c->tier[id] != T_HOST && c->tier[id] != T_LOCAL) return ORC_EINVAL;
    for (uint32_t p = 0; p < c->n_planes; ++p)
        for (uint32_t l = 0; l < c->n_layers; ++l)
            memcpy(at(c->truth[p], c, c->max_objects, l, id), resolve(c, id, p, l), c->chunk_bytes);
    return ORC_OK;
}
