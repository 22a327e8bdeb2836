/*
 * Sanitizer run of the host side: the library in HARVEST_FLAG_NO_DEVICE mode (directory, slot and segment allocators -
 * no HIP call is made) and the CPU oracle, both built with -fsanitize=address,undefined, are driven in lock step through
 * long random sequences of every directory operation; the oracle also runs its data paths (fetches, write-backs) on
 * real buffers.  Any status or directory entry that differs, and anything the sanitizers find, ends the run with a
 * non-zero exit status.  Built and run by tests/test_sanitizers.py.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "harvest.h"

/* the oracle's C interface (oracle/harvest_oracle.c) */
typedef struct orc_class orc_class;
typedef struct orc_segpool orc_segpool;
typedef struct { uint64_t n_requests, n_local, n_cache, n_host, n_lost, n_invalid; } orc_counts;
typedef void (*orc_revoke_cb)(uint32_t id, void *user);
orc_segpool *orc_segpool_create(uint64_t bytes, uint64_t granule);
void orc_segpool_destroy(orc_segpool *g);
uint64_t orc_segpool_free_runs(const orc_segpool *g, uint64_t *off, uint64_t *len, uint64_t cap);
orc_class *orc_create(uint32_t n_layers, uint32_t n_planes, uint64_t chunk_bytes, uint32_t max_objects,
                      uint32_t n_host_slots, uint32_t n_cache_slots, uint32_t n_local_slots, int poison);
void orc_destroy(orc_class *c);
int orc_attach_segpool(orc_class *c, orc_segpool *g);
uint8_t *orc_plane(orc_class *c, int which, uint32_t plane);
uint32_t orc_n_objects(const orc_class *c);
int orc_register(orc_class *c, uint32_t n, const int64_t *host_slot, int tier, uint32_t *out_ids);
int orc_restore(orc_class *c, const uint32_t *ids, uint32_t n);
int orc_lookup(const orc_class *c, uint32_t id, int *tier, int64_t *slot, uint32_t *gen, int64_t *host_slot);
int orc_place(orc_class *c, const uint32_t *ids, uint32_t n, int *status);
int orc_revoke(orc_class *c, const uint32_t *ids, uint32_t n, orc_revoke_cb cb, void *user);
int orc_fetch_kv(orc_class *c, uint32_t layer, const int32_t *table, const int32_t *n_blocks, uint32_t n_seq,
                 uint32_t max_blocks, uint8_t *dst_k, uint8_t *dst_v, const uint64_t *seq_dst_block,
                 uint64_t dst_capacity_blocks, uint32_t *miss_idx, uint32_t *n_miss, orc_counts *counts, int threads);
int orc_fetch_kv_head_major(orc_class *c, uint32_t layer, const int32_t *table, const int32_t *n_blocks,
                            uint32_t n_seq, uint32_t max_blocks, uint8_t *dst_k, uint8_t *dst_v,
                            const uint64_t *seq_dst_block, const uint32_t *seq_cap_blocks,
                            uint64_t dst_capacity_blocks, uint32_t n_heads, uint32_t block_tokens, uint32_t *miss_idx,
                            uint32_t *n_miss, orc_counts *counts);
int orc_fetch_experts(orc_class *c, uint32_t layer, uint32_t n_experts, const int32_t *topk, uint32_t n_tokens,
                      uint32_t k, uint8_t *staging, uint32_t n_staging_slots, int32_t *kind, int64_t *where,
                      uint32_t *miss_idx, uint32_t *n_miss, orc_counts *counts);
int orc_evict(orc_class *c, int layer, const uint32_t *ids, uint32_t n, const uint8_t *src_k, const uint8_t *src_v,
              const uint64_t *src_block, uint64_t src_layer_stride, int flags);

/* Only in this build of the library (-DHARVEST_FAULT_INJECTION): the nth device step from now fails like a HIP error.
 * A context without a device walks the same steps as one with a device, so every roll-back path runs here. */
void harvest_test_fail_at(int nth);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(uint32_t n)
{
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return n ? (uint32_t)((rng_state >> 11) % n) : 0;
}

#define FAIL(...) do { fprintf(stderr, __VA_ARGS__); fprintf(stderr, " (run %d step %d)\n", run_no, step_no); exit(1); } while (0)
static int run_no, step_no;

enum { KV_LAYERS = 3, KV_CHUNK = 128, KV_MAX = 48, KV_HOST = 40, KV_LOCAL = 6, EX_E = 8, EX_LAYERS = 3, EX_CHUNK = 1264 };

static int n_cb_lib, n_cb_orc;
static void cb_lib(int cls, harvest_obj id, void *user) { (void)cls; (void)id; (void)user; n_cb_lib++; }
static void cb_orc(uint32_t id, void *user) { (void)id; (void)user; n_cb_orc++; }

static void compare_all(harvest_ctx *h, orc_class *oc[2])
{
    for (int cls = 0; cls < 2; ++cls)
        for (uint32_t i = 0; i < orc_n_objects(oc[cls]); ++i) {
            int t0, t1; int64_t s0, s1, hs0, hs1; uint32_t g0, g1;
            int r0 = orc_lookup(oc[cls], i, &t0, &s0, &g0, &hs0), r1 = harvest_lookup(h, cls, i, &t1, &s1, &g1, &hs1);
            if (r0 || r1 || t0 != t1 || s0 != s1 || g0 != g1 || hs0 != hs1)
                FAIL("class %d object %u: oracle (%d,%lld,%u,%lld) library (%d,%lld,%u,%lld)", cls, i, t0, (long long)s0, g0,
                     (long long)hs0, t1, (long long)s1, g1, (long long)hs1);
        }
    if (n_cb_lib != n_cb_orc) FAIL("callbacks: library %d oracle %d", n_cb_lib, n_cb_orc);
}

static int n_injected, n_rolled_back;

/* r1 = call, about every third time with a fault injected at a random device step first.  A call that reports the
 * injected failure must have changed nothing - directory, callbacks and every statistic are as before - and is then made
 * again for real; a call that ended before the fault was due counts as the real one. */
#define CALL(r1, h, oc, call)                                                                                \
    do {                                                                                                     \
        int done_ = 0;                                                                                       \
        if (rnd(3) == 0) {                                                                                   \
            harvest_stats_t before_, after_;                                                                 \
            if (harvest_stats(h, &before_)) FAIL("stats");                                                   \
            int cb_before_ = n_cb_lib;                                                                       \
            harvest_test_fail_at(1 + (int)rnd(7));                                                           \
            int r_ = (call);                                                                                 \
            harvest_test_fail_at(0);                                                                         \
            n_injected++;                                                                                    \
            if (r_ == HARVEST_EHIP) {                                                                        \
                n_rolled_back++;                                                                             \
                if (harvest_stats(h, &after_)) FAIL("stats");                                                \
                if (memcmp(&before_, &after_, sizeof before_)) FAIL("statistics changed by a call that failed"); \
                if (n_cb_lib != cb_before_) FAIL("a call that failed invoked callbacks");                    \
                compare_all(h, oc);                                                                          \
            } else {                                                                                         \
                r1 = r_;                                                                                     \
                done_ = 1;                                                                                   \
            }                                                                                                \
        }                                                                                                    \
        if (!done_) r1 = (call);                                                                             \
    } while (0)

static void one_run(int shared)
{
    const uint32_t granule = 256;
    const uint64_t pool_bytes = 43ull * granule;
    harvest_config cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.flags = HARVEST_FLAG_NO_DEVICE | HARVEST_FLAG_POISON;
    harvest_class_config *kv = &cfg.cls[HARVEST_KV], *ex = &cfg.cls[HARVEST_EXPERT];
    kv->n_layers = KV_LAYERS; kv->n_planes = 2; kv->chunk_bytes = KV_CHUNK; kv->max_objects = KV_MAX;
    kv->n_host_slots = KV_HOST; kv->n_cache_slots = shared ? 0 : 11; kv->n_local_slots = KV_LOCAL;
    ex->n_layers = 1; ex->n_planes = 1; ex->chunk_bytes = EX_CHUNK; ex->max_objects = EX_E * EX_LAYERS;
    ex->n_host_slots = EX_E * EX_LAYERS; ex->n_cache_slots = shared ? 0 : 7; ex->n_local_slots = 4; ex->n_experts = EX_E;
    if (shared) { cfg.shared_cache_bytes = pool_bytes; cfg.shared_granule = granule; }
    harvest_ctx *h = NULL;
    if (harvest_create(&cfg, &h) != HARVEST_OK) FAIL("harvest_create");
    orc_segpool *pool = shared ? orc_segpool_create(pool_bytes, granule) : NULL;
    orc_class *oc[2];
    oc[0] = orc_create(KV_LAYERS, 2, KV_CHUNK, KV_MAX, KV_HOST, kv->n_cache_slots, KV_LOCAL, 1);
    oc[1] = orc_create(1, 1, EX_CHUNK, ex->max_objects, ex->n_host_slots, ex->n_cache_slots, 4, 1);
    if (shared && (orc_attach_segpool(oc[0], pool) || orc_attach_segpool(oc[1], pool))) FAIL("attach");
    n_cb_lib = n_cb_orc = 0;
    /* experts are registered up front (object number = layer * E + e), a few of them local */
    for (uint32_t i = 0; i < ex->max_objects; ++i) {
        int64_t hs = (int64_t)((i * 7 + 3) % ex->max_objects);
        int tier = (i % 6 == 1) ? HARVEST_LOCAL : HARVEST_HOST;
        uint32_t a, b;
        int r0 = orc_register(oc[1], 1, &hs, tier, &a), r1 = harvest_register(h, HARVEST_EXPERT, 1, &hs, tier, cb_lib, NULL, &b);
        if (r0 != r1 || (r0 == 0 && a != b)) FAIL("expert registration %u: %d %d", i, r0, r1);
    }
    static uint8_t src[KV_LAYERS * 8 * EX_CHUNK];
    for (size_t i = 0; i < sizeof src; ++i) src[i] = (uint8_t)(i * 31 + 7);
    uint32_t kv_host_next = 0;
    for (step_no = 0; step_no < 6000; ++step_no) {
        int cls = rnd(100) < 65 ? HARVEST_KV : HARVEST_EXPERT;
        orc_class *c = oc[cls];
        uint32_t n_obj = orc_n_objects(c);
        uint32_t ids[6], n = 1 + rnd(5);
        for (uint32_t i = 0; i < n; ++i) ids[i] = n_obj ? rnd(n_obj + (rnd(40) == 0)) : 0;
        switch (rnd(7)) {
        case 0: {                                           /* register KV blocks: backed on the host, or lossy local */
            if (cls != HARVEST_KV) break;
            uint32_t a[2] = { 0, 0 }, b[2] = { 0, 0 };
            if (rnd(3) == 0) {
                int r0 = orc_register(c, 1, NULL, HARVEST_LOCAL, a), r1 = harvest_register(h, cls, 1, NULL, HARVEST_LOCAL, cb_lib, NULL, b);
                if (r0 != r1 || (!r0 && a[0] != b[0])) FAIL("lossy registration: %d %d", r0, r1);
            } else {
                int64_t hs[2] = { (int64_t)(kv_host_next % (KV_HOST + 2)), (int64_t)((kv_host_next + 1) % (KV_HOST + 2)) };
                int tier = rnd(4) == 0 ? HARVEST_LOCAL : HARVEST_HOST;
                uint32_t k = 1 + rnd(2);
                int r0 = orc_register(c, k, hs, tier, a), r1 = harvest_register(h, cls, k, hs, tier, cb_lib, NULL, b);
                if (r0 != r1 || (!r0 && (a[0] != b[0] || (k == 2 && a[1] != b[1])))) FAIL("registration: %d %d", r0, r1);
                if (!r0) kv_host_next += k; else kv_host_next += 1;
            }
            break;
        }
        case 1: case 2: {
            if (!n_obj) break;
            int st0[6], st1[6];
            int r1;
            CALL(r1, h, oc, harvest_place(h, cls, ids, n, NULL, st1));
            int r0 = orc_place(c, ids, n, st0);
            if (r0 != r1 || (!r0 && memcmp(st0, st1, n * sizeof(int)))) FAIL("place: %d %d", r0, r1);
            break;
        }
        case 3: {
            if (!n_obj) break;
            int r1;
            CALL(r1, h, oc, harvest_revoke(h, cls, ids, n));
            int r0 = orc_revoke(c, ids, n, cb_orc, NULL);
            if (r0 != r1) FAIL("revoke: %d %d", r0, r1);
            break;
        }
        case 4: {                                           /* write-back, sometimes with demotion, sometimes one layer */
            if (!n_obj) break;
            uint64_t sb[6];
            for (uint32_t i = 0; i < n; ++i) sb[i] = rnd(8 + (rnd(30) == 0));
            int layer = (cls == HARVEST_KV && rnd(2)) ? (int)rnd(KV_LAYERS) : -1;
            int flags = rnd(2) ? HARVEST_EVICT_DEMOTE : 0;
            int r1;
            CALL(r1, h, oc, harvest_evict(h, cls, layer, ids, n, NULL, NULL, sb, 8, flags, NULL));
            int r0 = orc_evict(c, layer, ids, n, src, src + 64, sb, 8, flags);
            if (r0 != r1) FAIL("evict: %d %d", r0, r1);
            break;
        }
        case 5: {
            if (!n_obj) break;
            int r0 = orc_restore(c, ids, n > 2 ? 2 : n), r1 = harvest_restore(h, cls, ids, n > 2 ? 2 : n);
            if (r0 != r1) FAIL("restore: %d %d", r0, r1);
            for (uint32_t i = 0; i < n_obj; ++i) {          /* and one that can succeed */
                int t; int64_t s, hs; uint32_t g;
                orc_lookup(c, i, &t, &s, &g, &hs);
                if (t == HARVEST_NONE) {
                    r0 = orc_restore(c, &i, 1); r1 = harvest_restore(h, cls, &i, 1);
                    if (r0 != r1) FAIL("restore of a lost object: %d %d", r0, r1);
                    break;
                }
            }
            break;
        }
        default: {                                          /* the oracle's data paths on real buffers */
            if (cls == HARVEST_KV && n_obj) {
                int32_t table[3 * 7], nb[3] = { 7, (int32_t)rnd(9) - 1, (int32_t)rnd(8) };
                uint64_t sdb[3] = { 0, 7, 15 };
                uint32_t caps[3] = { 7, 8, 7 };
                for (int i = 0; i < 21; ++i) table[i] = (int32_t)rnd(n_obj + 2) - 1;
                static uint8_t dk[23 * KV_CHUNK], dv[23 * KV_CHUNK];
                uint32_t miss[21], n_miss = 0;
                orc_counts cnt;
                if (orc_fetch_kv(c, rnd(KV_LAYERS), table, nb, 3, 7, dk, dv, sdb, 22 + rnd(2), miss, &n_miss, &cnt, 1 + (int)rnd(3)))
                    FAIL("oracle fetch_kv");
                if (cnt.n_local + cnt.n_cache + cnt.n_host + cnt.n_lost + cnt.n_invalid != cnt.n_requests) FAIL("counts do not add up");
                if (orc_fetch_kv_head_major(c, rnd(KV_LAYERS), table, nb, 3, 7, dk, dv, sdb, caps, 23, 2, 4, miss, &n_miss, &cnt))
                    FAIL("oracle fetch_kv_head_major");
            } else if (cls == HARVEST_EXPERT) {
                int32_t topk[5 * 2];
                for (int i = 0; i < 10; ++i) topk[i] = (int32_t)rnd(EX_E + 2) - 1;
                static uint8_t staging[EX_E * EX_CHUNK];
                int32_t kind[EX_E]; int64_t where[EX_E]; uint32_t miss[EX_E], n_miss = 0;
                orc_counts cnt;
                if (orc_fetch_experts(c, rnd(EX_LAYERS), EX_E, topk, 5, 2, staging, rnd(EX_E + 1), kind, where, miss, &n_miss, &cnt))
                    FAIL("oracle fetch_experts");
            }
            break;
        }
        }
        compare_all(h, oc);
        if (shared && step_no % 16 == 0) {
            uint64_t off[64], len[64], n_runs = orc_segpool_free_runs(pool, off, len, 64), n_free = 0, longest = 0;
            for (uint64_t i = 0; i < n_runs && i < 64; ++i) { n_free += len[i]; if (len[i] > longest) longest = len[i]; }
            harvest_stats_t st;
            if (harvest_stats(h, &st)) FAIL("stats");
            if (st.shared_free_runs != n_runs || st.shared_granules_free != n_free || st.shared_longest_free_run != longest)
                FAIL("free runs: library (%llu,%llu,%llu) oracle (%llu,%llu,%llu)", (unsigned long long)st.shared_free_runs,
                     (unsigned long long)st.shared_granules_free, (unsigned long long)st.shared_longest_free_run,
                     (unsigned long long)n_runs, (unsigned long long)n_free, (unsigned long long)longest);
        }
    }
    harvest_destroy(h);
    orc_destroy(oc[0]); orc_destroy(oc[1]);
    if (pool) orc_segpool_destroy(pool);
}

int main(void)
{
    for (run_no = 0; run_no < 4; ++run_no) one_run(run_no & 1);
    if (n_rolled_back < 1000) { fprintf(stderr, "only %d of %d injected faults were hit\n", n_rolled_back, n_injected); return 1; }
    printf("injected faults rolled back: %d\n", n_rolled_back);
    printf("sanitizer run: ok\n");
    return 0;
}
