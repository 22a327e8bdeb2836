/*
 * The C ABI used from plain C, with no Python and no PyTorch in the process: pools from hipMalloc and
 * harvest_pinned_alloc, a block table in device memory, and one round of the path - register, place, fetch, revoke,
 * fetch again (now from the host copies), write new bytes back, fetch them, and fetch them once more through the entry
 * point that allocates nothing.  Every fetched byte is checked on the host against the pattern its block was filled with.  Prints "kv_fetch example: ok" and exits 0 when all of it holds.
 *
 *   hipcc -x hip --offload-arch=gfx950 -I include paper_2602_00328_amd/examples/kv_fetch.c -x none \
 *         -o paper_2602_00328_amd/examples/kv_fetch -L paper_2602_00328_amd -l:libharvest.so -Wl,-rpath,'$ORIGIN/..'
 */
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "harvest.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 1; } } while (0)
#define CHECK(x) do { int rc_ = (x); if (rc_ != HARVEST_OK) { fprintf(stderr, "%s: %s\n", #x, harvest_strerror(rc_)); return 1; } } while (0)

enum { LAYERS = 3, CHUNK = 32768, N_OBJ = 96, N_CACHE = 40, N_SEQ = 2, MAX_BLOCKS = 40 };

/* the byte at `off` of block `obj`, plane `p`, layer `l`, version `ver` */
static uint8_t pattern(uint32_t obj, uint32_t p, uint32_t l, uint32_t off, uint32_t ver)
{
    return (uint8_t)(obj * 131u + p * 17u + l * 29u + off * 7u + (off >> 8) + ver * 101u);
}

static int n_callbacks;
static void on_revoke(int cls, harvest_obj id, void *user) { (void)cls; (void)id; (void)user; n_callbacks++; }

static int verify(const uint8_t *k, const uint8_t *v, const int32_t *table, const int32_t *nb, const uint64_t *first,
                  uint32_t layer, const uint32_t *version, const char *what)
{
    for (int s = 0; s < N_SEQ; ++s)
        for (int j = 0; j < nb[s]; ++j) {
            uint32_t obj = (uint32_t)table[s * MAX_BLOCKS + j];
            const uint8_t *pk = k + (first[s] + j) * CHUNK, *pv = v + (first[s] + j) * CHUNK;
            for (uint32_t off = 0; off < CHUNK; ++off)
                if (pk[off] != pattern(obj, 0, layer, off, version[obj]) || pv[off] != pattern(obj, 1, layer, off, version[obj])) {
                    fprintf(stderr, "%s: sequence %d block %d (object %u) byte %u differs\n", what, s, j, obj, off);
                    return 1;
                }
        }
    return 0;
}

int main(void)
{
    CHECK_HIP(hipSetDevice(0));
    harvest_config cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.flags = HARVEST_FLAG_POISON;
    harvest_class_config *kv = &cfg.cls[HARVEST_KV];
    kv->n_layers = LAYERS; kv->n_planes = 2; kv->chunk_bytes = CHUNK; kv->max_objects = N_OBJ;
    kv->n_host_slots = N_OBJ; kv->n_cache_slots = N_CACHE; kv->n_local_slots = 0;
    size_t host_bytes = (size_t)LAYERS * N_OBJ * CHUNK, cache_bytes = (size_t)LAYERS * N_CACHE * CHUNK;
    for (int p = 0; p < 2; ++p) {
        kv->host_pool[p] = harvest_pinned_alloc(host_bytes);
        if (!kv->host_pool[p]) return 1;
        CHECK_HIP(hipMalloc(&kv->d_cache_pool[p], cache_bytes));
        CHECK_HIP(hipMemset(kv->d_cache_pool[p], 0, cache_bytes));
    }
    harvest_ctx *h = NULL;
    CHECK(harvest_create(&cfg, &h));

    /* objects 0..N_OBJ-1 with host slots in a scrambled order; every host chunk gets its block's pattern */
    int64_t host_slot[N_OBJ];
    uint32_t version[N_OBJ];
    for (uint32_t i = 0; i < N_OBJ; ++i) { host_slot[i] = (int64_t)((i * 37u + 11u) % N_OBJ); version[i] = 0; }
    harvest_obj ids[N_OBJ];
    CHECK(harvest_register(h, HARVEST_KV, N_OBJ, host_slot, HARVEST_HOST, on_revoke, NULL, ids));
    for (uint32_t i = 0; i < N_OBJ; ++i)
        for (uint32_t p = 0; p < 2; ++p)
            for (uint32_t l = 0; l < LAYERS; ++l) {
                uint8_t *c = (uint8_t *)kv->host_pool[p] + ((size_t)l * N_OBJ + (size_t)host_slot[i]) * CHUNK;
                for (uint32_t off = 0; off < CHUNK; ++off) c[off] = pattern(i, p, l, off, 0);
            }
    /* every other object moves into the cache tier, until it is full */
    harvest_obj want[N_OBJ / 2];
    int status[N_OBJ / 2], n_placed = 0, n_full = 0;
    for (uint32_t i = 0; i < N_OBJ / 2; ++i) want[i] = 2 * i;
    CHECK(harvest_place(h, HARVEST_KV, want, N_OBJ / 2, NULL, status));
    for (uint32_t i = 0; i < N_OBJ / 2; ++i) { n_placed += status[i] == HARVEST_OK; n_full += status[i] == HARVEST_ENOSPC; }
    if (n_placed != N_CACHE || n_full != N_OBJ / 2 - N_CACHE) { fprintf(stderr, "placement: %d placed, %d refused\n", n_placed, n_full); return 1; }

    /* two sequences: 40 and 33 blocks, any objects, some twice */
    int32_t table[N_SEQ * MAX_BLOCKS], nb[N_SEQ] = { 40, 33 };
    uint64_t first[N_SEQ] = { 0, 41 };
    const uint64_t cap = 41 + 33;
    for (int i = 0; i < N_SEQ * MAX_BLOCKS; ++i) table[i] = (int32_t)((i * 53u + 5u) % N_OBJ);
    int32_t *d_table, *d_nb; uint64_t *d_first; uint8_t *d_k, *d_v;
    CHECK_HIP(hipMalloc(&d_table, sizeof table)); CHECK_HIP(hipMemcpy(d_table, table, sizeof table, hipMemcpyHostToDevice));
    CHECK_HIP(hipMalloc(&d_nb, sizeof nb)); CHECK_HIP(hipMemcpy(d_nb, nb, sizeof nb, hipMemcpyHostToDevice));
    CHECK_HIP(hipMalloc(&d_first, sizeof first)); CHECK_HIP(hipMemcpy(d_first, first, sizeof first, hipMemcpyHostToDevice));
    CHECK_HIP(hipMalloc(&d_k, cap * CHUNK)); CHECK_HIP(hipMalloc(&d_v, cap * CHUNK));
    uint8_t *k = (uint8_t *)malloc(cap * CHUNK), *v = (uint8_t *)malloc(cap * CHUNK);
    hipStream_t stream;
    CHECK_HIP(hipStreamCreate(&stream));
    harvest_fetch_counts counts;
    uint32_t n_miss = 0;

    for (uint32_t layer = 0; layer < LAYERS; ++layer) {
        CHECK(harvest_fetch_kv(h, layer, d_table, d_nb, N_SEQ, MAX_BLOCKS, d_k, d_v, d_first, cap, stream));
        CHECK(harvest_fetch_info(h, stream, &counts, NULL, 0, &n_miss));
        CHECK_HIP(hipMemcpy(k, d_k, cap * CHUNK, hipMemcpyDeviceToHost)); CHECK_HIP(hipMemcpy(v, d_v, cap * CHUNK, hipMemcpyDeviceToHost));
        if (verify(k, v, table, nb, first, layer, version, "first fetch")) return 1;
        if (counts.n_requests != 73 || counts.n_cache + counts.n_host != 73 || counts.n_cache == 0 || n_miss != counts.n_host) {
            fprintf(stderr, "counts: %llu requests, %llu cache, %llu host, %u misses\n", (unsigned long long)counts.n_requests,
                    (unsigned long long)counts.n_cache, (unsigned long long)counts.n_host, n_miss);
            return 1;
        }
    }
    uint64_t cache_before = counts.n_cache;
    /* the cache tier loses a third of what it holds: the same bytes must come from the host copies now */
    harvest_obj gone[N_OBJ];
    uint32_t n_gone = 0;
    for (uint32_t i = 0; i < N_OBJ; i += 6) gone[n_gone++] = i;
    CHECK(harvest_revoke(h, HARVEST_KV, gone, n_gone));
    CHECK(harvest_fetch_kv(h, 1, d_table, d_nb, N_SEQ, MAX_BLOCKS, d_k, d_v, d_first, cap, stream));
    CHECK(harvest_fetch_info(h, stream, &counts, NULL, 0, &n_miss));
    CHECK_HIP(hipMemcpy(k, d_k, cap * CHUNK, hipMemcpyDeviceToHost)); CHECK_HIP(hipMemcpy(v, d_v, cap * CHUNK, hipMemcpyDeviceToHost));
    if (verify(k, v, table, nb, first, 1, version, "after revocation")) return 1;
    if (counts.n_cache >= cache_before || n_callbacks == 0) { fprintf(stderr, "revocation changed nothing\n"); return 1; }

    /* new bytes for the blocks of sequence 1's first ten requests, written back from the working layout */
    harvest_obj wb[10];
    uint64_t wb_block[10];
    uint32_t n_wb = 0;
    for (int j = 0; j < 10; ++j) {
        uint32_t obj = (uint32_t)table[1 * MAX_BLOCKS + j];
        int seen = 0;
        for (uint32_t q = 0; q < n_wb; ++q) seen |= wb[q] == obj;
        if (seen) continue;
        wb[n_wb] = obj; wb_block[n_wb] = first[1] + j; n_wb++;
        version[obj] = 1;
        for (uint32_t off = 0; off < CHUNK; ++off) {
            k[(first[1] + j) * CHUNK + off] = pattern(obj, 0, 2, off, 1);
            v[(first[1] + j) * CHUNK + off] = pattern(obj, 1, 2, off, 1);
        }
    }
    CHECK_HIP(hipMemcpy(d_k, k, cap * CHUNK, hipMemcpyHostToDevice)); CHECK_HIP(hipMemcpy(d_v, v, cap * CHUNK, hipMemcpyHostToDevice));
    CHECK(harvest_evict(h, HARVEST_KV, 2, wb, n_wb, d_k, d_v, wb_block, cap, 0, stream));
    CHECK_HIP(hipMemsetAsync(d_k, 0, cap * CHUNK, stream)); CHECK_HIP(hipMemsetAsync(d_v, 0, cap * CHUNK, stream));
    CHECK(harvest_fetch_kv(h, 2, d_table, d_nb, N_SEQ, MAX_BLOCKS, d_k, d_v, d_first, cap, stream));
    CHECK_HIP(hipStreamSynchronize(stream));
    CHECK_HIP(hipMemcpy(k, d_k, cap * CHUNK, hipMemcpyDeviceToHost)); CHECK_HIP(hipMemcpy(v, d_v, cap * CHUNK, hipMemcpyDeviceToHost));
    if (verify(k, v, table, nb, first, 2, version, "after the write-back")) return 1;

    /* the same fetch through the entry point that allocates nothing, on a stream the library has never seen: same bytes,
     * same counts; free device memory is the same after the call as before it */
    {
        hipStream_t fresh;
        CHECK_HIP(hipStreamCreate(&fresh));
        uint8_t *d_k2, *d_v2; uint32_t *d_info, *d_miss, info[8];
        CHECK_HIP(hipMalloc(&d_k2, cap * CHUNK)); CHECK_HIP(hipMalloc(&d_v2, cap * CHUNK));
        CHECK_HIP(hipMalloc(&d_info, sizeof info)); CHECK_HIP(hipMalloc(&d_miss, N_SEQ * MAX_BLOCKS * sizeof(uint32_t)));
        CHECK_HIP(hipMemset(d_k2, 0, cap * CHUNK)); CHECK_HIP(hipMemset(d_v2, 0, cap * CHUNK));
        CHECK_HIP(hipDeviceSynchronize());
        size_t free_before = 0, free_after = 0, total = 0;
        CHECK_HIP(hipMemGetInfo(&free_before, &total));
        CHECK(harvest_fetch_kv_static(h, 2, d_table, d_nb, N_SEQ, MAX_BLOCKS, d_k2, d_v2, d_first, cap, d_info, d_miss, fresh));
        CHECK_HIP(hipStreamSynchronize(fresh));
        CHECK_HIP(hipMemGetInfo(&free_after, &total));
        if (free_after != free_before) { fprintf(stderr, "harvest_fetch_kv_static changed the free device memory\n"); return 1; }
        CHECK(harvest_fetch_info(h, stream, &counts, NULL, 0, &n_miss));          /* of the fetch above, on `stream` */
        CHECK_HIP(hipMemcpy(info, d_info, sizeof info, hipMemcpyDeviceToHost));
        uint8_t *k2 = (uint8_t *)malloc(cap * CHUNK), *v2 = (uint8_t *)malloc(cap * CHUNK);
        CHECK_HIP(hipMemcpy(k2, d_k2, cap * CHUNK, hipMemcpyDeviceToHost)); CHECK_HIP(hipMemcpy(v2, d_v2, cap * CHUNK, hipMemcpyDeviceToHost));
        if (verify(k2, v2, table, nb, first, 2, version, "the fetch that allocates nothing")) return 1;
        if (info[0] != counts.n_requests || info[2] != counts.n_cache || info[3] != counts.n_host || info[6] != n_miss) {
            fprintf(stderr, "harvest_fetch_kv_static counted %u requests, %u cache, %u host, %u misses\n", info[0], info[2], info[3], info[6]);
            return 1;
        }
        if (harvest_fetch_kv_static(h, 2, d_table, d_nb, 4096, 4096, d_k2, d_v2, d_first, cap, NULL, NULL, fresh) != HARVEST_E2BIG) {
            fprintf(stderr, "a table beyond the fixed scratch was not refused\n");
            return 1;
        }
        free(k2); free(v2);
        CHECK_HIP(hipFree(d_k2)); CHECK_HIP(hipFree(d_v2)); CHECK_HIP(hipFree(d_info)); CHECK_HIP(hipFree(d_miss));
        CHECK_HIP(hipStreamDestroy(fresh));
    }

    harvest_stats_t st;
    CHECK(harvest_stats(h, &st));
    printf("kv_fetch example: ok (%llu requests served: %llu from the cache tier, %llu from the host; %llu revoked)\n",
           (unsigned long long)st.fetch[HARVEST_KV].n_requests, (unsigned long long)st.fetch[HARVEST_KV].n_cache,
           (unsigned long long)st.fetch[HARVEST_KV].n_host, (unsigned long long)st.n_revoked[HARVEST_KV]);
    CHECK(harvest_destroy(h));
    for (int p = 0; p < 2; ++p) { harvest_pinned_free(kv->host_pool[p]); CHECK_HIP(hipFree(kv->d_cache_pool[p])); }
    free(k); free(v);
    return 0;
}
