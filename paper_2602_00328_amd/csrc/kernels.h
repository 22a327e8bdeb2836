// Device code of the tiered cache fetch for gfx950 (CDNA4, wave64).
//
// Everything here is byte movement plus a few integers of metadata: no floating point, no MFMA.  The kernels are
//   resolve_kv / resolve_experts : directory lookup (paper Section 5.2 block table, Section 4.3 residency map),
//                                  classification by tier, wave-level compaction into an HBM list and a host
//                                  (miss) list;
//   copy_items                   : the gather itself.  HBM tier: one workgroup per 4 KiB tile, one 16-byte
//                                  non-temporal load and store per thread, as many workgroups as tiles (measured
//                                  on MI355X: many short workgroups beat deep unrolling and persistent grids by
//                                  ~15%).  Host tier: a few persistent workgroups with 8 loads in flight per
//                                  thread, enough to keep the PCIe link full while leaving the CUs to the HBM tier;
//   copy_items2                  : the scatter of the write-back path (one source, up to two destinations);
//   fill_items, dir_write        : slot poisoning after revocation, directory publication.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hv {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int WG = 256;                         // 4 wavefronts
constexpr uint32_t TILE_HBM = WG * 16;          // 4 KiB: one 16-byte access per thread
constexpr int UNROLL_HOST = 8;
constexpr uint32_t TILE_HOST = WG * 16 * UNROLL_HOST;   // 32 KiB: 8 accesses in flight per thread over PCIe

// directory entry: [1:0] tier, [31:2] slot in that tier (host slot for HOST), [63:32] generation
constexpr uint64_t TIER_MASK = 3;
__host__ __device__ inline uint32_t entry_tier(uint64_t e) { return (uint32_t)(e & TIER_MASK); }
__host__ __device__ inline uint32_t entry_slot(uint64_t e) { return (uint32_t)(e >> 2) & 0x3FFFFFFFu; }
__host__ __device__ inline uint64_t make_entry(uint32_t tier, uint32_t slot, uint32_t gen)
{
    return (uint64_t)tier | ((uint64_t)(slot & 0x3FFFFFFFu) << 2) | ((uint64_t)gen << 32);
}
enum { T_HOST = 0, T_CACHE = 1, T_LOCAL = 2, T_NONE = 3 };

struct Item { uint64_t src, dst; };
struct Item2 { uint64_t src, dst0, dst1, pad; };

// per-fetch counters (uint32) and running totals (uint64) share these indices
enum { C_REQ = 0, C_LOCAL, C_CACHE, C_HOST, C_LOST, C_INVALID, C_HBM_REQ, C_HOST_REQ, C_MISS, C_N = 16 };

struct ClassDev {
    const uint64_t *dir;
    uint32_t n_objects, n_planes;
    uint64_t chunk_bytes;
    uint64_t pool[3][2];      // [tier HOST/CACHE/LOCAL][plane] base address as the GPU sees it
    uint32_t n_slots[3];
    uint32_t pad;
};

__device__ inline uint32_t lane_id() { return __lane_id(); }

// Selects instead of indexing: a variable index into a kernel-argument struct would send it to scratch memory.
__device__ inline uint64_t pool_of(const ClassDev &c, int tier, uint32_t plane)
{
    uint64_t h = plane ? c.pool[T_HOST][1] : c.pool[T_HOST][0];
    uint64_t k = plane ? c.pool[T_CACHE][1] : c.pool[T_CACHE][0];
    uint64_t l = plane ? c.pool[T_LOCAL][1] : c.pool[T_LOCAL][0];
    return tier == T_HOST ? h : (tier == T_CACHE ? k : l);
}
__device__ inline uint32_t slots_of(const ClassDev &c, int tier)
{
    return tier == T_HOST ? c.n_slots[T_HOST] : (tier == T_CACHE ? c.n_slots[T_CACHE] : c.n_slots[T_LOCAL]);
}

// Exclusive rank of this lane among the lanes of its wavefront for which pred holds, and the wave total.
__device__ inline uint32_t wave_rank(bool pred, uint32_t &total)
{
    unsigned long long m = __ballot(pred);
    total = (uint32_t)__popcll(m);
    return (uint32_t)__popcll(m & ((1ull << lane_id()) - 1ull));
}

// One atomic per wavefront reserves `total` consecutive list positions; every lane learns the base.
__device__ inline uint32_t wave_reserve(uint32_t *counter, uint32_t total)
{
    uint32_t base = 0;
    if (lane_id() == 0 && total) base = atomicAdd(counter, total);
    return __shfl(base, 0);
}

__device__ inline void wave_count(bool pred, uint32_t *cnt, unsigned long long *totals, int which)
{
    uint32_t n = (uint32_t)__popcll(__ballot(pred));
    if (lane_id() == 0 && n) {
        atomicAdd(&cnt[which], n);
        atomicAdd(&totals[which], (unsigned long long)n);
    }
}

// ---------------------------------------------------------------------------------------------------------
// KV: one thread per (sequence, block-table column).
// ---------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(WG) void resolve_kv(ClassDev c, uint32_t layer, const int32_t *__restrict__ table,
                                                 const int32_t *__restrict__ n_blocks, uint32_t n_seq,
                                                 uint32_t max_blocks, uint64_t dst_k, uint64_t dst_v,
                                                 const uint64_t *__restrict__ seq_dst_block, uint64_t dst_cap,
                                                 Item *__restrict__ hbm_items, Item *__restrict__ host_items,
                                                 uint32_t *__restrict__ miss_idx, uint32_t *cnt, uint32_t *cnt_next,
                                                 unsigned long long *totals)
{
    uint32_t r = blockIdx.x * WG + threadIdx.x;
    if (blockIdx.x == 0 && threadIdx.x < C_N) cnt_next[threadIdx.x] = 0;   // the counters of the NEXT fetch
    uint32_t total = n_seq * max_blocks;
    int tier = -1;                       // -1 no request, 0..3 tier, 4 invalid
    uint64_t src_chunk = 0, dst_chunk = 0;
    if (r < total) {
        uint32_t s = r / max_blocks, j = r - s * max_blocks;
        int32_t nb = n_blocks[s];
        nb = nb < 0 ? 0 : (nb > (int32_t)max_blocks ? (int32_t)max_blocks : nb);
        if (j < (uint32_t)nb) {
            int32_t b = table[r];
            dst_chunk = seq_dst_block[s] + j;
            if (b < 0 || (uint32_t)b >= c.n_objects || dst_chunk >= dst_cap) {
                tier = 4;
            } else {
                uint64_t e = c.dir[b];
                tier = (int)entry_tier(e);
                uint32_t slot = entry_slot(e);
                if (tier != T_NONE) {
                    if (slot >= slots_of(c, tier)) tier = 4;        // never true for a directory the library wrote
                    else src_chunk = (uint64_t)layer * slots_of(c, tier) + slot;
                }
            }
        }
    }
    bool is_hbm = tier == T_LOCAL || tier == T_CACHE;
    bool is_host = tier == T_HOST;
    bool is_miss = tier == T_HOST || tier == T_NONE;
    uint32_t n_hbm, n_host, n_miss;
    uint32_t p_hbm = wave_rank(is_hbm, n_hbm);
    uint32_t p_host = wave_rank(is_host, n_host);
    uint32_t p_miss = wave_rank(is_miss, n_miss);
    p_hbm += wave_reserve(&cnt[C_HBM_REQ], n_hbm);
    p_host += wave_reserve(&cnt[C_HOST_REQ], n_host);
    p_miss += wave_reserve(&cnt[C_MISS], n_miss);
    if (is_hbm || is_host) {
        Item *list = is_hbm ? hbm_items : host_items;
        uint32_t pos = is_hbm ? p_hbm : p_host;
        for (uint32_t p = 0; p < c.n_planes; ++p) {
            Item it;
            it.src = pool_of(c, tier, p) + src_chunk * c.chunk_bytes;
            it.dst = (p ? dst_v : dst_k) + dst_chunk * c.chunk_bytes;
            list[(uint64_t)pos * c.n_planes + p] = it;
        }
    }
    if (is_miss) miss_idx[p_miss] = r;
    wave_count(tier >= 0, cnt, totals, C_REQ);
    wave_count(tier == T_LOCAL, cnt, totals, C_LOCAL);
    wave_count(tier == T_CACHE, cnt, totals, C_CACHE);
    wave_count(tier == T_HOST, cnt, totals, C_HOST);
    wave_count(tier == T_NONE, cnt, totals, C_LOST);
    wave_count(tier == 4, cnt, totals, C_INVALID);
}

// ---------------------------------------------------------------------------------------------------------
// Experts: one workgroup forms the distinct set of the routed expert numbers (bitmap in LDS), then walks the
// experts in ascending order so that staging ranks are the ranks among the staged members of the set.
// ---------------------------------------------------------------------------------------------------------
constexpr uint32_t MAX_EXPERTS = 8192;

__global__ __launch_bounds__(WG) void resolve_experts(ClassDev c, uint32_t layer, uint32_t n_experts,
                                                      const int32_t *__restrict__ topk, uint32_t n_ids,
                                                      uint64_t staging, uint32_t n_staging,
                                                      uint64_t *__restrict__ expert_ptr, Item *__restrict__ hbm_items,
                                                      Item *__restrict__ host_items, uint32_t *__restrict__ miss_idx,
                                                      uint32_t *cnt, uint32_t *cnt_next, unsigned long long *totals)
{
    __shared__ uint32_t bitmap[MAX_EXPERTS / 32];
    __shared__ uint32_t s_cnt[C_N];
    __shared__ uint32_t wave_tot[WG / 64];
    __shared__ uint32_t running;
    uint32_t tid = threadIdx.x;
    for (uint32_t i = tid; i < MAX_EXPERTS / 32; i += WG) bitmap[i] = 0;
    if (tid < C_N) { s_cnt[tid] = 0; cnt_next[tid] = 0; }
    if (tid == 0) running = 0;
    __syncthreads();
    for (uint32_t i = tid; i < n_ids; i += WG) {
        int32_t e = topk[i];
        if (e < 0 || (uint32_t)e >= n_experts) atomicAdd(&s_cnt[C_INVALID], 1u);
        else atomicOr(&bitmap[e >> 5], 1u << (e & 31));
    }
    __syncthreads();
    for (uint32_t base = 0; base < n_experts; base += WG) {
        uint32_t e = base + tid;
        bool sel = e < n_experts && ((bitmap[e >> 5] >> (e & 31)) & 1u);
        int tier = -1;
        uint32_t slot = 0;
        if (sel) {
            uint64_t id = (uint64_t)layer * n_experts + e;
            if (id >= c.n_objects) tier = 4;
            else {
                uint64_t en = c.dir[id];
                tier = (int)entry_tier(en);
                slot = entry_slot(en);
                if (tier != T_NONE && slot >= slots_of(c, tier)) tier = 4;
            }
        }
        bool staged = tier == T_CACHE || tier == T_HOST;
        uint32_t wtot;
        uint32_t rank = wave_rank(staged, wtot);
        if (lane_id() == 0) wave_tot[tid >> 6] = wtot;
        __syncthreads();
        uint32_t before = running;
        for (uint32_t w = 0; w < (tid >> 6); ++w) before += wave_tot[w];
        rank += before;
        uint64_t ptr = 0;
        if (sel) {
            atomicAdd(&s_cnt[C_REQ], 1u);
            if (tier == T_LOCAL) {
                ptr = c.pool[T_LOCAL][0] + (uint64_t)slot * c.chunk_bytes;
                atomicAdd(&s_cnt[C_LOCAL], 1u);
            } else if (staged) {
                if (rank >= n_staging) {
                    atomicAdd(&s_cnt[C_INVALID], 1u);
                } else {
                    ptr = staging + (uint64_t)rank * c.chunk_bytes;
                    Item it;
                    it.src = pool_of(c, tier, 0) + (uint64_t)slot * c.chunk_bytes;
                    it.dst = ptr;
                    if (tier == T_CACHE) {
                        hbm_items[atomicAdd(&s_cnt[C_HBM_REQ], 1u)] = it;
                        atomicAdd(&s_cnt[C_CACHE], 1u);
                    } else {
                        host_items[atomicAdd(&s_cnt[C_HOST_REQ], 1u)] = it;
                        miss_idx[atomicAdd(&s_cnt[C_MISS], 1u)] = e;
                        atomicAdd(&s_cnt[C_HOST], 1u);
                    }
                }
            } else if (tier == T_NONE) {
                miss_idx[atomicAdd(&s_cnt[C_MISS], 1u)] = e;
                atomicAdd(&s_cnt[C_LOST], 1u);
            } else {
                atomicAdd(&s_cnt[C_INVALID], 1u);
            }
        }
        if (e < n_experts) expert_ptr[e] = ptr;
        __syncthreads();
        if (tid == 0) {
            uint32_t t = 0;
            for (uint32_t w = 0; w < WG / 64; ++w) t += wave_tot[w];
            running += t;
        }
        __syncthreads();
    }
    if (tid < C_N) {
        cnt[tid] = s_cnt[tid];
        if (tid <= C_INVALID && s_cnt[tid]) atomicAdd(&totals[tid], (unsigned long long)s_cnt[tid]);
    }
}

// ---------------------------------------------------------------------------------------------------------
// The gather: persistent workgroups walk the tiles of a list of (src, dst) chunks.
// ---------------------------------------------------------------------------------------------------------
template <bool NT>
__device__ inline u32x4 ld16(const u32x4 *p)
{
    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}
template <bool NT>
__device__ inline void st16(u32x4 *p, u32x4 v)
{
    if (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

template <int UNROLL, bool NT>
__device__ inline void copy_tile(uint64_t src, uint64_t dst, uint64_t len, uint32_t tid)
{
    constexpr uint32_t TILE = WG * 16 * UNROLL;
    const u32x4 *s = reinterpret_cast<const u32x4 *>(src);
    u32x4 *d = reinterpret_cast<u32x4 *>(dst);
    if (len >= TILE) {
        u32x4 v[UNROLL];
#pragma unroll
        for (int i = 0; i < UNROLL; ++i) v[i] = ld16<NT>(s + tid + i * WG);
#pragma unroll
        for (int i = 0; i < UNROLL; ++i) st16<NT>(d + tid + i * WG, v[i]);
    } else {
        uint32_t n_vec = (uint32_t)(len >> 4);
        for (uint32_t i = tid; i < n_vec; i += WG) st16<NT>(d + i, ld16<NT>(s + i));
    }
}

// Tiles of a list of (src, dst) chunks; n_req = *n_req_ptr when given (a count produced on the device), else
// n_req_val.  The grid may be any size: with one workgroup per tile the loop body runs once.  `feedback`, when given,
// is a word of pinned host memory that receives n_req: the host sizes the next launch's grid from it, because
// workgroups that find no tile are not free (about 0.2 ns each on MI355X).
template <int UNROLL, bool NT>
__global__ __launch_bounds__(WG) void copy_items(const Item *__restrict__ items, const uint32_t *n_req_ptr,
                                                 uint32_t n_req_val, uint32_t items_per_req, uint64_t chunk_bytes,
                                                 uint32_t tiles_per_chunk, uint32_t *feedback)
{
    constexpr uint32_t TILE = WG * 16 * UNROLL;
    // The first tile's list entry is fetched before the count is known, so that the two scalar loads overlap: a
    // workgroup lives for one load and one store, and every dependent load in front of them costs bandwidth.  The
    // host never launches more workgroups than the list has room for, so the early read stays inside the list.
    uint64_t t = blockIdx.x;
    uint64_t it = t / tiles_per_chunk;
    Item x = items[it];
    uint64_t n_req = n_req_ptr ? *n_req_ptr : n_req_val;
    if (feedback && blockIdx.x == 0 && threadIdx.x == 0) *feedback = (uint32_t)n_req;
    uint64_t n_tiles = n_req * items_per_req * tiles_per_chunk;
    while (t < n_tiles) {
        uint64_t off = (t - it * tiles_per_chunk) * TILE;
        copy_tile<UNROLL, NT>(x.src + off, x.dst + off, chunk_bytes - off, threadIdx.x);
        t += gridDim.x;
        if (t >= n_tiles) break;
        it = t / tiles_per_chunk;
        x = items[it];
    }
}

// One source, one or two destinations (dst == 0: none): the write-back path reads each source byte once.
__global__ __launch_bounds__(WG) void copy_items2(const Item2 *__restrict__ items, uint32_t n_items,
                                                  uint64_t chunk_bytes, uint32_t tiles_per_chunk)
{
    constexpr uint32_t TILE = TILE_HOST;
    uint64_t n_tiles = (uint64_t)n_items * tiles_per_chunk;
    for (uint64_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        uint64_t it = t / tiles_per_chunk;
        uint64_t off = (t - it * tiles_per_chunk) * TILE;
        Item2 x = items[it];
        uint64_t len = chunk_bytes - off;
        if (len > TILE) len = TILE;
        const u32x4 *s = reinterpret_cast<const u32x4 *>(x.src + off);
        u32x4 *d0 = reinterpret_cast<u32x4 *>(x.dst0 + off);
        u32x4 *d1 = reinterpret_cast<u32x4 *>(x.dst1 + off);
        uint32_t n_vec = (uint32_t)(len >> 4);
        for (uint32_t i = threadIdx.x; i < n_vec; i += WG) {
            u32x4 v = s[i];
            if (x.dst0) d0[i] = v;
            if (x.dst1) d1[i] = v;
        }
    }
}

__global__ __launch_bounds__(WG) void fill_items(const Item *__restrict__ items, uint32_t n_items, uint64_t chunk_bytes,
                                                 uint32_t tiles_per_chunk, uint32_t pattern)
{
    constexpr uint32_t TILE = TILE_HOST;
    uint64_t n_tiles = (uint64_t)n_items * tiles_per_chunk;
    u32x4 v = { pattern, pattern, pattern, pattern };
    for (uint64_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        uint64_t it = t / tiles_per_chunk;
        uint64_t off = (t - it * tiles_per_chunk) * TILE;
        uint64_t len = chunk_bytes - off;
        if (len > TILE) len = TILE;
        u32x4 *d = reinterpret_cast<u32x4 *>(items[it].dst + off);
        uint32_t n_vec = (uint32_t)(len >> 4);
        for (uint32_t i = threadIdx.x; i < n_vec; i += WG) d[i] = v;
    }
}

__global__ __launch_bounds__(WG) void dir_write(uint64_t *dir, const uint32_t *__restrict__ ids,
                                                const uint64_t *__restrict__ entries, uint32_t n)
{
    uint32_t i = blockIdx.x * WG + threadIdx.x;
    if (i < n) dir[ids[i]] = entries[i];
}

// Plain contiguous copy with the HBM-tier inner loop (reference ceiling / counter calibration).
__global__ __launch_bounds__(WG) void plain_copy(uint64_t dst, uint64_t src, uint64_t bytes)
{
    uint64_t n_tiles = (bytes + TILE_HBM - 1) / TILE_HBM;
    for (uint64_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        uint64_t off = t * TILE_HBM;
        copy_tile<1, true>(src + off, dst + off, bytes - off, threadIdx.x);
    }
}

}  // namespace hv
