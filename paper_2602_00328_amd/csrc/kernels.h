// Device code of the tiered cache fetch for gfx950 (CDNA4, wave64).
//
// Everything here is byte movement plus a few integers of metadata: no floating point, no MFMA.
//
//   classify_kv + compact_kv : directory lookup (paper Section 5.2: the extended KV block table), classification of
//                              every request by tier, and an ORDER-PRESERVING compaction into an HBM list and a host
//                              (miss) list: wavefront ballots rank the lanes, LDS carries the wave totals, and the
//                              workgroup totals of the first kernel become the offsets of the second.  Keeping the
//                              lists in request order makes the gather's writes one ascending stream, worth ~6% of
//                              HBM bandwidth over lists ordered by racing atomics.
//                              Very large tables get a middle pass (scan_groups) that groups the workgroup totals.
//   fetch_kv_small           : small block tables - the whole fetch in one launch, every workgroup resolving its own cell.
//   resolve_experts          : the same for expert weights (Section 4.3: residency map) - one workgroup forms the
//                              distinct set of routed experts and walks it in ascending order (very large batches of
//                              routing ids are marked by many workgroups first: mark_experts).
//   gather                   : the copy itself.  HBM tier: one wavefront per workgroup and 1 KiB tile, one 16-byte
//                              non-temporal load and store per thread, as many workgroups as tiles; plane K before
//                              plane V, or - where the cache tier keeps them side by side - both planes of a request
//                              in one pass (measured on MI355X: short workgroups beat deep unrolling and persistent
//                              grids by ~15%, one-wavefront workgroups beat four-wavefront ones by 2-5%, non-temporal
//                              accesses are worth ~11%, 64 KiB source runs 4-5% over 32 KiB ones).
//   gather_host              : host tier - a couple of dozen persistent workgroups with two loads in flight per
//                              thread over 4 KiB sub-tiles: enough compute units to keep the PCIe link full, and no
//                              more host reads in flight than the link absorbs, because the rest would only stand in
//                              the HBM tier's way.
//   gather_hm, gather_hm_host: the same two into a head-major working layout.
//   copy_items, copy_items2, fill_items, dir_write : host-built lists - placement, write-back (one source, up to two
//                              destinations), slot poisoning after revocation, directory publication; the _hbm forms
//                              of the first three serve copies that stay inside HBM.  The forms that cross PCIe are a
//                              dozen persistent workgroups whose tiles are counted out one at a time, and they stand
//                              back while a fetch has announced that it needs the link (link_announce, yield_link).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hv {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int WG = 256;                         // 4 wavefronts
constexpr int WAVES = WG / 64;
constexpr uint32_t TILE_4K = WG * 16;           // 4 KiB: one 16-byte access per thread of a 256-thread workgroup
constexpr int HBM_WG = 64;                      // the HBM-tier gather runs one wavefront per workgroup (see gather)
constexpr int UNROLL_HOST = 8;
constexpr uint32_t TILE_HOST = WG * 16 * UNROLL_HOST;   // 32 KiB tiles of the host-built copy lists (place, write-back)
constexpr int HOST_LOADS = 2;                   // 16-byte loads a thread of the host-tier gather keeps in flight

// directory entry: [1:0] tier, [31:2] slot in that tier (host slot for HOST), [63:32] generation
constexpr uint64_t TIER_MASK = 3;
__host__ __device__ inline uint32_t entry_tier(uint64_t e) { return (uint32_t)(e & TIER_MASK); }
__host__ __device__ inline uint32_t entry_slot(uint64_t e) { return (uint32_t)(e >> 2) & 0x3FFFFFFFu; }
__host__ __device__ inline uint64_t make_entry(uint32_t tier, uint32_t slot, uint32_t gen)
{
    return (uint64_t)tier | ((uint64_t)(slot & 0x3FFFFFFFu) << 2) | ((uint64_t)gen << 32);
}
enum { T_HOST = 0, T_CACHE = 1, T_LOCAL = 2, T_NONE = 3 };

// One request of a fetch, the same for every plane of its class:
//   src = byte offset of the chunk inside its tier's plane pool, tier in bits [1:0] (offsets are multiples of 16);
//   dst = byte offset of the chunk inside the destination plane.
struct Rec { uint64_t src, dst; };
// Host-built lists carry absolute addresses.
struct Item { uint64_t src, dst; };
struct Item2 { uint64_t src, dst0, dst1, pad; };

// per-fetch counters (uint32) and running totals (uint64) share these indices
enum { C_REQ = 0, C_LOCAL, C_CACHE, C_HOST, C_LOST, C_INVALID, C_HBM_REQ, C_HOST_REQ, C_MISS, C_N = 16 };
// request kinds handed from classify_kv to compact_kv
enum { K_NONE = 0, K_HBM = 1, K_HOST = 2, K_LOST = 3 };

struct ClassDev {
    const uint64_t *dir;
    uint32_t n_objects, n_planes;
    uint64_t chunk_bytes;
    uint64_t pool[3][2];      // [tier HOST/CACHE/LOCAL][plane] base address as the GPU sees it
    uint32_t n_slots[3];      // slot numbers a directory entry may carry, per tier
    uint32_t pad;
    // chunk (layer, slot) of a tier's plane sits at  layer * layer_stride + slot * slot_stride  from the plane's base:
    // [layer][slot][chunk] pools have (n_slots * chunk, chunk); segments of the shared cache pool, [layer][plane][chunk]
    // from granule number `slot` on, have (n_planes * chunk, granule)
    uint64_t layer_stride[3];
    uint64_t slot_stride[3];
};

struct GatherArgs {
    uint64_t src_base[3][2];  // [tier][plane]
    uint64_t dst_base[2];     // [plane]
    uint64_t chunk_bytes;
    uint32_t tiles_per_chunk;
    uint32_t n_planes;
};

__device__ inline uint32_t lane_id() { return __lane_id(); }

// Selects instead of indexing: a variable index into a kernel-argument struct would send it to scratch memory.
__device__ inline uint32_t slots_of(const ClassDev &c, int tier)
{
    return tier == T_HOST ? c.n_slots[T_HOST] : (tier == T_CACHE ? c.n_slots[T_CACHE] : c.n_slots[T_LOCAL]);
}
__device__ inline uint64_t chunk_offset(const ClassDev &c, int tier, uint32_t layer, uint32_t slot)
{
    uint64_t ls = tier == T_HOST ? c.layer_stride[T_HOST] : (tier == T_CACHE ? c.layer_stride[T_CACHE] : c.layer_stride[T_LOCAL]);
    uint64_t ss = tier == T_HOST ? c.slot_stride[T_HOST] : (tier == T_CACHE ? c.slot_stride[T_CACHE] : c.slot_stride[T_LOCAL]);
    return (uint64_t)layer * ls + (uint64_t)slot * ss;
}
__device__ inline uint64_t src_base_of(const GatherArgs &a, uint32_t tier, uint32_t plane)
{
    uint64_t h = plane ? a.src_base[T_HOST][1] : a.src_base[T_HOST][0];
    uint64_t k = plane ? a.src_base[T_CACHE][1] : a.src_base[T_CACHE][0];
    uint64_t l = plane ? a.src_base[T_LOCAL][1] : a.src_base[T_LOCAL][0];
    return tier == T_HOST ? h : (tier == T_CACHE ? k : l);
}

// Exclusive rank of this lane among the lanes of its wavefront for which pred holds, and the wave total.
__device__ inline uint32_t wave_rank(bool pred, uint32_t &total)
{
    unsigned long long m = __ballot(pred);
    total = (uint32_t)__popcll(m);
    return (uint32_t)__popcll(m & ((1ull << lane_id()) - 1ull));
}

__device__ inline uint32_t wave_sum(uint32_t v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// ---------------------------------------------------------------------------------------------------------
// KV, pass 1: one thread per (sequence, block-table column) looks its block up and says what kind of request
// it is; every workgroup leaves its totals in blk_counts[BC_N * blockIdx + ...].  Nothing is accumulated with
// atomics and nothing needs zeroing, so a fetch can be replayed from a captured graph as it is.
// ---------------------------------------------------------------------------------------------------------
enum { BC_HBM = 0, BC_HOST, BC_MISS, BC_REQ, BC_LOCAL, BC_CACHE, BC_LOST, BC_INVALID, BC_N = 8 };

// What cell r of the block table asks for: -1 nothing (beyond the row's length), 0..3 the tier of its block, 4 an invalid
// request (unknown block, or a destination that does not fit).  For tiers 0..2 rec names source and destination.
__device__ inline int resolve_cell(const ClassDev &c, uint32_t layer, const int32_t *__restrict__ table,
                                   const int32_t *__restrict__ n_blocks, uint32_t max_blocks,
                                   const uint64_t *__restrict__ seq_dst_block, uint64_t dst_cap,
                                   const uint32_t *__restrict__ seq_cap_blocks, uint64_t strip_bytes, uint32_t r, Rec &rec)
{
    uint32_t s = r / max_blocks, j = r - s * max_blocks;
    int32_t nb = n_blocks[s];
    nb = nb < 0 ? 0 : (nb > (int32_t)max_blocks ? (int32_t)max_blocks : nb);
    if (j >= (uint32_t)nb) return -1;
    int32_t b = table[r];
    uint64_t first = seq_dst_block[s];
    uint64_t dst_chunk = first + j;
    bool fits = dst_chunk < dst_cap;
    uint64_t cap = 0;
    if (seq_cap_blocks) {
        cap = seq_cap_blocks[s];
        fits = first + cap <= dst_cap && j < cap && cap < 65536;
    }
    if (b < 0 || (uint32_t)b >= c.n_objects || !fits) return 4;
    uint64_t e = c.dir[b];
    int tier = (int)entry_tier(e);
    uint32_t slot = entry_slot(e);
    rec.dst = seq_cap_blocks ? first * c.chunk_bytes + (uint64_t)j * strip_bytes : dst_chunk * c.chunk_bytes;
    if (tier != T_NONE) {
        if (slot >= slots_of(c, tier)) return 4;                // never true for a directory the library wrote
        rec.src = chunk_offset(c, tier, layer, slot) | (uint64_t)tier | (cap << 48);
    }
    return tier;
}

__global__ __launch_bounds__(WG) void classify_kv(ClassDev c, uint32_t layer, const int32_t *__restrict__ table,
                                                  const int32_t *__restrict__ n_blocks, uint32_t n_seq,
                                                  uint32_t max_blocks, const uint64_t *__restrict__ seq_dst_block,
                                                  uint64_t dst_cap, Rec *__restrict__ tmp, uint8_t *__restrict__ kind,
                                                  uint32_t *__restrict__ blk_counts,
                                                  const uint32_t *__restrict__ seq_cap_blocks, uint64_t strip_bytes)
{
    // seq_cap_blocks != nullptr selects the head-major working layout: sequence s owns seq_cap_blocks[s] destination
    // blocks, laid out [head][token][head_bytes]; strip_bytes = block_tokens * head_bytes is what one block adds to
    // one head's strip.  The record then carries the sequence's capacity (in blocks) in bits [63:48] of src.
    __shared__ uint32_t s_cnt[BC_N];
    uint32_t tid = threadIdx.x;
    uint32_t r = blockIdx.x * WG + tid;
    if (tid < BC_N) s_cnt[tid] = 0;
    __syncthreads();
    uint32_t total = n_seq * max_blocks;
    int tier = -1;                       // -1 no request, 0..3 tier, 4 invalid
    Rec rec = { 0, 0 };
    if (r < total)
        tier = resolve_cell(c, layer, table, n_blocks, max_blocks, seq_dst_block, dst_cap, seq_cap_blocks, strip_bytes, r, rec);
    uint32_t k = (tier == T_LOCAL || tier == T_CACHE) ? K_HBM
                                                      : (tier == T_HOST ? K_HOST : (tier == T_NONE ? K_LOST : K_NONE));
    if (r < total) {
        kind[r] = (uint8_t)k;
        if (k == K_HBM || k == K_HOST) tmp[r] = rec;
    }
    // wave ballots -> LDS -> one row of totals per workgroup
    const int which[BC_N] = { BC_HBM, BC_HOST, BC_MISS, BC_REQ, BC_LOCAL, BC_CACHE, BC_LOST, BC_INVALID };
    const bool pred[BC_N] = { k == K_HBM, k == K_HOST, k == K_HOST || k == K_LOST, tier >= 0,
                              tier == T_LOCAL, tier == T_CACHE, tier == T_NONE, tier == 4 };
#pragma unroll
    for (int i = 0; i < BC_N; ++i) {
        uint32_t n = (uint32_t)__popcll(__ballot(pred[i]));
        if (lane_id() == 0 && n) atomicAdd(&s_cnt[which[i]], n);
    }
    __syncthreads();
    if (tid < BC_N) blk_counts[blockIdx.x * BC_N + tid] = s_cnt[tid];
}

// KV, middle pass for large tables only.  In pass 2 every workgroup adds up the rows of all workgroups before it: fine for
// a few hundred rows, quadratic beyond (a table of 8 M cells has 32 768 rows: 17 GB of reads).  This pass makes groups of
// WG rows: workgroup g leaves the totals of its group in grp_totals[g] and, for each of its rows, the list counters of the
// group's earlier rows in row_prefix[row] - pass 2 then adds up whole groups only.
__global__ __launch_bounds__(WG) void scan_groups(const uint32_t *__restrict__ blk_counts, uint32_t n_rows,
                                                  uint32_t *__restrict__ grp_totals, uint32_t *__restrict__ row_prefix)
{
    __shared__ uint32_t s_wave[WAVES][BC_N];
    uint32_t tid = threadIdx.x, wave = tid >> 6, lane = lane_id();
    uint32_t row = blockIdx.x * WG + tid;
    uint32_t v[BC_N], incl[3];
#pragma unroll
    for (int i = 0; i < BC_N; ++i) v[i] = row < n_rows ? blk_counts[row * BC_N + i] : 0u;
    // inclusive scan of the three list counters (BC_HBM, BC_HOST, BC_MISS are 0, 1, 2) within the wavefront
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        uint32_t x = v[k];
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            uint32_t y = __shfl_up(x, o);
            if (lane >= (uint32_t)o) x += y;
        }
        incl[k] = x;
    }
    uint32_t tot[BC_N];
#pragma unroll
    for (int i = 0; i < BC_N; ++i) tot[i] = wave_sum(v[i]);
    if (lane == 0) {
#pragma unroll
        for (int i = 0; i < BC_N; ++i) s_wave[wave][i] = tot[i];
    }
    __syncthreads();
    if (row < n_rows) {
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            uint32_t before = 0;
            for (uint32_t w = 0; w < wave; ++w) before += s_wave[w][k];
            row_prefix[row * 3 + k] = before + incl[k] - v[k];
        }
    }
    if (tid < BC_N) {
        uint32_t t = 0;
        for (int w = 0; w < WAVES; ++w) t += s_wave[w][tid];
        grp_totals[blockIdx.x * BC_N + tid] = t;
    }
}

// KV, pass 2: list position = (totals of the workgroups before mine) + (totals of the waves before mine in the
// workgroup) + (rank in my wave), so the lists come out in request order.  The last workgroup has seen every
// total: it writes the counters of this fetch and adds them to the running totals.
__global__ __launch_bounds__(WG) void compact_kv(uint32_t total, const Rec *__restrict__ tmp,
                                                 const uint8_t *__restrict__ kind, const uint32_t *__restrict__ blk_counts,
                                                 Rec *__restrict__ hbm_recs, Rec *__restrict__ host_recs,
                                                 uint32_t *__restrict__ miss_idx, uint32_t *cnt,
                                                 unsigned long long *totals, const uint32_t *__restrict__ grp_totals,
                                                 const uint32_t *__restrict__ row_prefix)
{
    // grp_totals / row_prefix: what scan_groups left (large tables), or null - then the rows themselves are added up.
    __shared__ uint32_t s_pre[BC_N];
    __shared__ uint32_t s_wave[WAVES][3];
    uint32_t tid = threadIdx.x, wave = tid >> 6;
    uint32_t r = blockIdx.x * WG + tid;
    bool last = blockIdx.x == gridDim.x - 1;
    if (wave == 0) {
        uint32_t a[BC_N];
#pragma unroll
        for (int i = 0; i < BC_N; ++i) a[i] = 0;
        const uint32_t *rows = grp_totals ? grp_totals : blk_counts;
        uint32_t n_all = grp_totals ? (gridDim.x + WG - 1) / WG : gridDim.x;
        uint32_t mine = grp_totals ? blockIdx.x / WG : blockIdx.x;
        uint32_t upto = last ? n_all : mine;                    // the last workgroup sums everybody, itself included
        for (uint32_t b = lane_id(); b < upto; b += 64) {
#pragma unroll
            for (int i = 0; i < BC_N; ++i) a[i] += rows[b * BC_N + i];
        }
#pragma unroll
        for (int i = 0; i < BC_N; ++i) a[i] = wave_sum(a[i]);
        if (lane_id() == 0) {
#pragma unroll
            for (int i = 0; i < BC_N; ++i) s_pre[i] = a[i];
        }
    }
    uint32_t k = r < total ? kind[r] : (uint32_t)K_NONE;
    uint32_t n_hbm, n_host, n_miss;
    uint32_t p_hbm = wave_rank(k == K_HBM, n_hbm);
    uint32_t p_host = wave_rank(k == K_HOST, n_host);
    uint32_t p_miss = wave_rank(k == K_HOST || k == K_LOST, n_miss);
    if (lane_id() == 0) { s_wave[wave][0] = n_hbm; s_wave[wave][1] = n_host; s_wave[wave][2] = n_miss; }
    __syncthreads();
    uint32_t b_hbm = s_pre[BC_HBM], b_host = s_pre[BC_HOST], b_miss = s_pre[BC_MISS];
    if (last) {                                  // its sums included its own row (its whole group): take that out
        const uint32_t *own = grp_totals ? grp_totals + (blockIdx.x / WG) * BC_N : blk_counts + blockIdx.x * BC_N;
        b_hbm -= own[BC_HBM];
        b_host -= own[BC_HOST];
        b_miss -= own[BC_MISS];
    }
    if (row_prefix) {                            // the rows of my group before mine
        b_hbm += row_prefix[blockIdx.x * 3 + BC_HBM];
        b_host += row_prefix[blockIdx.x * 3 + BC_HOST];
        b_miss += row_prefix[blockIdx.x * 3 + BC_MISS];
    }
    for (uint32_t w = 0; w < wave; ++w) { b_hbm += s_wave[w][0]; b_host += s_wave[w][1]; b_miss += s_wave[w][2]; }
    if (k == K_HBM) hbm_recs[b_hbm + p_hbm] = tmp[r];
    if (k == K_HOST) host_recs[b_host + p_host] = tmp[r];
    if (k == K_HOST || k == K_LOST) miss_idx[b_miss + p_miss] = r;
    if (last && tid == 0) {
        cnt[C_HBM_REQ] = s_pre[BC_HBM]; cnt[C_HOST_REQ] = s_pre[BC_HOST]; cnt[C_MISS] = s_pre[BC_MISS];
        const int from[6] = { BC_REQ, BC_LOCAL, BC_CACHE, BC_HOST, BC_LOST, BC_INVALID };
        const int to[6] = { C_REQ, C_LOCAL, C_CACHE, C_HOST, C_LOST, C_INVALID };
        for (int i = 0; i < 6; ++i) {
            uint32_t v = s_pre[from[i]];
            cnt[to[i]] = v;
            if (v) atomicAdd(&totals[to[i]], (unsigned long long)v);
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// Experts: one workgroup forms the distinct set of the routed expert numbers (bitmap in LDS), then walks the
// experts in ascending order so that staging ranks are the ranks among the staged members of the set.
// ---------------------------------------------------------------------------------------------------------
constexpr uint32_t MAX_EXPERTS = 8192;

// Large batches only: many workgroups mark the routed experts - each in a bitmap of its own in LDS, merged into
// g_bitmap with one atomic per non-zero word - so that the single workgroup of resolve_experts need not read every
// routing id itself (half a million ids cost it 0.4 ms).  g_bitmap and g_invalid are zero on entry; resolve_experts
// takes their contents and leaves them zero again, so nothing has to be cleared between fetches or graph replays.
__global__ __launch_bounds__(WG) void mark_experts(const int32_t *__restrict__ topk, uint32_t n_ids, uint32_t n_experts,
                                                   uint32_t *g_bitmap, uint32_t *g_invalid)
{
    __shared__ uint32_t bm[MAX_EXPERTS / 32];
    __shared__ uint32_t inval;
    uint32_t tid = threadIdx.x, words = (n_experts + 31) / 32;
    for (uint32_t i = tid; i < words; i += WG) bm[i] = 0;
    if (tid == 0) inval = 0;
    __syncthreads();
    for (uint64_t i = (uint64_t)blockIdx.x * WG + tid; i < n_ids; i += (uint64_t)gridDim.x * WG) {
        int32_t e = topk[i];
        if (e < 0 || (uint32_t)e >= n_experts) atomicAdd(&inval, 1u);
        else atomicOr(&bm[e >> 5], 1u << (e & 31));
    }
    __syncthreads();
    for (uint32_t i = tid; i < words; i += WG)
        if (bm[i]) atomicOr(&g_bitmap[i], bm[i]);
    if (tid == 0 && inval) atomicAdd(g_invalid, inval);
}

__global__ __launch_bounds__(WG) void resolve_experts(ClassDev c, uint32_t layer, uint32_t n_experts,
                                                      const int32_t *__restrict__ topk, uint32_t n_ids,
                                                      uint64_t staging, uint32_t n_staging,
                                                      uint64_t *__restrict__ expert_ptr, Rec *__restrict__ hbm_recs,
                                                      Rec *__restrict__ host_recs, uint32_t *__restrict__ miss_idx,
                                                      uint32_t *cnt, unsigned long long *totals, uint32_t *g_bitmap,
                                                      uint32_t *g_invalid)
{
    // g_bitmap != nullptr: mark_experts has already formed the routed set; it is taken from there (and cleared).
    __shared__ uint32_t bitmap[MAX_EXPERTS / 32];
    __shared__ uint32_t s_cnt[C_N];
    __shared__ uint32_t wave_tot[WG / 64];
    __shared__ uint32_t running;
    uint32_t tid = threadIdx.x;
    for (uint32_t i = tid; i < MAX_EXPERTS / 32; i += WG) {
        uint32_t w = 0;
        if (g_bitmap && i < (n_experts + 31) / 32) { w = g_bitmap[i]; g_bitmap[i] = 0; }
        bitmap[i] = w;
    }
    if (tid < C_N) s_cnt[tid] = 0;
    if (tid == 0) running = 0;
    __syncthreads();
    if (g_bitmap) {
        if (tid == 0) { s_cnt[C_INVALID] = *g_invalid; *g_invalid = 0; }
    } else {
        for (uint32_t i = tid; i < n_ids; i += WG) {
            int32_t e = topk[i];
            if (e < 0 || (uint32_t)e >= n_experts) atomicAdd(&s_cnt[C_INVALID], 1u);
            else atomicOr(&bitmap[e >> 5], 1u << (e & 31));
        }
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
                    Rec it;                 // few, large objects: their order in the lists does not matter
                    it.src = chunk_offset(c, tier, 0, slot) | (uint64_t)tier;
                    it.dst = (uint64_t)rank * c.chunk_bytes;
                    if (tier == T_CACHE) {
                        hbm_recs[atomicAdd(&s_cnt[C_HBM_REQ], 1u)] = it;
                        atomicAdd(&s_cnt[C_CACHE], 1u);
                    } else {
                        host_recs[atomicAdd(&s_cnt[C_HOST_REQ], 1u)] = it;
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
// The gather.
// ---------------------------------------------------------------------------------------------------------
// Every payload access names the global address space: an address computed as an integer would otherwise compile to
// flat_load / flat_store, which pay for an aperture check on each access; global_load / global_store do not.
typedef __attribute__((address_space(1))) u32x4 g_u32x4;

template <bool NT>
__device__ inline u32x4 ld16(const u32x4 *p)
{
    const g_u32x4 *g = (const g_u32x4 *)(uint64_t)p;
    if (NT) return __builtin_nontemporal_load(g);
    return *g;
}
template <bool NT>
__device__ inline void st16(u32x4 *p, u32x4 v)
{
    g_u32x4 *g = (g_u32x4 *)(uint64_t)p;
    if (NT) __builtin_nontemporal_store(v, g);
    else *g = v;
}

// One tile of NTHR * 16 * UNROLL bytes (or the first len bytes of it) by a workgroup of NTHR threads.
template <int NTHR, int UNROLL, bool NT>
__device__ inline void copy_tile(uint64_t src, uint64_t dst, uint64_t len, uint32_t tid)
{
    constexpr uint32_t TILE = NTHR * 16 * UNROLL;
    const u32x4 *s = reinterpret_cast<const u32x4 *>(src);
    u32x4 *d = reinterpret_cast<u32x4 *>(dst);
    if (len >= TILE) {
        u32x4 v[UNROLL];
#pragma unroll
        for (int i = 0; i < UNROLL; ++i) v[i] = ld16<NT>(s + tid + i * NTHR);
#pragma unroll
        for (int i = 0; i < UNROLL; ++i) st16<NT>(d + tid + i * NTHR, v[i]);
    } else {
        uint32_t n_vec = (uint32_t)(len >> 4);
        for (uint32_t i = tid; i < n_vec; i += NTHR) st16<NT>(d + i, ld16<NT>(s + i));
    }
}

// Tiles of the chunks named by a request list whose length lives on the device.  blockIdx.y is the plane, so a
// two-plane class is gathered plane after plane.  The grid's x size is free: with one workgroup per tile the loop body
// runs once; a smaller grid loops.  `feedback`, when given, is a word of pinned host memory that receives the list
// length: the host sizes the next launch from it, because workgroups that find no tile are not free (about 0.2 ns
// each on MI355X) while a grid somewhat short of the tile count is.
//
// NTHR threads per workgroup, one 16-byte load and store each: a tile is NTHR * 16 bytes.  Measured on MI355X
// (768 MiB gathered from scattered runs, read+write): one-wavefront workgroups (1 KiB tiles) move 6.29 TB/s from 32 KiB
// runs and 6.57 TB/s from 64 KiB runs, 256-thread workgroups 6.12 and 6.40 - a wavefront that is its own workgroup
// frees its slot the moment it is done instead of waiting for three others.
//
// FOLD: the planes of a request are taken in one pass - tile numbers run through plane 0, then plane 1, of each
// request - instead of plane after plane over the whole list (blockIdx.y).  Where the cache tier keeps the planes of an
// object next to each other this turns two 32 KiB source runs into one 64 KiB run, the length from which scattered
// runs read as fast as a contiguous buffer (6.29 -> 6.57 TB/s in the measurement above); where the planes live in
// pools of their own, plane after plane is the faster order (6.24 against 6.11 TB/s).
template <int NTHR, bool NT, bool FOLD>
__global__ __launch_bounds__(NTHR) void gather(const Rec *__restrict__ recs, const uint32_t *__restrict__ n_req_ptr,
                                               GatherArgs a, uint32_t *feedback)
{
    constexpr uint32_t TILE = NTHR * 16;
    uint32_t bx = blockIdx.x, gx = gridDim.x;
    // The first tile's list entry is fetched before the length is known, so that the two scalar loads overlap: a
    // workgroup lives for one load and one store, and every dependent load in front of them costs bandwidth.  The
    // host never launches more workgroups (in x) than the list has room for tiles, so the early read stays inside
    // the list; it also guarantees capacity * tiles per request < 2^32, so tile numbers fit 32-bit division.
    uint32_t tpc = a.tiles_per_chunk;
    uint32_t tpr = FOLD ? tpc * a.n_planes : tpc;              // tiles per request in this grid's x dimension
    uint64_t t = bx;
    uint32_t idx = (uint32_t)t / tpr;
    Rec x = recs[idx];
    uint32_t n_req = *n_req_ptr;
    if (feedback && bx == 0 && blockIdx.y == 0 && threadIdx.x == 0) *feedback = n_req;
    uint64_t n_tiles = (uint64_t)n_req * tpr;
    while (t < n_tiles) {
        uint32_t k = (uint32_t)t - idx * tpr;
        uint32_t plane = FOLD ? (k >= tpc ? 1u : 0u) : blockIdx.y;
        uint64_t off = (uint64_t)(FOLD ? k - plane * tpc : k) * TILE;
        uint64_t src = src_base_of(a, (uint32_t)(x.src & 3), plane) + (x.src & ~(uint64_t)3) + off;
        uint64_t dst_base = plane ? a.dst_base[1] : a.dst_base[0];
        copy_tile<NTHR, 1, NT>(src, dst_base + x.dst + off, a.chunk_bytes - off, threadIdx.x);
        t += gx;
        if (t >= n_tiles) break;
        idx = (uint32_t)t / tpr;
        x = recs[idx];
    }
}

// Who gets the PCIe link.  A fetch that reads from the host announces, in a word of device memory, until when it
// expects to need the link (link_announce: now + its host-tier bytes at the link's rate, on the device's constant 100 MHz
// clock); the copies that cross the link outside a fetch - placements, write-backs - look at that word before they take
// their next tile and stand back while the time has not come (yield_link), though never for longer than YIELD_TICKS per
// tile, so that they always get on (at a tenth of the link's rate or so when fetches never pause).  A miss is on the
// critical path and a placement is best effort (paper Sections 2.2 and 3.1).  An estimate instead of an exact begin /
// end: nothing has to be counted or taken back, and a word that is stale means no more than "nobody is fetching".  The
// estimate is on the short side (the rate of an undisturbed fetch, no margin): a copy that follows the fetch on the same
// stream, which cannot run beside it anyway, must not be kept waiting for a fetch that is already over.
constexpr uint64_t LINK_BYTES_PER_TICK = 575;      // 57.5 GB/s at 100 MHz
constexpr uint64_t YIELD_TICKS = 6000;             // 60 us
__device__ inline void link_announce(unsigned long long *lease, uint64_t host_bytes)
{
    if (!lease || !host_bytes) return;
    atomicMax(lease, (unsigned long long)(wall_clock64() + host_bytes / LINK_BYTES_PER_TICK));
}
__device__ inline void yield_link(const unsigned long long *lease)
{
    if (!lease) return;
    const uint64_t t0 = wall_clock64();
    for (;;) {
        const uint64_t now = wall_clock64();
        if (now - t0 >= YIELD_TICKS || now >= __hip_atomic_load(lease, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) return;
        __builtin_amdgcn_s_sleep(127);
    }
}

// The whole KV fetch in one kernel, for small block tables (token-major layout, one layer).  A fetch of a few blocks is
// made of launch gaps, not of bytes: resolve, compaction and the two gathers are four dependent kernels of a few
// microseconds each.  Here workgroup (cell r, tile k, plane p) resolves cell r by itself and copies its tile from whichever
// tier holds the block (a host-tier tile is read over PCIe by the same 16-byte loads); nothing is compacted, so the grid
// covers the padded table - which is why this is for small tables only.  blockIdx.z counts consecutive layers (an object
// has the same slot in every layer): layer + z is read, dst_step * z further into the destination is written.  The books (counters, miss list in request
// order) are kept by the first workgroup alone, which walks the whole table once more, a cell per thread: no atomics on
// shared counters (a thousand of them on one address take longer than the copy), nothing to zero.
__global__ __launch_bounds__(WG) void fetch_kv_small(ClassDev c, uint32_t layer, const int32_t *__restrict__ table,
                                                     const int32_t *__restrict__ n_blocks, uint32_t n_seq,
                                                     uint32_t max_blocks, const uint64_t *__restrict__ seq_dst_block,
                                                     uint64_t dst_cap, GatherArgs a, uint64_t dst_step,
                                                     uint32_t *__restrict__ miss_idx, uint32_t *cnt,
                                                     unsigned long long *totals, uint32_t *feedback_hbm,
                                                     uint32_t *feedback_host, unsigned long long *lease)
{
    uint32_t tpc = a.tiles_per_chunk;
    uint32_t r = blockIdx.x / tpc, k = blockIdx.x - r * tpc, plane = blockIdx.y;
    uint32_t total = n_seq * max_blocks;                       // the host launches exactly total * tpc workgroups in x
    {
        Rec rec = { 0, 0 };
        int tier = resolve_cell(c, layer + blockIdx.z, table, n_blocks, max_blocks, seq_dst_block, dst_cap, nullptr, 0, r, rec);
        if (tier == T_HOST || tier == T_CACHE || tier == T_LOCAL) {
            uint64_t off = (uint64_t)k * TILE_4K;
            uint64_t src = src_base_of(a, (uint32_t)tier, plane) + (rec.src & 0x0000FFFFFFFFFFFCull) + off;
            uint64_t dst = (plane ? a.dst_base[1] : a.dst_base[0]) + (uint64_t)blockIdx.z * dst_step + rec.dst + off;
            if (tier == T_HOST) copy_tile<WG, 1, false>(src, dst, a.chunk_bytes - off, threadIdx.x);
            else copy_tile<WG, 1, true>(src, dst, a.chunk_bytes - off, threadIdx.x);
        }
    }
    if (blockIdx.x != 0 || plane != 0 || blockIdx.z != 0) return;
    // ---- the books: every cell once more, one per thread (residency is the same for every layer) ----
    __shared__ uint32_t s_cnt[C_N];
    __shared__ uint32_t s_wave[WAVES];
    __shared__ uint32_t s_base;
    uint32_t tid = threadIdx.x, wave = tid >> 6;
    if (tid < C_N) s_cnt[tid] = 0;
    if (tid == 0) s_base = 0;
    __syncthreads();
    for (uint32_t first = 0; first < total; first += WG) {
        uint32_t q = first + tid;
        Rec rec = { 0, 0 };
        int tier = q < total ? resolve_cell(c, layer, table, n_blocks, max_blocks, seq_dst_block, dst_cap, nullptr, 0, q, rec) : -1;
        bool miss = tier == T_HOST || tier == T_NONE;
        uint32_t n_miss;
        uint32_t rank = wave_rank(miss, n_miss);
        if (lane_id() == 0) s_wave[wave] = n_miss;
        const int which[6] = { C_REQ, C_LOCAL, C_CACHE, C_HOST, C_LOST, C_INVALID };
        const bool pred[6] = { tier >= 0, tier == T_LOCAL, tier == T_CACHE, tier == T_HOST, tier == T_NONE, tier == 4 };
#pragma unroll
        for (int i = 0; i < 6; ++i) {
            uint32_t n = (uint32_t)__popcll(__ballot(pred[i]));
            if (lane_id() == 0 && n) atomicAdd(&s_cnt[which[i]], n);
        }
        __syncthreads();
        uint32_t before = s_base;
        for (uint32_t w = 0; w < wave; ++w) before += s_wave[w];
        if (miss) miss_idx[before + rank] = q;
        __syncthreads();
        if (tid == 0) {
            uint32_t t = 0;
            for (int w = 0; w < WAVES; ++w) t += s_wave[w];
            s_base += t;
        }
        __syncthreads();
    }
    if (tid == 0) {
        uint32_t hbm = s_cnt[C_LOCAL] + s_cnt[C_CACHE], host = s_cnt[C_HOST];
        for (int i = 0; i <= C_INVALID; ++i) {
            cnt[i] = s_cnt[i];
            if (s_cnt[i]) atomicAdd(&totals[i], (unsigned long long)s_cnt[i]);
        }
        cnt[C_HBM_REQ] = hbm;
        cnt[C_HOST_REQ] = host;
        cnt[C_MISS] = s_base;
        *feedback_hbm = hbm;
        *feedback_host = host;
        link_announce(lease, (uint64_t)host * a.chunk_bytes * a.n_planes * gridDim.z);
    }
}

// The gather into a head-major working layout: a pool block is [token][head][head_bytes], the destination of a
// sequence is [head][token][head_bytes].  Threads walk the block in DESTINATION order (16-byte units), so stores are
// fully contiguous per head strip and loads come as head_bytes-long runs (256 B at the paper-shaped config: two whole
// 128-byte lines).  No LDS: nothing is reused, the permutation is pure address arithmetic.  Staging through LDS was
// measured on MI355X and lost: a whole 32 KiB block per workgroup (source-order loads, 8 strips of 4 KiB stored) moves
// 5.31 TB/s against 5.81 for this kernel (12 041 scattered blocks, alone), and tiles of 4 tokens x 4 heads (every wave
// instruction a contiguous kilobyte on both sides) 5.91 in isolation but 5.85 against 5.94 once inside the library's
// looping, feedback-sized launch.  One-wavefront workgroups (1 KiB tiles), the token-major gather's shape, are a
// wash here: 5.95 against 5.90 TB/s alone, 5.32 against 5.35 inside the step.
struct HmArgs {
    uint32_t n_heads;
    uint32_t upr;             // 16-byte units per head row (head_bytes / 16)
    uint32_t ups;             // units one block adds to one head strip (block_tokens * upr)
    uint32_t pad;
};

template <int UNROLL, bool NT>
__global__ __launch_bounds__(WG) void gather_hm(const Rec *__restrict__ recs, const uint32_t *__restrict__ n_req_ptr,
                                                GatherArgs a, HmArgs h, uint32_t *feedback)
{
    // blockIdx.y is the plane: taking both planes of a request in one pass, as gather does for a cache tier that keeps
    // them side by side, was measured to lose here (5.60 against 5.98 TB/s alone): the stores are 4 KiB strips, and with
    // two planes' strips interleaved they no longer follow each other
    constexpr uint32_t UNITS = WG * UNROLL;
    uint32_t tpr = a.tiles_per_chunk;
    uint64_t t = blockIdx.x;
    uint32_t idx = (uint32_t)t / tpr;
    Rec x = recs[idx];                                   // speculative, as in gather
    uint32_t n_req = *n_req_ptr;
    if (feedback && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *feedback = n_req;
    uint64_t n_tiles = (uint64_t)n_req * tpr;
    uint32_t chunk_units = (uint32_t)(a.chunk_bytes >> 4);
    while (t < n_tiles) {
        uint32_t k = (uint32_t)t - idx * tpr;
        uint32_t plane = blockIdx.y;
        uint64_t dst_plane = plane ? a.dst_base[1] : a.dst_base[0];
        uint32_t u0 = k * UNITS + threadIdx.x;
        uint64_t cap = x.src >> 48;
        uint64_t src = src_base_of(a, (uint32_t)(x.src & 3), plane) + (x.src & 0x0000FFFFFFFFFFFCull);
        uint64_t dst = dst_plane + x.dst;
        uint64_t head_stride = cap * h.ups * 16;
        // unit u (in walking order) -> source unit and destination byte offset
        auto map = [&](uint32_t u, uint32_t &s_unit, uint64_t &d_off) {
            uint32_t head = u / h.ups, rem = u - head * h.ups;
            uint32_t tok = rem / h.upr, col = rem - tok * h.upr;
            s_unit = (tok * h.n_heads + head) * h.upr + col;
            d_off = head * head_stride + (uint64_t)rem * 16;
        };
        uint32_t tile_first = k * UNITS;
        if (tile_first + UNITS <= chunk_units) {
            // whole tile: no per-element branches, so all loads are in flight before the first store
            u32x4 v[UNROLL];
            uint64_t d_off[UNROLL];
#pragma unroll
            for (int i = 0; i < UNROLL; ++i) {
                uint32_t s_unit;
                map(u0 + i * WG, s_unit, d_off[i]);
                v[i] = ld16<NT>(reinterpret_cast<const u32x4 *>(src) + s_unit);
            }
#pragma unroll
            for (int i = 0; i < UNROLL; ++i) st16<true>(reinterpret_cast<u32x4 *>(dst + d_off[i]), v[i]);
        } else {
            for (uint32_t u = u0; u < chunk_units; u += WG) {
                uint32_t s_unit;
                uint64_t d_off;
                map(u, s_unit, d_off);
                st16<true>(reinterpret_cast<u32x4 *>(dst + d_off), ld16<NT>(reinterpret_cast<const u32x4 *>(src) + s_unit));
            }
        }
        t += gridDim.x;
        if (t >= n_tiles) break;
        idx = (uint32_t)t / tpr;
        x = recs[idx];
    }
}

// Host tier: the same request list format, read over PCIe from pinned host memory by a few persistent workgroups.
//
// What the link needs (measured on MI355X): one compute unit sustains about 12.8 GB/s of reads from host memory however
// many loads its threads have outstanding, so the rate is set by how many CUs take part (5 saturate the 57 GB/s link) -
// and every host read in flight beyond what the link can absorb (about 128 KiB) only queues in the memory pipeline the
// HBM-tier gather is using at the same time: 8 workgroups x 16 loads per thread cost that kernel 12 %, 24 workgroups x
// 2 loads cost it 8 % and serve the link better (57.1 against 56.8 GB/s).  Hence: HOST_LOADS = 2 loads of 16 bytes per
// thread, a couple of dozen workgroups.
//
// Work is cut into 4 KiB sub-tiles numbered through the whole list (request * sub-tiles per chunk + position), so the
// bytes in flight do not depend on the chunk size (16 KiB blocks of an fp8 KV cache and ragged sizes run at the same
// rate as 32 KiB blocks).  A two-plane class takes one sub-tile of both planes per step, a one-plane class two
// consecutive sub-tiles.  Each load is issued as soon as its list entry has arrived.  Lanes beyond a chunk's end
// re-read the chunk's first bytes and store nothing: loads stay free of branches.
struct HostSub {
    uint64_t src;      // offset of this lane's 16 bytes inside the tier's plane pool
    uint64_t dst;      // offset of the chunk inside the destination plane (head-major: of the sequence's region)
    uint32_t tier;
    uint32_t unit;     // this lane's 16-byte unit inside the chunk (0 when inactive)
    uint64_t cap;      // head-major only: the sequence's capacity in blocks
    bool act;
};

__device__ inline HostSub host_sub(const Rec *__restrict__ recs, uint64_t g, uint64_t n_sub, uint32_t spc,
                                   uint32_t chunk_units, uint32_t tid)
{
    HostSub r;
    bool valid = g < n_sub;
    uint32_t idx = valid ? (uint32_t)g / spc : 0;             // a step exists only when the list is not empty
    Rec x = recs[idx];
    uint32_t j = valid ? (uint32_t)g - idx * spc : 0;
    uint32_t u = j * WG + tid;
    r.act = valid && u < chunk_units;
    r.unit = r.act ? u : 0;
    r.src = (x.src & 0x0000FFFFFFFFFFFCull) + (uint64_t)r.unit * 16;
    r.dst = x.dst;
    r.tier = (uint32_t)(x.src & 3);
    r.cap = x.src >> 48;
    return r;
}

template <int PLANES>
__global__ __launch_bounds__(WG) void gather_host(const Rec *__restrict__ recs, const uint32_t *__restrict__ n_req_ptr,
                                                  GatherArgs a, uint32_t *feedback, unsigned long long *lease)
{
    constexpr int U = HOST_LOADS / PLANES;                     // sub-tiles per step
    uint32_t spc = a.tiles_per_chunk;                          // 4 KiB sub-tiles per chunk
    uint32_t n_req = *n_req_ptr;
    if (feedback && blockIdx.x == 0 && threadIdx.x == 0) *feedback = n_req;      // as in gather: a hint for the host
    if (blockIdx.x == 0 && threadIdx.x == 0) link_announce(lease, (uint64_t)n_req * a.chunk_bytes * PLANES);
    uint64_t n_sub = (uint64_t)n_req * spc;
    uint64_t n_steps = (n_sub + U - 1) / U;
    uint32_t chunk_units = (uint32_t)(a.chunk_bytes >> 4);
    uint32_t tid = threadIdx.x;
    for (uint64_t b = blockIdx.x; b < n_steps; b += gridDim.x) {
        HostSub q[U];
        u32x4 v0[U], v1[U];
#pragma unroll
        for (int i = 0; i < U; ++i) {
            q[i] = host_sub(recs, b * U + i, n_sub, spc, chunk_units, tid);
            v0[i] = ld16<false>(reinterpret_cast<const u32x4 *>(src_base_of(a, q[i].tier, 0) + q[i].src));
            if (PLANES == 2) v1[i] = ld16<false>(reinterpret_cast<const u32x4 *>(src_base_of(a, q[i].tier, 1) + q[i].src));
        }
#pragma unroll
        for (int i = 0; i < U; ++i) {
            if (!q[i].act) continue;
            uint64_t d = q[i].dst + (uint64_t)q[i].unit * 16;
            st16<true>(reinterpret_cast<u32x4 *>(a.dst_base[0] + d), v0[i]);
            if (PLANES == 2) st16<true>(reinterpret_cast<u32x4 *>(a.dst_base[1] + d), v1[i]);
        }
    }
}

// The same for the head-major layout.  Unlike the HBM-tier kernel above, threads walk the block in SOURCE order, so that
// every wave load is one contiguous kilobyte (PCIe reads of 256-byte pieces reach only 22 GB/s); the stores, which go to
// HBM, are the ones cut into head rows.  K and V of a unit go to the same place in their planes: one address
// computation serves both.
template <int PLANES>
__global__ __launch_bounds__(WG) void gather_hm_host(const Rec *__restrict__ recs, const uint32_t *__restrict__ n_req_ptr,
                                                     GatherArgs a, HmArgs h, uint32_t *feedback, unsigned long long *lease)
{
    uint32_t spc = a.tiles_per_chunk;
    uint32_t n_req = *n_req_ptr;
    if (feedback && blockIdx.x == 0 && threadIdx.x == 0) *feedback = n_req;
    if (blockIdx.x == 0 && threadIdx.x == 0) link_announce(lease, (uint64_t)n_req * a.chunk_bytes * PLANES);
    uint64_t n_sub = (uint64_t)n_req * spc;
    uint32_t chunk_units = (uint32_t)(a.chunk_bytes >> 4);
    uint32_t tid = threadIdx.x;
    uint32_t row_units = h.n_heads * h.upr;                    // one token: all heads
    for (uint64_t g = blockIdx.x; g < n_sub; g += gridDim.x) {
        HostSub q = host_sub(recs, g, n_sub, spc, chunk_units, tid);
        u32x4 v0 = ld16<false>(reinterpret_cast<const u32x4 *>(src_base_of(a, q.tier, 0) + q.src)), v1;
        if (PLANES == 2) v1 = ld16<false>(reinterpret_cast<const u32x4 *>(src_base_of(a, q.tier, 1) + q.src));
        uint32_t tok = q.unit / row_units, rem = q.unit - tok * row_units;
        uint32_t head = rem / h.upr, col = rem - head * h.upr;
        uint64_t d = q.dst + head * (q.cap * h.ups * 16) + (uint64_t)(tok * h.upr + col) * 16;
        if (q.act) {
            st16<true>(reinterpret_cast<u32x4 *>(a.dst_base[0] + d), v0);
            if (PLANES == 2) st16<true>(reinterpret_cast<u32x4 *>(a.dst_base[1] + d), v1);
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// Host-built lists (absolute addresses).
// ---------------------------------------------------------------------------------------------------------
constexpr size_t LIST_HEADER = 16;       // a host-built list travels behind this many bytes, the first 8 of them the
                                         // zeroed tile counter of the kernel that walks it
// The tiles of a persistent copy.  next == nullptr: workgroup b takes tiles b, b + grid, b + 2 grid, ...  Otherwise the
// tiles are counted out one at a time from *next (zero at launch): when something else is using the link as well, the
// workgroups of one launch progress at very different rates (a 3.4-fold spread was measured), and with fixed shares
// the launch ends with a few workgroups working off their backlog alone - a 906 MB placement beside a stream of
// fetches took 106 ms that way.  Every thread of the workgroup gets the same tile number and leaves the loop together.
template <typename F>
__device__ inline void for_each_tile(unsigned long long *next, uint64_t n_tiles, const unsigned long long *lease, F body)
{
    if (!next) {
        for (uint64_t t = blockIdx.x; t < n_tiles; t += gridDim.x) body(t);
        return;
    }
    __shared__ unsigned long long s_tile;
    for (;;) {
        if (threadIdx.x == 0) {
            yield_link(lease);                    // a fetch that is using the link goes first
            s_tile = atomicAdd(next, 1ull);
        }
        __syncthreads();
        const uint64_t t = s_tile;
        __syncthreads();                          // all have read it before thread 0 writes the next one
        if (t >= n_tiles) return;
        body(t);
    }
}

__global__ __launch_bounds__(WG) void copy_items(const Item *__restrict__ items, uint32_t n_items, uint64_t chunk_bytes,
                                                 uint32_t tiles_per_chunk, unsigned long long *next,
                                                 const unsigned long long *lease)
{
    for_each_tile(next, (uint64_t)n_items * tiles_per_chunk, lease, [&](uint64_t t) {
        uint64_t it = t / tiles_per_chunk;
        uint64_t off = (t - it * tiles_per_chunk) * TILE_HOST;
        Item x = items[it];
        copy_tile<WG, UNROLL_HOST, false>(x.src + off, x.dst + off, chunk_bytes - off, threadIdx.x);
    });
}

// One source, one or two destinations (dst == 0: none): the write-back path reads each source byte once.
__global__ __launch_bounds__(WG) void copy_items2(const Item2 *__restrict__ items, uint32_t n_items,
                                                  uint64_t chunk_bytes, uint32_t tiles_per_chunk, unsigned long long *next,
                                                  const unsigned long long *lease)
{
    constexpr uint32_t TILE = TILE_HOST;
    for_each_tile(next, (uint64_t)n_items * tiles_per_chunk, lease, [&](uint64_t t) {
        uint64_t it = t / tiles_per_chunk;
        uint64_t off = (t - it * tiles_per_chunk) * TILE;
        Item2 x = items[it];
        uint64_t len = chunk_bytes - off;
        if (len > TILE) len = TILE;
        const u32x4 *s = reinterpret_cast<const u32x4 *>(x.src + off);
        u32x4 *d0 = reinterpret_cast<u32x4 *>(x.dst0 + off);
        u32x4 *d1 = reinterpret_cast<u32x4 *>(x.dst1 + off);
        if (len == TILE) {                       // whole tile: all loads in flight, then the stores
            u32x4 v[UNROLL_HOST];
#pragma unroll
            for (int i = 0; i < UNROLL_HOST; ++i) v[i] = ld16<false>(s + threadIdx.x + i * WG);
            if (x.dst0) {
#pragma unroll
                for (int i = 0; i < UNROLL_HOST; ++i) st16<false>(d0 + threadIdx.x + i * WG, v[i]);
            }
            if (x.dst1) {
#pragma unroll
                for (int i = 0; i < UNROLL_HOST; ++i) st16<false>(d1 + threadIdx.x + i * WG, v[i]);
            }
        } else {
            uint32_t n_vec = (uint32_t)(len >> 4);
            for (uint32_t i = threadIdx.x; i < n_vec; i += WG) {
                u32x4 v = ld16<false>(s + i);
                if (x.dst0) st16<false>(d0 + i, v);
                if (x.dst1) st16<false>(d1 + i, v);
            }
        }
    });
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
        for (uint32_t i = threadIdx.x; i < n_vec; i += WG) st16<false>(d + i, v);
    }
}

// The same three between HBM pools only (placement from a staged copy, poisoning, demotion of lossy objects): nothing
// crosses PCIe, so they take the HBM-tier gather's shape - one wavefront per workgroup, one 1 KiB tile each,
// non-temporal accesses - instead of the few fat persistent workgroups that suit the link (measured on 17 GB of
// staged experts: 4.99 TB/s in the persistent form).  Tile numbers are 32-bit: the host checks n_items * tiles_per_chunk.
template <int NTHR>
__global__ __launch_bounds__(NTHR) void copy_items_hbm(const Item *__restrict__ items, uint32_t n_items,
                                                       uint64_t chunk_bytes, uint32_t tiles_per_chunk)
{
    constexpr uint32_t TILE = NTHR * 16;
    uint32_t n_tiles = n_items * tiles_per_chunk;
    for (uint32_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        uint32_t it = t / tiles_per_chunk;
        uint64_t off = (uint64_t)(t - it * tiles_per_chunk) * TILE;
        Item x = items[it];
        copy_tile<NTHR, 1, true>(x.src + off, x.dst + off, chunk_bytes - off, threadIdx.x);
        if (n_tiles - t <= gridDim.x) break;
    }
}

template <int NTHR>
__global__ __launch_bounds__(NTHR) void copy_items2_hbm(const Item2 *__restrict__ items, uint32_t n_items,
                                                        uint64_t chunk_bytes, uint32_t tiles_per_chunk)
{
    constexpr uint32_t TILE = NTHR * 16;
    uint32_t n_tiles = n_items * tiles_per_chunk;
    for (uint32_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        uint32_t it = t / tiles_per_chunk;
        uint64_t off = (uint64_t)(t - it * tiles_per_chunk) * TILE;
        Item2 x = items[it];
        uint64_t len = chunk_bytes - off;
        uint32_t n_vec = (uint32_t)((len > TILE ? TILE : len) >> 4);
        if (threadIdx.x < n_vec) {
            u32x4 v = ld16<true>(reinterpret_cast<const u32x4 *>(x.src + off) + threadIdx.x);
            if (x.dst0) st16<true>(reinterpret_cast<u32x4 *>(x.dst0 + off) + threadIdx.x, v);
            if (x.dst1) st16<true>(reinterpret_cast<u32x4 *>(x.dst1 + off) + threadIdx.x, v);
        }
        if (n_tiles - t <= gridDim.x) break;
    }
}

template <int NTHR>
__global__ __launch_bounds__(NTHR) void fill_items_hbm(const Item *__restrict__ items, uint32_t n_items,
                                                       uint64_t chunk_bytes, uint32_t tiles_per_chunk, uint32_t pattern)
{
    constexpr uint32_t TILE = NTHR * 16;
    uint32_t n_tiles = n_items * tiles_per_chunk;
    u32x4 v = { pattern, pattern, pattern, pattern };
    for (uint32_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        uint32_t it = t / tiles_per_chunk;
        uint64_t off = (uint64_t)(t - it * tiles_per_chunk) * TILE;
        uint64_t len = chunk_bytes - off;
        uint32_t n_vec = (uint32_t)((len > TILE ? TILE : len) >> 4);
        if (threadIdx.x < n_vec) st16<true>(reinterpret_cast<u32x4 *>(items[it].dst + off) + threadIdx.x, v);
        if (n_tiles - t <= gridDim.x) break;
    }
}

__global__ __launch_bounds__(WG) void dir_write(uint64_t *dir, const uint32_t *__restrict__ ids,
                                                const uint64_t *__restrict__ entries, uint32_t n)
{
    uint32_t i = blockIdx.x * WG + threadIdx.x;
    if (i < n) dir[ids[i]] = entries[i];
}

// A fetch repeated from the lists of the one before it serves the same requests again: they are added to the running totals.
__global__ void repeat_totals(const uint32_t *__restrict__ cnt, unsigned long long *totals)
{
    uint32_t i = threadIdx.x;
    if (i <= C_INVALID && cnt[i]) atomicAdd(&totals[i], (unsigned long long)cnt[i]);
}

// The counters of a fetch, as harvest_fetch_kv_static hands them to its caller: requests, local, cache, host, lost,
// invalid, length of the miss list, 0.  any == 0: the fetch had no table cell and ran no kernel - all zero.
__global__ void export_info(const uint32_t *__restrict__ cnt, uint32_t *__restrict__ info, uint32_t any)
{
    uint32_t i = threadIdx.x;
    if (i < 8) info[i] = !any ? 0u : (i <= C_INVALID ? cnt[i] : (i == 6 ? cnt[C_MISS] : 0u));
}

// Plain contiguous copy with the HBM-tier inner loop (reference ceiling / counter calibration).
template <int NTHR>
__global__ __launch_bounds__(NTHR) void plain_copy(uint64_t dst, uint64_t src, uint64_t bytes)
{
    constexpr uint32_t TILE = NTHR * 16;
    uint64_t n_tiles = (bytes + TILE - 1) / TILE;
    for (uint64_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        uint64_t off = t * TILE;
        copy_tile<NTHR, 1, true>(src + off, dst + off, bytes - off, threadIdx.x);
    }
}

// Read-only and write-only streams (one non-temporal 16-byte access per thread): what the memory system delivers in each
// direction alone, from which the bound of any copy follows.  With one-wavefront workgroups these two measure the
// dispatcher instead (one access per workgroup: 4.8 TB/s, 4.7 G workgroups/s), so the host launches them with the
// workgroup size that was measured fastest: 1024 threads for reads (7.5 TB/s), 256 for writes (6.7 TB/s).
template <int NTHR>
__global__ __launch_bounds__(NTHR) void plain_read(uint64_t src, uint64_t bytes, uint32_t *sink)
{
    constexpr uint32_t TILE = NTHR * 16;
    uint64_t n_vec = bytes >> 4;
    uint32_t acc = 0;
    for (uint64_t t = blockIdx.x; t * (TILE / 16) < n_vec; t += gridDim.x) {
        uint64_t i = t * (TILE / 16) + threadIdx.x;
        if (i < n_vec) {
            u32x4 v = ld16<true>(reinterpret_cast<const u32x4 *>(src) + i);
            acc ^= v.x ^ v.y ^ v.z ^ v.w;
        }
    }
    if (acc == 0x9E3779B9u) *sink = acc;             // never true for the calibration buffers: keeps the loads alive
}

template <int NTHR>
__global__ __launch_bounds__(NTHR) void plain_write(uint64_t dst, uint64_t bytes, uint32_t pattern)
{
    constexpr uint32_t TILE = NTHR * 16;
    uint64_t n_vec = bytes >> 4;
    u32x4 v = { pattern, pattern, pattern, pattern };
    for (uint64_t t = blockIdx.x; t * (TILE / 16) < n_vec; t += gridDim.x) {
        uint64_t i = t * (TILE / 16) + threadIdx.x;
        if (i < n_vec) st16<true>(reinterpret_cast<u32x4 *>(dst) + i, v);
    }
}

}  // namespace hv
