"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.
Everything is byte work, so the bar is bit-exact (numpy.array_equal on raw bytes) for payload, directory entries,
statuses, counts and (sorted) miss lists."""
import sys

import numpy as np
import pytest

import workloads as W
from workloads import scenarios as S
import parity as P

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


# ---- config 1: tiny KV fetch, scatter back, round trip ------------------------------------------------------

LAYOUTS = pytest.mark.parametrize("adjacent", [False, True], ids=["k-pool-and-v-pool", "k-v-adjacent"])


@LAYOUTS
@pytest.mark.parametrize("general", [False, True], ids=["one-kernel", "general"])
@pytest.mark.parametrize("fill", [W.FILL_NORMAL, W.FILL_TAG])
def test_config1_tiny_kv_fetch_and_round_trip(fill, general, adjacent):
    say(f"config1 fill={fill}")
    wl = W.kv_tiny(0, fill_mode=fill)
    eo, eh = P.make_engines(wl, hip_kwargs=dict(general_fetch=general, cache_planes_adjacent=adjacent))
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        assert np.array_equal(ro.place_status, rh.place_status) and (rh.place_status == 0).all()
        P.assert_dirs_equal(eo, eh, S.KV, wl.n_objects, "after place")
        P.assert_tiers_equal(eo, eh, S.KV, 2, tiers=(S.HOST, S.CACHE), what="after place")
        a, b = ro.fetch(0), rh.fetch(0)
        P.assert_kv_equal(a, b, "config1 fetch")
        assert b[3]["n_cache"] + b[3]["n_host"] == 256 and b[3]["n_invalid"] == 0
        if fill == W.FILL_TAG:                                  # no reference buffer needed at all
            chunk = wl.shape.chunk_bytes
            flat = np.concatenate(wl.tables)
            for j, blk in enumerate(flat):
                assert W.check_tag(b[0][j * chunk:(j + 1) * chunk], 0, W.CLS_KV, 0, 0, int(blk))
                assert W.check_tag(b[1][j * chunk:(j + 1) * chunk], 0, W.CLS_KV, 1, 0, int(blk))
        # scatter the gathered bytes back: every tier must be unchanged
        ids = np.concatenate(wl.tables).astype(np.uint32)
        for e, r in ((eo, a), (eh, b)):
            e.evict(S.KV, 0, ids, r[0], r[1], np.arange(256), 256)
        P.assert_tiers_equal(eo, eh, S.KV, 2, tiers=(S.HOST, S.CACHE), what="after identity evict")
        P.assert_kv_equal(a, rh.fetch(0), "fetch after identity evict")
        # scatter new bytes, gather them again
        g = W.rng(0, 500)
        yk = g.integers(0, 256, size=a[0].size, dtype=np.uint8)
        yv = g.integers(0, 256, size=a[0].size, dtype=np.uint8)
        for e in (eo, eh):
            e.evict(S.KV, 0, ids, yk, yv, np.arange(256), 256)
        c, d = ro.fetch(0), rh.fetch(0)
        P.assert_kv_equal(c, d, "fetch after evict of new bytes")
        assert np.array_equal(d[0], yk) and np.array_equal(d[1], yv)
        P.assert_tiers_equal(eo, eh, S.KV, 2, tiers=(S.HOST, S.CACHE), what="after evict of new bytes")
    finally:
        eh.close(); eo.close()


# ---- tier independence on the GPU -----------------------------------------------------------------------------

@pytest.mark.parametrize("general", [False, True], ids=["one-kernel", "general"])
@pytest.mark.parametrize("p_cache", [0.0, 0.35, 1.0])
def test_fetch_is_the_same_for_every_residency(p_cache, general):
    say(f"residency p={p_cache}")
    wl = W.kv_decode(seed=1, n_layers=2, n_seq=3, min_len=300, max_len=900, p_cache=p_cache, n_steps=1)
    ref = W.kv_decode(seed=1, n_layers=2, n_seq=3, min_len=300, max_len=900, p_cache=0.5, n_steps=1)
    eo, eh = P.make_engines(wl, hip_kwargs=dict(general_fetch=general))
    eo2, _unused = None, None
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        for layer in range(2):
            a, b = ro.fetch(layer), rh.fetch(layer)
            P.assert_kv_equal(a, b, f"p={p_cache} layer {layer}")
            if p_cache == 0.0:
                assert b[3]["n_cache"] == 0
            if p_cache == 1.0:
                assert b[3]["n_host"] == 0 and b[2].size == 0
        assert all(np.array_equal(x, y) for x, y in zip(wl.tables, ref.tables))   # same requests, other residency
    finally:
        eh.close(); eo.close()


# ---- config 2, small: decode steps with append, write-back, demotion, placement -------------------------------

@LAYOUTS
@pytest.mark.parametrize("general", [False, True], ids=["one-kernel", "general"])
def test_kv_decode_steps_small(general, adjacent):
    say("kv decode small")
    wl = W.kv_decode(seed=2, n_layers=3, n_seq=4, min_len=500, max_len=2000, n_steps=40)
    eo, eh = P.make_engines(wl, hip_kwargs=dict(general_fetch=general, cache_planes_adjacent=adjacent))
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        for t in range(40):
            P.assert_kv_equal(ro.step(t), rh.step(t), f"decode step {t}")
        P.assert_dirs_equal(eo, eh, S.KV, wl.n_objects, "after 40 steps")
        P.assert_tiers_equal(eo, eh, S.KV, 2, what="after 40 steps")
        st = eh.h.stats()
        assert st.n_demoted[0] == sum(len(f) for f in wl.future_blocks) and st.fetch[0].n_invalid == 0
    finally:
        eh.close(); eo.close()


def test_fetch_sizes_that_jump_between_calls():
    """The gather's grid is sized from what the previous fetch on the stream reported: a fetch far larger than the one
    before runs on a grid far too short and has to loop, one far smaller finds most of its grid empty."""
    say("jumping fetch sizes")
    wl = W.kv_decode(seed=31, n_layers=2, n_seq=3, min_len=12000, max_len=24000, p_cache=0.8, n_steps=1)
    eo, eh = P.make_engines(wl, hip_kwargs=dict(general_fetch=True))          # the path whose grids are sized that way
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        table, nb = rh.table_arrays()
        assert int(nb.sum()) * wl.shape.chunk_bytes // 4096 > 5 * 16 * 256          # several times the grid's floor
        tiny = np.minimum(nb, [2, 0, 1]).astype(np.int32)
        heads, tokens = wl.shape.n_kv_heads, wl.shape.block_tokens
        caps = np.diff(np.append(rh.seq_dst_block, rh.cap).astype(np.int64)).astype(np.uint32)   # blocks per sequence
        for i, n in enumerate((tiny, nb, tiny, nb // 2, nb, tiny)):
            P.assert_kv_equal(eo.fetch_kv(i % 2, table, n, ro.seq_dst_block, ro.cap),
                              eh.fetch_kv(i % 2, table, n, rh.seq_dst_block, rh.cap), f"token-major call {i}")
            P.assert_kv_equal(eo.fetch_kv_head_major(i % 2, table, n, ro.seq_dst_block, caps, ro.cap, heads, tokens),
                              eh.fetch_kv_head_major(i % 2, table, n, rh.seq_dst_block, caps, rh.cap, heads, tokens),
                              f"head-major call {i}")
    finally:
        eh.close(); eo.close()


def test_block_table_large_enough_for_the_grouped_compaction():
    """More than 262 144 table cells: the compaction takes its three-kernel form (workgroup totals are grouped before they
    are added up).  Sparse rows, empty rows, one full row, invalid ids and a row that runs past the destination."""
    say("large block table")
    wl = W.kv_decode(seed=35, n_layers=2, n_seq=3, min_len=3000, max_len=6000, p_cache=0.6, n_steps=1)
    eo, eh = P.make_engines(wl)
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        g = W.rng(35, 9)
        n_seq, max_blocks = 41, 8192
        assert n_seq * max_blocks > 1024 * 256
        table = g.integers(0, wl.n_closed, size=(n_seq, max_blocks)).astype(np.int32)
        table[g.random(table.shape) < 0.001] = -7                                # unknown ids here and there
        table[5, 17] = wl.n_objects + 100
        nb = g.integers(0, 300, size=n_seq).astype(np.int32)
        nb[3], nb[11], nb[29], nb[40] = 0, max_blocks, 0, 1
        sdb = np.concatenate([[0], np.cumsum(nb)[:-1]]).astype(np.uint64)
        cap = int(nb.sum()) - 40                                                 # the last rows do not fit entirely
        for layer in range(2):
            a = eo.fetch_kv(layer, table, nb, sdb, cap)
            b = eh.fetch_kv(layer, table, nb, sdb, cap)
            P.assert_kv_equal(a, b, f"large table, layer {layer}")
            assert b[3]["n_invalid"] > 40 and b[3]["n_requests"] == int(nb.sum())
        caps = nb.astype(np.uint32)
        a = eo.fetch_kv_head_major(0, table, nb, sdb, caps, int(nb.sum()), wl.shape.n_kv_heads, wl.shape.block_tokens)
        b = eh.fetch_kv_head_major(0, table, nb, sdb, caps, int(nb.sum()), wl.shape.n_kv_heads, wl.shape.block_tokens)
        P.assert_kv_equal(a, b, "large table, head-major")
    finally:
        eh.close(); eo.close()


# ---- chunk sizes that are not a multiple of the 32 KiB tile -----------------------------------------------------

@pytest.mark.parametrize("heads,dim,tokens,elt", [(1, 8, 1, 2), (3, 8, 16, 2), (8, 129 - 1, 16, 2), (8, 136, 16, 2),
                                                  (5, 200, 48, 2), (8, 128, 16, 1), (8, 128, 16, 4), (2, 80, 16, 1)])
@pytest.mark.parametrize("general,threads,adjacent", [(False, 0, False), (True, 0, False), (True, 0, True), (True, 128, True),
                                                      (True, 256, False)],
                         ids=["one-kernel", "general", "general-adjacent", "general-128-threads-adjacent", "general-256-threads"])
def test_ragged_chunk_sizes(heads, dim, tokens, elt, general, threads, adjacent):
    """Block sizes off the 1 KiB / 4 KiB / 32 KiB tiles, and the element sizes of fp8, fp16 / bf16 and fp32 KV caches; the
    gather with one, two and four wavefronts per workgroup, plane after plane and both planes of a request in one pass."""
    shape = W.KVShape(n_layers=2, block_tokens=tokens, n_kv_heads=heads, head_dim=dim, elt_bytes=elt)
    say(f"ragged chunk {shape.chunk_bytes} bytes")
    wl = W.kv_decode(seed=4, n_seq=3, min_len=20 * tokens, max_len=60 * tokens, n_steps=2 * tokens, shape=shape,
                     fill_mode=W.FILL_TAG)
    eo, eh = P.make_engines(wl, hip_kwargs=dict(general_fetch=general, gather_threads=threads, cache_planes_adjacent=adjacent))
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        for t in range(2 * tokens):
            P.assert_kv_equal(ro.step(t), rh.step(t), f"chunk {shape.chunk_bytes} step {t}")
        P.assert_tiers_equal(eo, eh, S.KV, 2, what=f"chunk {shape.chunk_bytes}")
    finally:
        eh.close(); eo.close()


@pytest.mark.parametrize("pcie_wgs", [1, 5, 300])
@pytest.mark.parametrize("heads,dim,tokens", [(5, 200, 48), (8, 128, 16)])
def test_pcie_copies_with_any_number_of_workgroups(pcie_wgs, heads, dim, tokens):
    """Placements and write-backs count their tiles out to however many persistent workgroups the context was given:
    one, a few, more than there are tiles; 93.75 KiB chunks (two whole 32 KiB tiles and a ragged third) and 32 KiB ones."""
    shape = W.KVShape(n_layers=2, block_tokens=tokens, n_kv_heads=heads, head_dim=dim, elt_bytes=2)
    say(f"pcie copies with {pcie_wgs} workgroups, chunk {shape.chunk_bytes} bytes")
    wl = W.kv_decode(seed=6, n_seq=3, min_len=20 * tokens, max_len=60 * tokens, n_steps=2 * tokens, shape=shape,
                     fill_mode=W.FILL_TAG)
    eo, eh = P.make_engines(wl, poison=True, hip_kwargs=dict(pcie_wgs=pcie_wgs))
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        for t in range(2 * tokens):                              # roll-overs: write-back, placement, registration
            P.assert_kv_equal(ro.step(t), rh.step(t), f"step {t}")
        a, b = ro.revoke_quarter(0), rh.revoke_quarter(0)        # and one larger batch each way
        assert np.array_equal(a[0], b[0]) and len(a[0]) > 0
        assert np.array_equal(ro.replace_revoked(), rh.replace_revoked())
        P.assert_kv_equal(ro.fetch(1), rh.fetch(1), "after re-placing")
        P.assert_dirs_equal(eo, eh, S.KV, wl.n_objects)
        P.assert_tiers_equal(eo, eh, S.KV, 2, what=f"{pcie_wgs} workgroups")
    finally:
        eh.close(); eo.close()


# ---- degenerate requests ----------------------------------------------------------------------------------------

@pytest.mark.parametrize("general", [False, True], ids=["one-kernel", "general"])
def test_empty_invalid_duplicate_and_overflowing_requests(general):
    say("edge cases")
    wl = W.kv_decode(seed=5, n_layers=1, n_seq=2, min_len=64, max_len=128, n_steps=1, fill_mode=W.FILL_TAG)
    eo, eh = P.make_engines(wl, hip_kwargs=dict(general_fetch=general))
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        n = wl.n_closed
        sdb = np.array([0, 6], np.uint64)
        cases = {
            "all empty": (np.zeros((2, 5), np.int32), np.array([0, 0], np.int32), sdb, 12),
            "negative and oversized n_blocks": (np.arange(10, dtype=np.int32).reshape(2, 5) % n,
                                                np.array([-3, 99], np.int32), sdb, 12),
            "unknown and negative ids": (np.array([[0, -1, 2, 10 ** 6, 1], [n + 50, 1, 1, 1, 0]], np.int32),
                                         np.array([5, 5], np.int32), sdb, 12),
            "duplicates": (np.full((2, 5), 3, np.int32), np.array([5, 4], np.int32), sdb, 12),
            "destination overflow": (np.arange(10, dtype=np.int32).reshape(2, 5) % n, np.array([5, 5], np.int32),
                                     np.array([0, 9], np.uint64), 12),
        }
        for name, (table, nb, s, cap) in cases.items():
            say(f"  {name}")
            a = eo.c[S.KV].fetch_kv(0, table, nb, s, cap, dst_k=np.full(cap * wl.shape.chunk_bytes, 0xEE, np.uint8),
                                    dst_v=np.full(cap * wl.shape.chunk_bytes, 0xEE, np.uint8))
            a = (a[0], a[1], np.sort(a[2]), a[3])
            b = eh.fetch_kv(0, table, nb, s, cap, dst_fill=0xEE)
            P.assert_kv_equal(a, b, name)
        # no sequences at all
        eh.h.fetch_kv(0, __import__("torch").zeros((0, 4), dtype=__import__("torch").int32, device="cuda"),
                      None, None, None, None, 0)
        counts, miss, n_miss = eh.h.fetch_info()
        assert counts["n_requests"] == 0 and n_miss == 0
    finally:
        eh.close(); eo.close()


# ---- config 3, small: expert fetch with local / cached / host experts -------------------------------------------

def test_expert_fetch_small():
    say("experts small")
    sh = W.ExpertShape(n_layers=4, n_experts=16, d_model=64, d_ff=100)          # 38 400-byte experts: ragged tiles
    ex = W.expert_offload(seed=6, shape=sh, n_tokens=64)
    eo, eh = P.make_engines(ex_wl=ex)
    try:
        xo, xh = S.ExpertRun(eo, ex), S.ExpertRun(eh, ex)
        assert np.array_equal(xo.place_status, xh.place_status)
        for t in range(3):
            for layer in range(4):
                a, b = xo.fetch(t, layer), xh.fetch(t, layer)
                P.assert_experts_equal(a, b, f"experts step {t} layer {layer}")
                U = sorted(set(int(e) for e in ex.routing(t, layer).reshape(-1)))
                assert [e for e in range(16) if b[0][e] is not None] == U
        # staging too small, ids out of range
        topk = np.array([[0, 1], [2, 3], [4, 5], [-7, 16], [6, 7]], np.int32)
        for n_staging in (0, 2, 16):
            a = eo.fetch_experts(1, topk, n_staging)
            b = eh.fetch_experts(1, topk, n_staging)
            P.assert_experts_equal(a, b, f"staging {n_staging}")
        none = np.zeros((0, 2), np.int32)                                      # a batch without tokens: nothing is routed
        a, b = eo.fetch_experts(2, none, 16), eh.fetch_experts(2, none, 16)
        P.assert_experts_equal(a, b, "no tokens")
        assert b[4]["n_requests"] == 0 and all(x is None for x in b[0])
        P.assert_dirs_equal(eo, eh, S.EXPERT, ex.n_objects)
    finally:
        eh.close(); eo.close()


# ---- config 4, small: cache tier driven by an LRU policy --------------------------------------------------------

def test_expert_fetch_with_a_very_large_batch_of_routing_ids():
    """More than 32 768 routing ids: the routed set is marked by many workgroups before the resolving workgroup runs.
    Every call must see its own routing only (the marks are cleared on the way), invalid ids are counted."""
    say("experts, large batch")
    ex = W.expert_offload(seed=37, shape=W.ExpertShape(n_layers=2, n_experts=48, d_model=64, d_ff=100), n_tokens=64)
    eo, eh = P.make_engines(ex_wl=ex, poison=True)
    try:
        xo, xh = S.ExpertRun(eo, ex), S.ExpertRun(eh, ex)
        g = W.rng(37, 3)
        everything = g.integers(0, 48, size=(30000, 4)).astype(np.int32)
        everything[g.random(everything.shape) < 0.0005] = 48 + 5                      # a few ids no expert has
        everything[17, 2] = -1
        few = g.choice(np.arange(0, 48, 3), size=(20000, 2)).astype(np.int32)         # every third expert only
        small = ex.routing(0, 1)
        for i, (layer, topk) in enumerate(((0, everything), (1, few), (1, small), (0, few), (1, everything))):
            a, b = eo.fetch_experts(layer, topk, 48), eh.fetch_experts(layer, topk, 48)
            P.assert_experts_equal(a, b, f"large batch, call {i}")
            assert b[4]["n_invalid"] == int(((topk < 0) | (topk >= 48)).sum())
        assert eh.fetch_experts(1, few, 48)[4]["n_requests"] == len(np.unique(few))
    finally:
        eh.close(); eo.close()


@pytest.mark.parametrize("from_staging", [False, True])
def test_expert_lru_small(from_staging):
    """from_staging: experts that enter the cache tier are copied from the staging buffer the fetch has just filled
    (harvest_place_from), those the buffer had no room for from their host copies; 30 staging slots force both."""
    say(f"experts lru small, from_staging={from_staging}")
    sh = W.ExpertShape(n_layers=3, n_experts=60, d_model=32, d_ff=44)
    ex = W.expert_lru(seed=7, shape=sh, n_tokens=24, top_k=4)
    eo, eh = P.make_engines(ex_wl=ex, poison=True)
    try:
        n_staging = 30 if from_staging else None
        xo, xh = S.ExpertRun(eo, ex, n_staging=n_staging), S.ExpertRun(eh, ex, n_staging=n_staging)
        hits = 0
        for t in range(6):
            for layer in range(3):
                a, b = xo.fetch(t, layer), xh.fetch(t, layer)
                P.assert_experts_equal(a, b, f"lru step {t} layer {layer}")
                hits += b[4]["n_cache"]
                ua, ub = xo.lru_update(t, layer, from_staging), xh.lru_update(t, layer, from_staging)
                assert ua[0] == ub[0] and ua[1] == ub[1] and ua[2] == ub[2] and np.array_equal(ua[3], ub[3])
        assert hits > 0
        P.assert_dirs_equal(eo, eh, S.EXPERT, ex.n_objects)
        P.assert_tiers_equal(eo, eh, S.EXPERT, 1, tiers=(S.CACHE,), what="lru cache pool (poisoned slots included)")
    finally:
        eh.close(); eo.close()


def test_place_from_device_memory_kv_all_layers():
    """harvest_place_from on a two-plane, three-layer class, with source bytes unlike any host copy: the cache tier must
    hold exactly the named source blocks, the host pool must stay as it was, fetches serve the new bytes until the
    objects are revoked and the host bytes afterwards.  Equal-size slots and best-fit segments."""
    say("place_from, kv")
    for shared, adjacent in ((0, False), (1, False), (0, True)):
        wl = W.kv_decode(seed=33, n_layers=3, n_seq=2, min_len=200, max_len=400, p_cache=0.0, n_steps=1)
        nbytes = 64 * 256 * 3 * 2 * wl.shape.chunk_bytes // 64 if shared else 0
        eo, eh = P.make_engines(wl, poison=True, cache_slack=16, shared_cache_bytes=nbytes, shared_granule=256 if shared else 0,
                                hip_kwargs=dict(cache_planes_adjacent=adjacent))
        try:
            ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
            chunk, stride = wl.shape.chunk_bytes, 7
            g = W.rng(33, 5)
            src = [g.integers(0, 256, size=3 * stride * chunk, dtype=np.uint8) for _ in range(2)]
            host_before = [eh.tier_plane(S.KV, S.HOST, p).copy() for p in range(2)]
            ids, blk = [5, 2, 9, 2, 11], [6, 0, 3, 1, 3]                     # a repeat: the second mention is a no-op
            a = eo.place_from(S.KV, ids, src[0], src[1], blk, stride)
            b = eh.place_from(S.KV, ids, src[0], src[1], blk, stride)
            assert np.array_equal(a, b) and list(b) == [0] * 5
            P.assert_dirs_equal(eo, eh, S.KV, wl.n_objects)
            if shared:
                P.assert_shared_pools_equal(eo, eh, "after place_from")
            else:
                P.assert_tiers_equal(eo, eh, S.KV, 2, tiers=(S.CACHE,), what="after place_from")
            assert all(np.array_equal(eh.tier_plane(S.KV, S.HOST, p), host_before[p]) for p in range(2))
            for layer in range(3):
                P.assert_kv_equal(ro.fetch(layer), rh.fetch(layer), f"after place_from, layer {layer}")
            assert eo.revoke(S.KV, [5, 9]) == eh.revoke(S.KV, [5, 9]) == [5, 9]
            for layer in range(3):
                P.assert_kv_equal(ro.fetch(layer), rh.fetch(layer), f"after revocation, layer {layer}")
            for bad_ids, bad_blk in (([0, 10 ** 6], [0, 0]), ([0, 1], [0, stride])):
                with pytest.raises(Exception):
                    eh.place_from(S.KV, bad_ids, src[0], src[1], bad_blk, stride)
                assert eh.lookup(S.KV, 0)[0] == S.HOST
        finally:
            eh.close(); eo.close()


# ---- config 5, small: KV and experts on two streams with periodic revocation -------------------------------------

N_STRESS = 500          # the step count of the revocation-stress configuration


@pytest.mark.parametrize("general", [False, True], ids=["one-kernel", "general"])
@pytest.mark.parametrize("overlap_revoke", [False, True])
def test_revocation_stress_two_streams(overlap_revoke, general):
    say(f"revocation stress overlap={overlap_revoke}")
    wl = W.kv_decode(seed=8, n_layers=2, n_seq=3, min_len=400, max_len=1200, n_steps=N_STRESS)
    sh = W.ExpertShape(n_layers=2, n_experts=16, d_model=64, d_ff=100)
    ex = W.expert_offload(seed=8, shape=sh, n_tokens=64)
    # (the runs with overlapping revocations also keep K and V of a block side by side in the cache tier)
    eo, eh = P.make_engines(wl, ex, poison=True, two_streams=True,
                            hip_kwargs=dict(general_fetch=general, cache_planes_adjacent=overlap_revoke))
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        xo, xh = S.ExpertRun(eo, ex), S.ExpertRun(eh, ex)
        n_revoked = 0
        for t in range(N_STRESS):
            layer = t % 2
            revoke_now = t % 10 == 0 and t > 0
            ha, hx = rh.fetch_begin(layer), xh.fetch_begin(t, layer)          # both in flight on their own streams
            a, x = ro.fetch(layer), xo.fetch(t, layer)
            if revoke_now and overlap_revoke:                                 # revoke while the fetches are in flight
                rk_o, rk_h = ro.revoke_quarter(t), rh.revoke_quarter(t)
                rx_o, rx_h = xo.revoke_quarter(t), xh.revoke_quarter(t)
            b, y = eh.fetch_end(ha), eh.fetch_end(hx)
            racy = revoke_now and overlap_revoke      # such a fetch may have resolved before or after the revocation
            P.assert_kv_equal(a, b, f"stress kv step {t}", counts=not racy)
            P.assert_experts_equal(x, y, f"stress experts step {t}", counts=not racy)
            if revoke_now and not overlap_revoke:
                rk_o, rk_h = ro.revoke_quarter(t), rh.revoke_quarter(t)
                rx_o, rx_h = xo.revoke_quarter(t), xh.revoke_quarter(t)
            if revoke_now:
                assert np.array_equal(rk_o[0], rk_h[0]) and rk_o[1] == rk_h[1] == [int(i) for i in rk_o[0]]
                assert np.array_equal(rx_o[0], rx_h[0]) and rx_o[1] == rx_h[1]
                n_revoked += len(rk_o[0]) + len(rx_o[0])
            if t % 10 == 5:
                assert np.array_equal(ro.replace_revoked(), rh.replace_revoked())
                assert np.array_equal(xo.replace_revoked(), xh.replace_revoked())
            ro.append(t); rh.append(t)
        assert n_revoked > 20 * N_STRESS // 60
        P.assert_dirs_equal(eo, eh, S.KV, wl.n_objects)
        P.assert_dirs_equal(eo, eh, S.EXPERT, ex.n_objects)
        P.assert_tiers_equal(eo, eh, S.KV, 2, what="stress kv")
        P.assert_tiers_equal(eo, eh, S.EXPERT, 1, what="stress experts")
    finally:
        eh.close(); eo.close()


def test_two_threads_drive_one_context():
    """One host thread per class, each on its own stream, revoking and re-placing as it goes: every call runs under the
    context's lock, a revocation of one class drains the other class's stream too, and no result changes."""
    import threading
    say("two threads")
    n_steps = 120
    wl = W.kv_decode(seed=29, n_layers=2, n_seq=3, min_len=400, max_len=1200, n_steps=n_steps)
    ex = W.expert_offload(seed=29, shape=W.ExpertShape(n_layers=2, n_experts=16, d_model=64, d_ff=100), n_tokens=64)
    eo, eh = P.make_engines(wl, ex, poison=True, two_streams=True)
    errors = []

    def kv_side():
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        for t in range(n_steps):
            P.assert_kv_equal(ro.fetch(t % 2), rh.fetch(t % 2), f"threads kv step {t}")
            if t % 10 == 0 and t > 0:
                a, b = ro.revoke_quarter(t), rh.revoke_quarter(t)
                assert np.array_equal(a[0], b[0]) and a[1] == b[1]
            if t % 10 == 5:
                assert np.array_equal(ro.replace_revoked(), rh.replace_revoked())
            ro.append(t); rh.append(t)

    def expert_side():
        xo, xh = S.ExpertRun(eo, ex), S.ExpertRun(eh, ex)
        for t in range(n_steps):
            P.assert_experts_equal(xo.fetch(t, t % 2), xh.fetch(t, t % 2), f"threads experts step {t}")
            if t % 7 == 0 and t > 0:
                a, b = xo.revoke_quarter(t), xh.revoke_quarter(t)
                assert np.array_equal(a[0], b[0]) and a[1] == b[1]
            if t % 7 == 3:
                assert np.array_equal(xo.replace_revoked(), xh.replace_revoked())

    def guarded(f):
        def run():
            try:
                f()
            except BaseException as e:                                     # reported by the main thread
                errors.append(e)
        return run

    try:
        threads = [threading.Thread(target=guarded(f)) for f in (kv_side, expert_side)]
        for th in threads:
            th.start()
        for th in threads:
            th.join(100)
            assert not th.is_alive(), "a thread did not finish"
        if errors:
            raise errors[0]
        P.assert_dirs_equal(eo, eh, S.KV, wl.n_objects)
        P.assert_dirs_equal(eo, eh, S.EXPERT, ex.n_objects)
        P.assert_tiers_equal(eo, eh, S.KV, 2, what="threads kv")
        P.assert_tiers_equal(eo, eh, S.EXPERT, 1, what="threads experts")
    finally:
        eh.close(); eo.close()


def test_a_revocation_waits_without_holding_up_the_other_thread():
    """The expert thread places several large experts (milliseconds of PCIe traffic queued on its stream) and at once
    revokes others, which has to wait for that queue to drain; the KV thread keeps fetching on its own stream meanwhile.
    The wait happens outside the context's lock: a third thread's directory lookups - calls that need the lock and
    nothing else - and fetch calls start and return while the revocation is still waiting.
    And each class orders its fetches after its own directory edits only: the KV fetches complete while the experts'
    placements - whose new entries are published behind their copies - are still in flight."""
    import threading
    import time
    import torch
    say("revocation without stalling the other thread")
    wl = W.kv_decode(seed=30, n_layers=1, n_seq=2, min_len=1500, max_len=2500, n_steps=1)
    ex = W.expert_offload(seed=30, shape=W.ExpertShape(n_layers=1, n_experts=16, d_model=4096, d_ff=4096), n_local=0)
    eo, eh = P.make_engines(wl, ex, poison=True, two_streams=True)
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        xo, xh = S.ExpertRun(eo, ex), S.ExpertRun(eh, ex)
        cached = sorted(xh.live)
        on_host = [i for i in range(ex.n_objects) if i not in xh.live]
        assert len(cached) >= 4 and len(on_host) >= 4
        half = cached[:len(cached) // 2]
        for e in (eo, eh):                                   # room in the cache tier for what will be placed
            e.revoke(S.EXPERT, half)
        table, nb = rh.table_arrays()
        dev = eh.dev
        d_table, d_nb = torch.from_numpy(table).to(dev), torch.from_numpy(nb).to(dev)
        d_sdb = torch.from_numpy(rh.seq_dst_block.view(np.int64)).to(dev)
        dst = [torch.zeros(rh.cap * wl.shape.chunk_bytes, dtype=torch.uint8, device=dev) for _ in range(2)]
        kv_stream = eh.streams[S.KV]
        with torch.cuda.stream(kv_stream):
            eh.h.fetch_kv(0, d_table, d_nb, dst[0], dst[1], d_sdb, rh.cap)          # the stream's scratch exists from here on
        independent, _ = P.streams_run_independently(dev, eh.streams[S.EXPERT], kv_stream)
        window, calls, looks, stop, errors = [], [], [], threading.Event(), []

        def kv_side():
            try:
                with torch.cuda.stream(kv_stream):
                    while not stop.is_set():
                        a = time.perf_counter()
                        eh.h.fetch_kv(0, d_table, d_nb, dst[0], dst[1], d_sdb, rh.cap)
                        b = time.perf_counter()
                        kv_stream.synchronize()
                        calls.append((a, b, time.perf_counter()))
            except BaseException as e:
                errors.append(e)

        def lookup_side():                                   # a call that only needs the context's lock, no device
            try:
                while not stop.is_set():
                    a = time.perf_counter()
                    eh.h.lookup(S.EXPERT, cached[0])
                    looks.append((a, time.perf_counter()))
                    time.sleep(2e-4)
            except BaseException as e:
                errors.append(e)

        threads = [threading.Thread(target=kv_side), threading.Thread(target=lookup_side)]
        for th in threads:
            th.start()
        time.sleep(0.02)
        n_place = min(len(half), len(on_host))
        st = eh.place(S.EXPERT, on_host[:n_place])            # ~100 MiB each over PCIe: milliseconds of queued work
        a = time.perf_counter()
        revoked = eh.revoke(S.EXPERT, cached[len(cached) // 2:])     # has to wait for the placements
        window = (a, time.perf_counter())
        stop.set()
        for th in threads:
            th.join(30)
            assert not th.is_alive()
        assert not errors, errors
        assert (st == 0).all() and len(revoked) == len(cached) - len(cached) // 2
        inside = [c for c in calls if c[0] > window[0] and c[1] < window[1]]
        looks_inside = [c for c in looks if c[0] > window[0] and c[1] < window[1]]
        from conftest import live
        live(f"  (the device runs the two streams independently: {independent})")
        live(f"  the revocation waited {1e3 * (window[1] - window[0]):.1f} ms; inside it {len(looks_inside)} lookups and "
             f"{len(inside)} KV fetch calls started and returned")
        live("  KV calls (start, returned, stream idle; ms after the revocation began): " + " ".join(
            f"({1e3 * (c[0] - a):.2f} {1e3 * (c[1] - a):.2f} {1e3 * (c[2] - a):.2f})" for c in calls if a < c[2])[:400])
        # Calls that took the lock and returned inside the window show that the lock was free during the wait: the lookups
        # need the lock and nothing of the device.  The KV fetches also need the device to run their stream while the
        # other one is busy - which it does as long as no stream of the library sits waiting in a hardware queue that the
        # KV stream shares (the drain is a wait of the host for that reason): they take their usual 0.15 ms each.
        assert window[1] - window[0] > 2e-3 and len(looks_inside) >= 5
        if independent:
            assert len(inside) >= 3
        # and nothing is wrong afterwards
        assert np.array_equal(eo.place(S.EXPERT, on_host[:n_place]), st)
        eo.revoke(S.EXPERT, cached[len(cached) // 2:])
        P.assert_kv_equal(ro.fetch(0), rh.fetch(0), "kv after the overlap")
        P.assert_experts_equal(xo.fetch(0, 0), xh.fetch(0, 0), "experts after the overlap")
        P.assert_dirs_equal(eo, eh, S.EXPERT, ex.n_objects)
    finally:
        eh.close(); eo.close()


def test_two_revocations_at_once_both_wait_for_the_work_in_flight():
    """A revocation takes each stream's latest-work event out of the stream's state while it waits.  A second revocation,
    started by another thread meanwhile, must wait for that work too: here a gather that reads cache slots (a repeat of
    an earlier fetch, so its lists name the slots already) is queued behind a sleeping kernel; one thread revokes experts
    - and takes the KV stream's event -, then the main thread revokes the very KV blocks the gather will read, with
    poisoning on.  The gather must still deliver the blocks' bytes, not the poison."""
    import threading
    import time
    import torch
    say("two revocations at once")
    wl = W.kv_decode(seed=35, n_layers=2, n_seq=2, min_len=5000, max_len=8000, p_cache=0.6, n_steps=1)
    ex = W.expert_offload(seed=35, shape=W.ExpertShape(n_layers=1, n_experts=8, d_model=256, d_ff=512), n_local=0)
    eo, eh = P.make_engines(wl, ex, poison=True, two_streams=True, hip_kwargs=dict(general_fetch=True))
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        xo, xh = S.ExpertRun(eo, ex), S.ExpertRun(eh, ex)
        want = ro.fetch(1)
        table, nb = rh.table_arrays()
        dev = eh.dev
        d_table, d_nb = torch.from_numpy(table).to(dev), torch.from_numpy(nb).to(dev)
        d_sdb = torch.from_numpy(rh.seq_dst_block.view(np.int64)).to(dev)
        dst = [torch.zeros(rh.cap * wl.shape.chunk_bytes, dtype=torch.uint8, device=dev) for _ in range(2)]
        kv_stream, x_stream = eh.streams[S.KV], eh.streams[S.EXPERT]
        P.assert_experts_equal(xo.fetch(0, 0), xh.fetch(0, 0), "experts before")      # the expert stream has work on record
        with torch.cuda.stream(kv_stream):
            eh.h.fetch_kv(0, d_table, d_nb, dst[0], dst[1], d_sdb, rh.cap)            # resolves: the lists name cache slots
        _, cycles = P.streams_run_independently(dev, kv_stream, x_stream, ms=150.0)        # (only the calibrated sleep is used)
        for t in dst:
            t.zero_()
        torch.cuda.synchronize()
        in_cache = [b for s in range(wl.n_seq) for b in rh.tables[s][:-1] if eh.lookup(S.KV, b)[0] == S.CACHE]
        assert len(in_cache) > 100
        with torch.cuda.stream(kv_stream):
            torch.cuda._sleep(cycles)
            eh.h.fetch_kv_again(1, dst[0], dst[1])                                    # a gather from those slots, behind the sleep
        errors = []

        def expert_side():
            try:
                eh.revoke(S.EXPERT, sorted(xh.live)[:2])                              # waits for both streams' work
            except BaseException as e:
                errors.append(e)

        th = threading.Thread(target=expert_side)
        th.start()
        time.sleep(0.03)                                                              # the other revocation is waiting by now
        a = time.perf_counter()
        eh.revoke(S.KV, in_cache)                                                     # frees and poisons what the gather reads
        waited = time.perf_counter() - a
        th.join(30)
        assert not th.is_alive() and not errors, errors
        torch.cuda.synchronize()
        from conftest import live
        live(f"  the second revocation waited {1e3 * waited:.1f} ms for a gather queued behind a sleep of 150 ms")
        got = (dst[0].cpu().numpy(), dst[1].cpu().numpy())
        assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1]), "the gather read slots that were already freed"
        assert waited > 0.05
        # lock step again, and nothing else is wrong
        eo.revoke(S.EXPERT, sorted(xo.live)[:2]); eo.revoke(S.KV, in_cache)
        P.assert_kv_equal(ro.fetch(0), rh.fetch(0), "kv afterwards")
        P.assert_dirs_equal(eo, eh, S.KV, wl.n_objects)
        P.assert_dirs_equal(eo, eh, S.EXPERT, ex.n_objects)
    finally:
        eh.close(); eo.close()


def test_a_kv_fetch_does_not_wait_for_the_experts_directory_edits():
    """Directory edits are ordered per class. The expert stream is held up by a sleeping kernel with a placement (copies,
    then the directory write that publishes them) queued behind it; a KV fetch on the other stream completes while that
    kernel still sleeps. Skipped when the device runs the two streams through one hardware queue."""
    import torch
    say("a KV fetch while the experts' directory edits are pending")
    wl = W.kv_decode(seed=31, n_layers=1, n_seq=2, min_len=300, max_len=600, n_steps=1)
    ex = W.expert_offload(seed=31, shape=W.ExpertShape(n_layers=1, n_experts=8, d_model=256, d_ff=512), n_local=0)
    eo, eh = P.make_engines(wl, ex, poison=True, two_streams=True)
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        xo, xh = S.ExpertRun(eo, ex), S.ExpertRun(eh, ex)
        cached = sorted(xh.live)
        for e in (eo, eh):
            e.revoke(S.EXPERT, cached[:2])
        want = ro.fetch(0)
        P.assert_kv_equal(want, rh.fetch(0), "kv before")                 # every stream's scratch exists from here on
        kv_stream, x_stream = eh.streams[S.KV], eh.streams[S.EXPERT]
        table, nb = rh.table_arrays()
        d_table, d_nb = torch.from_numpy(table).to(eh.dev), torch.from_numpy(nb).to(eh.dev)
        d_sdb = torch.from_numpy(rh.seq_dst_block.view(np.int64)).to(eh.dev)
        dst = [torch.zeros(rh.cap * wl.shape.chunk_bytes, dtype=torch.uint8, device=eh.dev) for _ in range(2)]
        torch.cuda.synchronize()
        independent, cycles = P.streams_run_independently(eh.dev, x_stream, kv_stream, ms=150.0)
        if not independent:
            pytest.skip("the two streams share a hardware queue in this process")
        with torch.cuda.stream(x_stream):
            torch.cuda._sleep(cycles)
        st = eh.place(S.EXPERT, cached[:2])                                # queued behind the sleeping kernel
        still = torch.cuda.Event()
        with torch.cuda.stream(x_stream):
            still.record()
        with torch.cuda.stream(kv_stream):                                 # nothing but the library's kernels in the timed part
            eh.h.fetch_kv(0, d_table, d_nb, dst[0], dst[1], d_sdb, rh.cap)
        kv_stream.synchronize()
        pending = not still.query()
        torch.cuda.synchronize()
        assert pending, "the KV fetch waited for the expert class's directory edits"
        assert np.array_equal(eo.place(S.EXPERT, cached[:2]), st)
        assert np.array_equal(dst[0].cpu().numpy(), want[0]) and np.array_equal(dst[1].cpu().numpy(), want[1]), "kv during"
        P.assert_experts_equal(xo.fetch(0, 0), xh.fetch(0, 0), "experts after")
        P.assert_dirs_equal(eo, eh, S.EXPERT, ex.n_objects)
    finally:
        eh.close(); eo.close()


def test_a_kv_fetch_does_not_wait_for_a_placement_on_another_stream():
    """A placement is best effort and a fetch is not: KV blocks are placed on a second stream that is held up by a sleeping
    kernel, and a fetch of the same blocks on the first stream completes meanwhile, served from the host copies - the same
    bytes.  Once the placement is through, the next fetch finds the blocks in the cache tier.  A revocation made while the
    placement is still queued is seen by every later fetch, as always."""
    import torch
    say("a KV fetch while a placement of the same class is queued on another stream")
    wl = W.kv_decode(seed=34, n_layers=1, n_seq=2, min_len=9000, max_len=12000, p_cache=0.3, n_steps=1)
    eo, eh = P.make_engines(wl, poison=True, cache_slack=2000)
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        want = ro.fetch(0)
        P.assert_kv_equal(want, rh.fetch(0), "before")
        on_host = [b for s in range(wl.n_seq) for b in rh.tables[s][:-1] if eh.lookup(S.KV, b)[0] == S.HOST][:302]
        assert len(on_host) == 302
        warm, on_host = on_host[300:], on_host[:300]
        other = torch.cuda.Stream(eh.dev)
        main = torch.cuda.current_stream()
        independent, cycles = P.streams_run_independently(eh.dev, other, main, ms=150.0)
        if not independent:
            pytest.skip("the two streams share a hardware queue in this process")
        table, nb = rh.table_arrays()
        d_table, d_nb = torch.from_numpy(table).to(eh.dev), torch.from_numpy(nb).to(eh.dev)
        d_sdb = torch.from_numpy(rh.seq_dst_block.view(np.int64)).to(eh.dev)
        dst = [torch.zeros(rh.cap * wl.shape.chunk_bytes, dtype=torch.uint8, device=eh.dev) for _ in range(2)]
        with torch.cuda.stream(other):                                    # this stream's scratch exists from here on: a first
            eh.h.fetch_kv(0, d_table, d_nb, dst[0], dst[1], d_sdb, rh.cap)   # fetch or placement waits for the stream and allocates
            assert np.array_equal(eh.h.place(S.KV, warm), eo.place(S.KV, warm))
        want = ro.fetch(0)
        torch.cuda.synchronize()
        for t in dst:
            t.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(other):
            torch.cuda._sleep(cycles)
            st = eh.h.place(S.KV, on_host)                                # queued behind the sleeping kernel
            still = torch.cuda.Event(); still.record()
        eh.h.fetch_kv(0, d_table, d_nb, dst[0], dst[1], d_sdb, rh.cap)
        main.synchronize()
        pending = not still.query()
        counts, miss, n_miss = eh.h.fetch_info(miss_cap=table.size, cls=S.KV)
        assert pending, "the fetch waited for the other stream's placement"
        assert (st == 0).all() and np.array_equal(eo.place(S.KV, on_host), st)
        got = (dst[0].cpu().numpy(), dst[1].cpu().numpy(), np.sort(miss), counts)
        P.assert_kv_equal(want, got, "during the placement", counts=False)
        assert got[3]["n_host"] == want[3]["n_host"], "the fetch was served through entries that were not published yet"
        # a revocation while the placement is still queued: later fetches see it (and, behind it in the chain, the placement)
        a, b = ro.revoke_quarter(0), rh.revoke_quarter(0)
        assert np.array_equal(a[0], b[0])
        P.assert_kv_equal(ro.fetch(0), rh.fetch(0), "after the placement and a revocation")
        P.assert_dirs_equal(eo, eh, S.KV, wl.n_objects)
        P.assert_tiers_equal(eo, eh, S.KV, 2, tiers=(S.CACHE,), what="cache tier")
    finally:
        eh.close(); eo.close()


def test_a_released_stream_starts_afresh():
    """harvest_release_stream frees what the context keeps for a caller stream; the next call on the stream sets it up
    again and fetches the same bytes; a prefetcher's stream is not the caller's to release."""
    import torch
    from paper_2602_00328_amd import binding as B
    say("release of a stream's state")
    wl = W.kv_decode(seed=33, n_layers=2, n_seq=3, min_len=9000, max_len=20000, n_steps=1)
    ex = W.expert_offload(seed=33, shape=W.ExpertShape(n_layers=1, n_experts=8, d_model=256, d_ff=512), n_local=1)
    eo, eh = P.make_engines(wl, ex, two_streams=True)
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        xo, xh = S.ExpertRun(eo, ex), S.ExpertRun(eh, ex)
        want = ro.fetch(1)
        P.assert_kv_equal(want, rh.fetch(1), "before the release")
        P.assert_experts_equal(xo.fetch(0, 0), xh.fetch(0, 0), "experts before")
        kv_stream = eh.streams[S.KV]
        eh.h.release_stream(kv_stream)
        with pytest.raises(B.HarvestError) as e:
            eh.h.fetch_info(stream=kv_stream, cls=S.KV)
        assert e.value.code == B.ENOENT
        with pytest.raises(B.HarvestError) as e:
            eh.h.release_stream(kv_stream)
        assert e.value.code == B.ENOENT
        with pytest.raises(B.HarvestError) as e:                   # no single-layer fetch to repeat any more
            with torch.cuda.stream(kv_stream):
                d = torch.zeros(16, dtype=torch.uint8, device=eh.dev)
                eh.h.fetch_kv_again(0, d, d)
        assert e.value.code == B.EINVAL
        P.assert_kv_equal(want, rh.fetch(1), "after the release")
        # a revocation between two uses of a released and re-made stream state still drains what is in flight
        a, b = ro.revoke_quarter(0), rh.revoke_quarter(0)
        assert np.array_equal(a[0], b[0])
        P.assert_kv_equal(ro.fetch(0), rh.fetch(0), "after a revocation")
        P.assert_experts_equal(xo.fetch(0, 0), xh.fetch(0, 0), "experts after")
        P.assert_dirs_equal(eo, eh, S.KV, wl.n_objects)
    finally:
        eh.close(); eo.close()


# ---- head-major working layout ----------------------------------------------------------------------------------

@LAYOUTS
@pytest.mark.parametrize("heads,dim,tokens,elt", [(8, 128, 16, 2), (8, 128, 16, 1), (3, 24, 4, 2), (1, 8, 1, 2), (5, 104, 48, 2),
                                                  (4, 512, 8, 2), (16, 32, 12, 2), (8, 128, 6, 2)])
def test_head_major_fetch(heads, dim, tokens, elt, adjacent):
    shape = W.KVShape(n_layers=2, block_tokens=tokens, n_kv_heads=heads, head_dim=dim, elt_bytes=elt)
    say(f"head-major: {heads} heads x {dim} x {elt} B, {tokens}-token blocks, chunk {shape.chunk_bytes}")
    wl = W.kv_decode(seed=12, n_seq=3, min_len=30 * tokens, max_len=90 * tokens, n_steps=tokens + 3, shape=shape,
                     fill_mode=W.FILL_NORMAL)
    eo, eh = P.make_engines(wl, hip_kwargs=dict(cache_planes_adjacent=adjacent, general_fetch=True))
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        final = [len(t) + len(f) for t, f in zip(wl.tables, wl.future_blocks)]
        caps = np.array(final, np.uint32)
        for t in range(tokens + 3):
            table, nb = ro.table_arrays()
            layer = t % 2
            a = eo.fetch_kv_head_major(layer, table, nb, ro.seq_dst_block, caps, ro.cap, heads, tokens, dst_fill=0x5A)
            b = eh.fetch_kv_head_major(layer, table, nb, rh.seq_dst_block, caps, rh.cap, heads, tokens, dst_fill=0x5A)
            P.assert_kv_equal(a, b, f"head-major step {t}")
            # and against the token-major fetch of the library itself: a pure transpose per sequence
            if t == 0:
                tm = rh.fetch(layer)
                hb = dim * elt
                for s in range(3):
                    lo, hi = int(ro.seq_dst_block[s]) * shape.chunk_bytes, (int(ro.seq_dst_block[s]) + int(nb[s])) * shape.chunk_bytes
                    x = tm[0][lo:hi].reshape(int(nb[s]) * tokens, heads, hb)
                    full = b[0][int(ro.seq_dst_block[s]) * shape.chunk_bytes:(int(ro.seq_dst_block[s]) + final[s]) * shape.chunk_bytes]
                    y = full.reshape(heads, final[s] * tokens, hb)[:, :int(nb[s]) * tokens]
                    assert np.array_equal(np.transpose(x, (1, 0, 2)), y)
            ro.append(t); rh.append(t)
        # capacities that do not fit, and a table longer than a capacity
        small = caps.copy(); small[1] = 2
        table, nb = ro.table_arrays()
        a = eo.fetch_kv_head_major(0, table, nb, ro.seq_dst_block, small, ro.cap - 1, heads, tokens, dst_fill=0x5A)
        b = eh.fetch_kv_head_major(0, table, nb, rh.seq_dst_block, small, rh.cap - 1, heads, tokens, dst_fill=0x5A)
        P.assert_kv_equal(a, b, "head-major with short capacities")
        assert b[3]["n_invalid"] > 0
    finally:
        eh.close(); eo.close()


# ---- two contexts alive on the device at once --------------------------------------------------------------------

def test_two_contexts_side_by_side():
    say("two contexts")
    wl_a = W.kv_decode(seed=27, n_layers=2, n_seq=2, min_len=300, max_len=700, n_steps=6)
    wl_b = W.kv_decode(seed=28, n_layers=3, n_seq=3, min_len=200, max_len=500, n_steps=6,
                       shape=W.KVShape(n_layers=3, n_kv_heads=4, head_dim=64))
    eo_a, eh_a = P.make_engines(wl_a, poison=True)
    eo_b, eh_b = P.make_engines(wl_b, poison=True)
    try:
        ra_o, ra_h, rb_o, rb_h = S.KVRun(eo_a, wl_a), S.KVRun(eh_a, wl_a), S.KVRun(eo_b, wl_b), S.KVRun(eh_b, wl_b)
        for t in range(6):
            ha, hb = ra_h.fetch_begin(t % 2), rb_h.fetch_begin(t % 3)            # both contexts have work in flight
            if t == 3:
                x, y = ra_o.revoke_quarter(t), ra_h.revoke_quarter(t)            # a revocation in one of them
                assert np.array_equal(x[0], y[0])
            P.assert_kv_equal(ra_o.fetch(t % 2), eh_a.fetch_end(ha), f"context a step {t}", counts=t != 3)
            P.assert_kv_equal(rb_o.fetch(t % 3), eh_b.fetch_end(hb), f"context b step {t}")
            ra_o.append(t); ra_h.append(t); rb_o.append(t); rb_h.append(t)
        P.assert_dirs_equal(eo_a, eh_a, S.KV, wl_a.n_objects)
        P.assert_dirs_equal(eo_b, eh_b, S.KV, wl_b.n_objects)
    finally:
        eh_a.close(); eo_a.close(); eh_b.close(); eo_b.close()


# ---- the paper's own three calls ---------------------------------------------------------------------------------

def test_alloc_and_free_by_their_paper_names():
    say("harvest_alloc / harvest_free / harvest_register_cb")
    wl = W.kv_decode(seed=26, n_layers=2, n_seq=2, min_len=200, max_len=400, p_cache=0.0, n_steps=1, fill_mode=W.FILL_TAG)
    eo, eh = P.make_engines(wl, poison=True, cache_slack=5)
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        blocks = rh.tables[0][:7]
        st = [eh.h.alloc(S.KV, b) for b in blocks]                 # five cache slots: the last two stay on the host
        assert st == [0, 0, 0, 0, 0, -2, -2] and list(eo.place(S.KV, blocks)) == st
        P.assert_kv_equal(ro.fetch(1), rh.fetch(1), "after harvest_alloc")
        eh.h.register_cb(S.KV, blocks[1], enabled=False)
        eh.h.free(S.KV, blocks[0]); eo.revoke(S.KV, [blocks[0]])
        eh.revoke(S.KV, [blocks[1], blocks[2]]); eo.revoke(S.KV, [blocks[1], blocks[2]])
        assert [i for _c, i in eh.h.revoked_log] == [int(blocks[2])]      # freed: no callback; cleared: no callback
        a, b = ro.fetch(0), rh.fetch(0)
        P.assert_kv_equal(a, b, "after harvest_free")
        assert b[3]["n_cache"] == 2
        P.assert_dirs_equal(eo, eh, S.KV, wl.n_objects)
        P.assert_tiers_equal(eo, eh, S.KV, 2, what="alloc / free")
    finally:
        eh.close(); eo.close()


# ---- a one-plane KV class (a latent cache, say): every kernel's one-plane instantiation -------------------------

def test_one_plane_kv_class():
    say("one-plane KV class")
    shape = W.KVShape(n_layers=3, block_tokens=16, n_kv_heads=4, head_dim=72, elt_bytes=2)       # 9 216-byte chunks
    wl = W.kv_decode(seed=25, n_seq=3, min_len=300, max_len=900, n_steps=20, shape=shape)
    kv = S.kv_spec(wl, n_planes=1)
    eo, eh = P.make_engines(kv_spec=kv, poison=True)
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        caps = np.array([len(t) + len(f) for t, f in zip(wl.tables, wl.future_blocks)], np.uint32)
        for t in range(20):
            layer = t % 3
            a, b = ro.fetch(layer), rh.fetch(layer)
            assert b[1] is None
            P.assert_kv_equal(a, b, f"one plane step {t}")
            table, nb = rh.table_arrays()
            a = eo.fetch_kv_head_major(layer, table, nb, ro.seq_dst_block, caps, ro.cap, 4, 16)
            b = eh.fetch_kv_head_major(layer, table, nb, rh.seq_dst_block, caps, rh.cap, 4, 16)
            P.assert_kv_equal(a, b, f"one plane head-major step {t}")
            if t % 5 == 0:
                layers, miss, counts = eh.fetch_kv_layers(0, 3, table, nb, rh.seq_dst_block, rh.cap)
                for r, (k, v) in enumerate(layers):
                    P.assert_kv_equal(eo.fetch_kv(r, table, nb, ro.seq_dst_block, ro.cap), (k, v, miss, counts), f"layers {t}.{r}")
            if t == 8:
                x, y = ro.revoke_quarter(t), rh.revoke_quarter(t)
                assert np.array_equal(x[0], y[0])
            if t == 14:
                assert np.array_equal(ro.replace_revoked(), rh.replace_revoked())
            ro.append(t); rh.append(t)
        P.assert_dirs_equal(eo, eh, S.KV, wl.n_objects)
        P.assert_tiers_equal(eo, eh, S.KV, 1, what="one plane")
    finally:
        eh.close(); eo.close()


# ---- the same fetch again for another layer ------------------------------------------------------------------------

@LAYOUTS
@pytest.mark.parametrize("general", [False, True], ids=["one-kernel", "general"])
@pytest.mark.parametrize("head_major", [False, True])
def test_fetch_again_for_another_layer(general, head_major, adjacent):
    """harvest_fetch_kv_again walks the layers of a step on the lists of the first fetch; every directory edit in between
    (placement, revocation, demotion, registration) makes it resolve again.  Either way it must deliver what a fetch of
    that layer delivers."""
    say(f"fetch again, general path {general}, head-major {head_major}")
    wl = W.kv_decode(seed=41, n_layers=4, n_seq=3, min_len=600, max_len=1500, p_cache=0.6, n_steps=48)
    eo, eh = P.make_engines(wl, poison=True, cache_slack=32,
                            hip_kwargs=dict(general_fetch=general, cache_planes_adjacent=adjacent))
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        heads, tokens = wl.shape.n_kv_heads, wl.shape.block_tokens
        final = [len(t) + len(f) for t, f in zip(wl.tables, wl.future_blocks)]

        def first(e, r, layer):
            table, nb = r.table_arrays()
            if head_major:
                return e.fetch_kv_head_major(layer, table, nb, r.seq_dst_block, np.array(final, np.uint32), r.cap, heads,
                                             tokens, dst_fill=0x5A)
            return e.fetch_kv(layer, table, nb, r.seq_dst_block, r.cap)

        fill = 0x5A if head_major else 0
        for t in range(12):
            P.assert_kv_equal(first(eo, ro, t % 4), first(eh, rh, t % 4), f"step {t}, first layer")
            for layer in ((t + 1) % 4, (t + 3) % 4, t % 4):
                if t % 3 == 1 and layer == (t + 3) % 4:                      # an edit between two layers of the step
                    if t % 2:
                        ids_o, ids_h = ro.revoke_quarter(t)[0], rh.revoke_quarter(t)[0]
                        assert np.array_equal(ids_o, ids_h)
                    else:
                        assert np.array_equal(ro.replace_revoked(), rh.replace_revoked())
                P.assert_kv_equal(eo.fetch_kv_again(layer, fill), eh.fetch_kv_again(layer, fill), f"step {t}, again at layer {layer}")
            for k in range(4):                                               # appends, roll-overs: registrations and demotions
                ro.append(4 * t + k); rh.append(4 * t + k)
        P.assert_dirs_equal(eo, eh, S.KV, wl.n_objects)
        st = eh.h.stats()
        f = st.fetch[0]                              # repeated fetches are counted in the running totals too
        assert f.n_requests == f.n_local + f.n_cache + f.n_host + f.n_lost + f.n_invalid
        assert f.n_requests >= 12 * 4 * sum(len(x) for x in wl.tables)
        with pytest.raises(Exception):
            eh.h.fetch_kv_again(99, None, None)
    finally:
        eh.close(); eo.close()


@pytest.mark.parametrize("general", [False, True], ids=["one-kernel", "general"])
@pytest.mark.parametrize("many_experts", [False, True], ids=["few-experts", "more-experts-than-table-cells"])
def test_fetch_again_after_an_expert_fetch_on_the_same_stream(general, many_experts):
    """A decode step walks its layers with KV and expert fetches in turn, all on one stream: KV fetch, expert fetch, the
    KV fetch again for the next layer.  Each class keeps request lists of its own on the stream, so the repeated KV
    fetch must deliver that layer's blocks whatever the expert fetch in between wrote - also when the expert class has
    more experts per layer than the block table has cells, which makes the expert fetch the one that sizes its lists."""
    say(f"fetch again after an expert fetch, general path {general}, many experts {many_experts}")
    wl = W.kv_decode(seed=43, n_layers=3, n_seq=2, min_len=300, max_len=700, p_cache=0.6, n_steps=8)
    n_exp = 2500 if many_experts else 12
    ex = W.expert_offload(seed=43, shape=W.ExpertShape(n_layers=3, n_experts=n_exp, d_model=16, d_ff=24), n_tokens=40,
                          n_local=2, fill_mode=W.FILL_TAG)
    eo, eh = P.make_engines(wl, ex, poison=True, hip_kwargs=dict(general_fetch=general))      # one stream for both classes
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        xo, xh = S.ExpertRun(eo, ex), S.ExpertRun(eh, ex)
        assert eh.streams[S.KV] is None and eh.streams[S.EXPERT] is None
        assert max(len(t) + len(f) for t, f in zip(wl.tables, wl.future_blocks)) * wl.n_seq < 2500
        for t in range(6):
            P.assert_kv_equal(ro.fetch(0), rh.fetch(0), f"step {t}, layer 0")
            for layer in (0, 1, 2):
                want_x = xo.fetch(t, layer)
                P.assert_experts_equal(want_x, xh.fetch(t, layer), f"step {t}, experts of layer {layer}")
                nxt = (layer + 1) % 3
                want_kv = eo.fetch_kv_again(nxt)
                P.assert_kv_equal(want_kv, eh.fetch_kv_again(nxt), f"step {t}, again at layer {nxt}")
                # each class keeps its own counters on the stream; harvest_fetch_info reports the latest fetch of either
                assert eh.h.fetch_info(cls=S.EXPERT)[0] == want_x[4] and eh.h.fetch_info(cls=S.KV)[0] == want_kv[3]
                assert eh.h.fetch_info()[0] == want_kv[3]
            ro.append(t); rh.append(t)
    finally:
        eh.close(); eo.close()


# ---- several layers in one call --------------------------------------------------------------------------------

@pytest.mark.parametrize("general", [False, True], ids=["one-kernel", "general"])
@pytest.mark.parametrize("shared,adjacent", [(False, False), (True, False), (False, True)],
                         ids=["k-pool-and-v-pool", "shared-pool", "k-v-adjacent"])
def test_fetch_of_several_layers_in_one_call(shared, adjacent, general):
    say(f"multi-layer fetch, shared pool {shared}, general path {general}")
    wl = W.kv_decode(seed=24, n_layers=5, n_seq=3, min_len=300, max_len=900, n_steps=20)
    kw = {}
    if shared:
        obj = 5 * 2 * wl.shape.chunk_bytes
        kw = dict(shared_cache_bytes=(int(wl.resident.sum()) - 3) * obj, shared_granule=4096)
    eo, eh = P.make_engines(wl, poison=True, hip_kwargs=dict(general_fetch=general, cache_planes_adjacent=adjacent), **kw)
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        for t in range(20):
            first, n = [(0, 5), (1, 3), (4, 1), (2, 2)][t % 4]
            table, nb = rh.table_arrays()
            layers, miss, counts = eh.fetch_kv_layers(first, n, table, nb, rh.seq_dst_block, rh.cap)
            assert len(layers) == n
            for r, (k, v) in enumerate(layers):
                want = eo.fetch_kv(first + r, table, nb, ro.seq_dst_block, ro.cap)
                P.assert_kv_equal(want, (k, v, miss, counts), f"step {t} layer {first + r}")
            if t == 7:
                a, b = ro.revoke_quarter(t), rh.revoke_quarter(t)
                assert np.array_equal(a[0], b[0])
            if t == 12:
                assert np.array_equal(ro.replace_revoked(), rh.replace_revoked())
            ro.append(t); rh.append(t)
        with pytest.raises(Exception):                         # layers beyond the pool
            eh.fetch_kv_layers(3, 3, table, nb, rh.seq_dst_block, rh.cap)
        P.assert_dirs_equal(eo, eh, S.KV, wl.n_objects)
    finally:
        eh.close(); eo.close()


# ---- one cache pool shared by both classes: variable-size segments, best-fit (Section 3.3) ----------------------

def shared_pool_bytes(wl, ex, frac, G):
    kv_bytes = wl.shape.n_layers * 2 * wl.shape.chunk_bytes
    demand = int(wl.resident.sum()) * kv_bytes + int((ex.tier0 == 1).sum()) * ex.shape.chunk_bytes
    return (int(frac * demand) // G) * G


@pytest.mark.parametrize("frac,granule", [(0.7, 1024), (1.5, 4096), (0.4, 256)])
def test_both_classes_share_one_cache_pool(frac, granule):
    say(f"shared cache pool: {frac} of the demand, granule {granule}")
    wl = W.kv_decode(seed=21, n_layers=2, n_seq=3, min_len=400, max_len=1200, n_steps=60)
    sh = W.ExpertShape(n_layers=2, n_experts=16, d_model=96, d_ff=100)
    ex = W.expert_offload(seed=21, shape=sh, n_tokens=64)
    eo, eh = P.make_engines(wl, ex, poison=True, two_streams=True,
                            shared_cache_bytes=shared_pool_bytes(wl, ex, frac, granule), shared_granule=granule)
    try:
        xo, xh = S.ExpertRun(eo, ex), S.ExpertRun(eh, ex)          # experts first, or the blocks take the whole pool
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        assert np.array_equal(ro.place_status, rh.place_status) and np.array_equal(xo.place_status, xh.place_status)
        enospc = int((ro.place_status != 0).sum() + (xo.place_status != 0).sum())
        assert (enospc > 0) == (frac < 1)
        P.assert_shared_pools_equal(eo, eh, "after the first placements")
        n_refused, most_runs = 0, 0
        for t in range(60):
            layer = t % 2
            P.assert_kv_equal(ro.fetch(layer), rh.fetch(layer), f"shared kv step {t}")
            P.assert_experts_equal(xo.fetch(t, layer), xh.fetch(t, layer), f"shared experts step {t}")
            if t % 10 == 0 and t:
                a, b = ro.revoke_quarter(t), rh.revoke_quarter(t)
                assert np.array_equal(a[0], b[0]) and a[1] == b[1]
                a, b = xo.revoke_quarter(t), xh.revoke_quarter(t)
                assert np.array_equal(a[0], b[0]) and a[1] == b[1]
                P.assert_shared_pools_equal(eo, eh, f"after the revocations of step {t}")
                # other objects move into the holes (experts into the holes blocks left, and so on): the pool fragments
                other_kv = [b for b in range(wl.n_closed)
                            if eo.lookup(S.KV, b)[0] == S.HOST and b not in ro.pending_replace][:6]
                other_ex = [e for e in range(ex.n_objects)
                            if eo.lookup(S.EXPERT, e)[0] == S.HOST and e not in xo.pending_replace][:3]
                for cls, ids, runs in ((S.EXPERT, other_ex, (xo, xh)), (S.KV, other_kv, (ro, rh))):
                    if ids:
                        st_o, st_h = eo.place(cls, ids), eh.place(cls, ids)
                        assert np.array_equal(st_o, st_h)
                        for r in runs:
                            r.live |= {int(i) for i, st in zip(ids, st_o) if st == 0}
                most_runs = max(most_runs, len(eo.shared_free_runs()))
                P.assert_shared_pools_equal(eo, eh, f"after filling the holes of step {t}")
            if t % 10 == 5:
                st_x, st_k = xo.replace_revoked(), ro.replace_revoked()
                assert np.array_equal(st_x, xh.replace_revoked()) and np.array_equal(st_k, rh.replace_revoked())
                n_refused += int((st_x != 0).sum() + (st_k != 0).sum())
            ro.append(t); rh.append(t)
        assert most_runs > 4 and (n_refused > 0) == (frac < 1)
        P.assert_dirs_equal(eo, eh, S.KV, wl.n_objects)
        P.assert_dirs_equal(eo, eh, S.EXPERT, ex.n_objects)
        P.assert_tiers_equal(eo, eh, S.KV, 2, what="shared kv")
        P.assert_tiers_equal(eo, eh, S.EXPERT, 1, what="shared experts")
        P.assert_shared_pools_equal(eo, eh, "at the end")
        st = eh.h.stats()
        assert st.cache_slots_in_use[S.KV] == len(rh.live) and st.cache_slots_in_use[S.EXPERT] == len(xh.live)
    finally:
        eh.close(); eo.close()


def test_head_major_fetch_from_the_shared_pool():
    say("head-major from shared segments")
    shape = W.KVShape(n_layers=3, block_tokens=16, n_kv_heads=4, head_dim=64, elt_bytes=1)
    wl = W.kv_decode(seed=22, n_seq=3, min_len=300, max_len=900, n_steps=4, shape=shape)
    n_res = int(wl.resident.sum())
    G = 512
    pool = -(-(3 * 2 * shape.chunk_bytes) // G) * G * (n_res - 5)          # five blocks too few
    eo, eh = P.make_engines(wl, shared_cache_bytes=pool, shared_granule=G)
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        assert np.array_equal(ro.place_status, rh.place_status) and (rh.place_status != 0).sum() > 0
        final = [len(t) + len(f) for t, f in zip(wl.tables, wl.future_blocks)]
        caps = np.array(final, np.uint32)
        for t in range(4):
            table, nb = ro.table_arrays()
            layer = t % 3
            a = eo.fetch_kv_head_major(layer, table, nb, ro.seq_dst_block, caps, ro.cap, 4, 16, dst_fill=0x5A)
            b = eh.fetch_kv_head_major(layer, table, nb, rh.seq_dst_block, caps, rh.cap, 4, 16, dst_fill=0x5A)
            P.assert_kv_equal(a, b, f"head-major shared step {t}")
            P.assert_kv_equal(ro.fetch(layer), rh.fetch(layer), f"token-major shared step {t}")
            ro.append(t); rh.append(t)
        P.assert_shared_pools_equal(eo, eh)
    finally:
        eh.close(); eo.close()


def test_lossy_objects_demote_into_shared_segments():
    from types import SimpleNamespace
    say("lossy objects into shared segments")
    chunk, G = 4096 + 48, 256
    spec = SimpleNamespace(n_layers=2, n_planes=2, chunk_bytes=chunk, max_objects=8, n_host_slots=4, n_cache_slots=0,
                           n_local_slots=4, n_experts=0)
    obj_g = -(-(2 * 2 * chunk) // G)
    eo, eh = P.make_engines(kv_spec=spec, poison=True, shared_cache_bytes=(2 * obj_g + 3) * G, shared_granule=G)
    try:
        for e in (eo, eh):
            ids = e.register(S.KV, 3, None, S.LOCAL)
            assert list(ids) == [0, 1, 2]
            for obj in range(3):
                for p in range(2):
                    for l in range(2):
                        e.write_local(S.KV, obj, p, l, 0, W.rng(23, obj, p, l).integers(0, 256, size=chunk, dtype=np.uint8))
        for e in (eo, eh):
            with pytest.raises(Exception):                   # three segments do not fit: nothing may change
                e.evict_from_local(S.KV, [0, 1, 2], S.EVICT_DEMOTE)
            assert e.lookup(S.KV, 0)[:2] == (S.LOCAL, 0)
        P.assert_shared_pools_equal(eo, eh, "after the refused demotion")
        for e in (eo, eh):
            e.evict_from_local(S.KV, [2, 0], S.EVICT_DEMOTE)
            assert e.lookup(S.KV, 2)[:2] == (S.CACHE, 0) and e.lookup(S.KV, 0)[:2] == (S.CACHE, obj_g)
        table = np.array([[0, 1, 2]], np.int32)
        nb, sdb = np.array([3], np.int32), np.array([0], np.uint64)
        for layer in range(2):
            P.assert_kv_equal(eo.fetch_kv(layer, table, nb, sdb, 3), eh.fetch_kv(layer, table, nb, sdb, 3), "lossy shared")
        for e in (eo, eh):
            e.revoke(S.KV, [2])
        P.assert_shared_pools_equal(eo, eh, "after revoking a lossy object")
        a = eo.c[S.KV].fetch_kv(0, table, nb, sdb, 3, dst_k=np.full(3 * chunk, 0xEE, np.uint8),
                                dst_v=np.full(3 * chunk, 0xEE, np.uint8))
        b = eh.fetch_kv(0, table, nb, sdb, 3, dst_fill=0xEE)
        P.assert_kv_equal((a[0], a[1], np.sort(a[2]), a[3]), b, "lossy shared after revocation")
        assert b[3]["n_lost"] == 1 and (b[0][2 * chunk:] == 0xEE).all()
    finally:
        eh.close(); eo.close()


# ---- lossy objects ------------------------------------------------------------------------------------------------

@LAYOUTS
def test_lossy_objects_move_to_the_cache_tier_and_are_lost_on_revocation(adjacent):
    from types import SimpleNamespace
    say("lossy objects")
    chunk = 4096 + 48
    spec = SimpleNamespace(n_layers=2, n_planes=2, chunk_bytes=chunk, max_objects=8, n_host_slots=4, n_cache_slots=3,
                           n_local_slots=3, n_experts=0)
    eo, eh = P.make_engines(kv_spec=spec, poison=True, hip_kwargs=dict(cache_planes_adjacent=adjacent))
    try:
        for e in (eo, eh):
            lossy = e.register(S.KV, 3, None, S.LOCAL)
            backed = e.register(S.KV, 2, [3, 1], S.HOST)
            so = np.full(4, W.NO_OBJECT, np.uint32); so[3] = backed[0]; so[1] = backed[1]
            e.fill_host(S.KV, so, 9, W.CLS_KV, W.FILL_TAG, 1.0)
            e.adopt(S.KV, backed)
            for obj in lossy:
                for p in range(2):
                    for l in range(2):
                        e.write_local(S.KV, obj, p, l, 0, W.chunk(9, W.CLS_APPEND, p, l, int(obj), chunk, W.FILL_TAG))
            assert list(e.place(S.KV, [backed[0]])) == [0]
            e.evict_from_local(S.KV, lossy[:2], S.EVICT_DEMOTE)            # two lossy blocks take the last two cache slots
        P.assert_dirs_equal(eo, eh, S.KV, 5)
        assert eh.lookup(S.KV, 0)[0] == S.CACHE and eh.lookup(S.KV, 2)[0] == S.LOCAL
        table = np.array([[0, 3, 1, 2, 4]], np.int32)
        nb, sdb = np.array([5], np.int32), np.array([0], np.uint64)
        for layer in range(2):
            P.assert_kv_equal(eo.fetch_kv(layer, table, nb, sdb, 5), eh.fetch_kv(layer, table, nb, sdb, 5), f"lossy {layer}")
        assert eo.revoke(S.KV, [0, 3]) == eh.revoke(S.KV, [0, 3]) == [0, 3]
        P.assert_dirs_equal(eo, eh, S.KV, 5)
        assert eh.lookup(S.KV, 0)[0] == S.NONE and eh.lookup(S.KV, 3)[0] == S.HOST
        c = eo.c[S.KV]
        a = c.fetch_kv(1, table, nb, sdb, 5, dst_k=np.full(5 * chunk, 0xEE, np.uint8), dst_v=np.full(5 * chunk, 0xEE, np.uint8))
        b = eh.fetch_kv(1, table, nb, sdb, 5, dst_fill=0xEE)
        P.assert_kv_equal((a[0], a[1], np.sort(a[2]), a[3]), b, "after revocation")
        assert b[3]["n_lost"] == 1 and (b[0][:chunk] == 0xEE).all() and list(b[2]) == [0, 1, 4]
        P.assert_tiers_equal(eo, eh, S.KV, 2, what="lossy")
        # reconstruction: the lost block returns to local HBM, is rebuilt there and served again
        for e in (eo, eh):
            e.restore(S.KV, [0])
            for p in range(2):
                for l in range(2):
                    e.write_local(S.KV, 0, p, l, 0, W.chunk(10, W.CLS_APPEND, p, l, 0, chunk, W.FILL_TAG))
        P.assert_dirs_equal(eo, eh, S.KV, 5)
        assert eh.lookup(S.KV, 0)[0] == S.LOCAL
        for layer in range(2):
            a, b = eo.fetch_kv(layer, table, nb, sdb, 5), eh.fetch_kv(layer, table, nb, sdb, 5)
            P.assert_kv_equal(a, b, f"rebuilt {layer}")
            assert b[3]["n_lost"] == 0 and W.check_tag(b[0][:chunk], 10, W.CLS_APPEND, 0, layer, 0)
        P.assert_tiers_equal(eo, eh, S.KV, 2, what="rebuilt")
    finally:
        eh.close(); eo.close()


def test_plain_copy_and_profile_counters():
    import torch
    from paper_2602_00328_amd import binding as B
    say("plain copy")
    for n in (16, 4096, 32768 + 16, 5 * 32768, (1 << 20) + 48):
        src = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda")
        dst = torch.zeros(n + 64, dtype=torch.uint8, device="cuda")
        B.plain_copy(dst, src, n)
        torch.cuda.synchronize()
        assert torch.equal(dst[:n], src) and int(dst[n:].sum()) == 0
    with pytest.raises(B.HarvestError):
        B.plain_copy(dst, src, 24)
    # the two halves of the copy on their own: the write fills exactly its range, the read touches nothing
    for n in (16, 1024 + 16, 5 * 32768, (1 << 20) + 48):
        dst = torch.zeros(n + 64, dtype=torch.uint8, device="cuda")
        B.plain_write(dst, n, 0x04030201)
        sink = torch.zeros(1, dtype=torch.int32, device="cuda")
        B.plain_read(dst, n, sink)
        torch.cuda.synchronize()
        want = torch.tensor([1, 2, 3, 4], dtype=torch.uint8, device="cuda").repeat(n // 4)
        assert torch.equal(dst[:n], want) and int(dst[n:].sum()) == 0 and int(sink[0]) == 0
    with pytest.raises(B.HarvestError):
        B.plain_write(dst, 24)


def test_smoke_entry():
    say("smoke")
    P.smoke()


# ---- the ABI from plain C, no Python in the process ---------------------------------------------------------------

def test_plain_c_example_runs():
    import os
    import subprocess
    say("plain-C example")
    exe = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2602_00328_amd", "examples", "kv_fetch")
    if not os.path.exists(exe):                          # a fresh checkout: built here, otherwise used as built
        from paper_2602_00328_amd import _build
        _build.build_example()
    r = subprocess.run([exe], capture_output=True, text=True, timeout=100)
    assert r.returncode == 0 and "kv_fetch example: ok" in r.stdout, r.stdout[-2000:] + r.stderr[-2000:]
