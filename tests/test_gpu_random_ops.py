"""Random sequences of every call - register (backed, local, lossy), place, place from device memory, revoke, evict (one
layer, all layers, with demotion), restore, and fetches in all four forms - run on the HIP library and on the oracle in
lock step: every status, every error code, every fetched byte, count and miss list, and in the end every directory entry
and every tier must agree.  The fixed scenarios elsewhere follow the paper's workloads; this one goes where they do not."""
from types import SimpleNamespace

import numpy as np
import pytest

import workloads as W
import parity as P
from oracle import OracleError
from oracle.engine import OracleEngine
from paper_2602_00328_amd.binding import HarvestError
from workloads.hip_engine import HipEngine

pytestmark = pytest.mark.gpu

KV, HOST, CACHE, LOCAL, NONE = 0, 0, 1, 2, 3
DEMOTE = 1


def both(fo, fh):
    eo = eh = None
    ro = rh = None
    try:
        ro = fo()
    except OracleError as e:
        eo = e.code
    try:
        rh = fh()
    except HarvestError as e:
        eh = e.code
    assert eo == eh, f"error codes differ: oracle {eo}, library {eh}"
    return ro, rh, eo


@pytest.mark.parametrize("seed,general,shared", [(s, bool(s % 2), bool((s // 2) % 2)) for s in range(12)])
def test_random_operations_in_lock_step(seed, general, shared):
    print(f"random operations, seed {seed}, general path {general}, shared pool {shared}", flush=True)
    g = W.rng(seed, 900)
    L, heads, tokens, hb = 3, 2, 4, 32
    chunk = heads * tokens * hb                                        # 256 bytes: [token][head][head_bytes]
    n_max, n_host, n_local = 96, 80, 6
    sp = SimpleNamespace(n_layers=L, n_planes=2, chunk_bytes=chunk, max_objects=n_max, n_host_slots=n_host,
                         n_cache_slots=0 if shared else 20, n_local_slots=n_local, n_experts=0)
    kw = dict(shared_cache_bytes=24 * 2048, shared_granule=256) if shared else {}      # an object: 1536 B = 6 granules
    eo = OracleEngine(kv=sp, poison=True, **kw)
    # (seeds 0, 1, 4 and 5 keep K and V of a block side by side in the cache tier; 8 and 9 keep a pool per plane)
    eh = HipEngine(kv=sp, poison=True, general_fetch=general, cache_planes_adjacent=seed in (0, 1, 4, 5), **kw)
    free_host = list(g.permutation(n_host))
    stride = 9

    def src_planes():
        return [g.integers(0, 256, size=L * stride * chunk, dtype=np.uint8) for _ in range(2)]

    def n_objects():
        n = 0
        while n < n_max:
            try:
                eo.lookup(KV, n)
            except OracleError:
                break
            n += 1
        return n

    try:
        n_fetch = 0
        for step in range(220):
            n = n_objects()
            op = int(g.integers(0, 10))
            if (op == 0 or n < 12) and n < n_max - 3:
                k = int(g.integers(1, 4))
                kind = g.random()
                if kind < 0.6 and len(free_host) >= k:                                   # backed, on the host
                    hs = [int(free_host.pop()) for _ in range(k)]
                    ro, rh, err = both(lambda: eo.register(KV, k, hs, HOST), lambda: eh.register(KV, k, hs, HOST))
                elif kind < 0.85 and len(free_host) >= k:                                # backed, in local HBM
                    hs = [int(free_host.pop()) for _ in range(k)]
                    ro, rh, err = both(lambda: eo.register(KV, k, hs, LOCAL), lambda: eh.register(KV, k, hs, LOCAL))
                    if err is not None:
                        free_host.extend(hs)
                else:                                                                    # lossy, in local HBM
                    ro, rh, err = both(lambda: eo.register(KV, k, None, LOCAL), lambda: eh.register(KV, k, None, LOCAL))
                if err is None:
                    assert np.array_equal(ro, rh)
                    s0, s1 = src_planes()                                                # give the new objects a value
                    blk = g.permutation(stride)[:k]
                    both(lambda: eo.evict(KV, -1, ro, s0, s1, blk, stride), lambda: eh.evict(KV, -1, rh, s0, s1, blk, stride))
                continue
            if n == 0:
                continue
            ids = g.integers(0, n + (1 if g.random() < 0.04 else 0), size=int(g.integers(1, 6))).astype(np.uint32)
            if op == 1:
                ro, rh, err = both(lambda: eo.place(KV, ids), lambda: eh.place(KV, ids))
                assert err is not None or np.array_equal(ro, rh)
            elif op == 2:
                s0, s1 = src_planes()
                blk = g.integers(0, stride + (1 if g.random() < 0.05 else 0), size=ids.size)
                ro, rh, err = both(lambda: eo.place_from(KV, ids, s0, s1, blk, stride),
                                   lambda: eh.place_from(KV, ids, s0, s1, blk, stride))
                assert err is not None or np.array_equal(ro, rh)
            elif op == 3:
                ro, rh, err = both(lambda: eo.revoke(KV, ids), lambda: eh.revoke(KV, ids))
                assert err is not None or [int(i) for i in ro] == [int(i) for i in rh]
            elif op == 4:
                layer = int(g.integers(-1, L))
                flags = DEMOTE if (layer < 0 and g.random() < 0.5) else 0
                s0, s1 = src_planes()
                blk = g.integers(0, stride, size=ids.size)
                uniq = np.unique(ids) if g.random() < 0.8 else ids                       # duplicates are an error: sometimes
                blk = blk[:uniq.size]
                if layer >= 0:
                    s0, s1 = s0[:stride * chunk], s1[:stride * chunk]
                both(lambda: eo.evict(KV, layer, uniq, s0, s1, blk, stride, flags),
                     lambda: eh.evict(KV, layer, uniq, s0, s1, blk, stride, flags))
            elif op == 5:
                lost = [i for i in range(n) if eo.lookup(KV, i)[0] == NONE][:2]
                pick = lost if lost and g.random() < 0.8 else [int(ids[0])]
                both(lambda: eo.restore(KV, pick), lambda: eh.restore(KV, pick))
                for i in pick:                                                           # rebuilt bytes for what came back
                    if i in lost and eo.lookup(KV, i)[0] == LOCAL:
                        s0, s1 = src_planes()
                        both(lambda: eo.evict(KV, -1, [i], s0, s1, [0], stride), lambda: eh.evict(KV, -1, [i], s0, s1, [0], stride))
            else:                                                                        # a fetch, in one of its forms
                n_fetch += 1
                n_seq, max_blocks = int(g.integers(1, 5)), int(g.integers(1, 30))
                table = g.integers(0, n, size=(n_seq, max_blocks)).astype(np.int32)
                table[g.random(table.shape) < 0.03] = int(g.integers(-3, n_max + 5))
                nb = g.integers(0, max_blocks + 1, size=n_seq).astype(np.int32)
                sdb = np.concatenate([[0], np.cumsum(nb)[:-1]]).astype(np.uint64)
                cap = max(1, int(nb.sum()) - (1 if g.random() < 0.2 else 0))
                form = int(g.integers(0, 3))
                what = f"step {step}, fetch form {form}"
                if form == 0:
                    layer = int(g.integers(0, L))
                    P.assert_kv_equal(eo.fetch_kv(layer, table, nb, sdb, cap), eh.fetch_kv(layer, table, nb, sdb, cap), what)
                elif form == 1:
                    layer = int(g.integers(0, L))
                    caps = nb.astype(np.uint32)
                    a = eo.fetch_kv_head_major(layer, table, nb, sdb, caps, cap, heads, tokens, dst_fill=0x5A)
                    b = eh.fetch_kv_head_major(layer, table, nb, sdb, caps, cap, heads, tokens, dst_fill=0x5A)
                    P.assert_kv_equal(a, b, what)
                else:
                    first = int(g.integers(0, L))
                    n_l = int(g.integers(1, L - first + 1))
                    a, b = [eo.fetch_kv(first + r, table, nb, sdb, cap) for r in range(n_l)], \
                        eh.fetch_kv_layers(first, n_l, table, nb, sdb, cap)
                    for r in range(n_l):
                        assert np.array_equal(a[r][0], b[0][r][0]) and np.array_equal(a[r][1], b[0][r][1]), what
                    assert np.array_equal(a[0][2], b[1]) and a[0][3] == b[2], what
            for i in range(n_objects()):
                assert eo.lookup(KV, i) == eh.lookup(KV, i), (step, i)
        assert n_fetch > 40
        P.assert_tiers_equal(eo, eh, KV, 2, what="after the random sequence")
        if shared:
            P.assert_shared_pools_equal(eo, eh, "after the random sequence")
    finally:
        eh.close(); eo.close()


EXPERT = 1


@pytest.mark.parametrize("seed", range(6))
def test_random_expert_operations_in_lock_step(seed):
    """The expert class: routing batches of every size (also beyond the batch size at which the routed set is marked by
    many workgroups), staging buffers that overflow, placements from the host and from the staging buffer the fetch
    has just filled, revocations, write-backs of new expert bytes."""
    print(f"random expert operations, seed {seed}", flush=True)
    g = W.rng(seed, 901)
    n_layers, E, chunk = 3, 12, 208
    n = n_layers * E
    sp = SimpleNamespace(n_layers=1, n_planes=1, chunk_bytes=chunk, max_objects=n, n_host_slots=n, n_cache_slots=14,
                         n_local_slots=6, n_experts=E)
    eo = OracleEngine(expert=sp, poison=True)
    eh = HipEngine(expert=sp, poison=True)
    try:
        local = set(int(i) for i in g.permutation(n)[:5])
        hs = g.permutation(n)
        for i in range(n):                                             # ids follow (layer, expert): one call per object
            tier = LOCAL if i in local else HOST
            ro, rh, err = both(lambda: eo.register(EXPERT, 1, [int(hs[i])], tier), lambda: eh.register(EXPERT, 1, [int(hs[i])], tier))
            assert err is None and int(ro[0]) == int(rh[0]) == i
        val = g.integers(0, 256, size=n * chunk, dtype=np.uint8)
        both(lambda: eo.evict(EXPERT, 0, np.arange(n), val, None, np.arange(n), n),
             lambda: eh.evict(EXPERT, 0, np.arange(n), val, None, np.arange(n), n))
        last = None                                                    # (layer, kind, where, n_staging) of the last fetch
        n_from = 0
        for step in range(120):
            op = int(g.integers(0, 8))
            ids = g.integers(0, n + (1 if g.random() < 0.04 else 0), size=int(g.integers(1, 6))).astype(np.uint32)
            if op == 0:
                ro, rh, err = both(lambda: eo.place(EXPERT, ids), lambda: eh.place(EXPERT, ids))
                assert err is not None or np.array_equal(ro, rh)
            elif op == 1:
                ro, rh, err = both(lambda: eo.revoke(EXPERT, ids), lambda: eh.revoke(EXPERT, ids))
                assert err is not None or [int(i) for i in ro] == [int(i) for i in rh]
            elif op == 2:
                uniq = np.unique(ids)
                y = g.integers(0, 256, size=uniq.size * chunk, dtype=np.uint8)
                both(lambda: eo.evict(EXPERT, 0, uniq, y, None, np.arange(uniq.size), uniq.size),
                     lambda: eh.evict(EXPERT, 0, uniq, y, None, np.arange(uniq.size), uniq.size))
            elif op == 3 and last is not None:                          # from the staging buffer of the last fetch
                layer, kind, where, n_staging = last
                staged = [layer * E + e for e in range(E) if kind[e] == 2]
                if staged:
                    pick = [int(i) for i in g.permutation(staged)[:3]]
                    ranks = [int(where[i - layer * E]) for i in pick]
                    ro, rh, err = both(lambda: eo.place_from(EXPERT, pick, eo.last_staging(), None, ranks, n_staging),
                                       lambda: eh.place_from(EXPERT, pick, eh.last_staging(), None, ranks, n_staging))
                    assert err is None and np.array_equal(ro, rh)
                    n_from += int((ro == 0).sum())
            else:
                layer = int(g.integers(0, n_layers))
                n_tok = int(g.choice([0, 1, 3, 40, 9000]))
                topk = g.integers(0, E, size=(n_tok, 4)).astype(np.int32)
                if n_tok:
                    topk[g.random(topk.shape) < 0.01] = int(g.integers(-2, E + 3))
                    if g.random() < 0.5:
                        topk = (topk // 3) * 3                          # a sparse set of experts
                n_staging = int(g.choice([E, E, 5, 1]))
                a, b = eo.fetch_experts(layer, topk, n_staging), eh.fetch_experts(layer, topk, n_staging)
                P.assert_experts_equal(a, b, f"step {step}")
                last = (layer, b[1], b[2], n_staging)
            for i in range(n):
                assert eo.lookup(EXPERT, i) == eh.lookup(EXPERT, i), (step, i)
        assert n_from > 3
        P.assert_tiers_equal(eo, eh, EXPERT, 1, what="after the random expert sequence")
    finally:
        eh.close(); eo.close()
