"""Pins for the CPU oracle: every check here compares the oracle with something other than itself -
self-describing payloads, closed forms, numpy library routines, brute-force enumeration with an
independent few-line model, and the invariants the paper fixes (Section 3.1: what the cache tier
holds must not change any result; Section 3.2: a revoked object is served from its host copy;
Section 5.2: blocks are found through the block table)."""
import itertools

import numpy as np
import pytest

import oracle as O
import workloads as W
from oracle import OracleClass, OracleError


def make_kv(n_layers=3, chunk=64, n_obj=40, n_cache=17, n_local=5, seed=0, poison=False, mode=W.FILL_TAG,
            extra_host=8, segpool=None):
    """Small KV class: objects start on the host, host slot != object id, payload = tag or normal fill."""
    n_host = n_obj + extra_host
    oc = OracleClass(n_layers, 2, chunk, n_obj + 8, n_host, 0 if segpool else n_cache, n_local, poison, segpool=segpool)
    hs = W.rng(seed, 100).permutation(n_host)[:n_obj]
    ids = oc.register(n_obj, hs, O.HOST)
    assert list(ids) == list(range(n_obj))
    so = np.full(n_host, W.NO_OBJECT, dtype=np.uint32)
    so[hs] = ids
    for p in range(2):
        W.fill_array(oc.plane(O.HOST, p), so, seed, W.CLS_KV, p, mode)
    oc.adopt(ids)
    return oc, ids, hs


def place_fraction(oc, ids, p, seed):
    order = W.rng(seed, 101).permutation(len(ids))
    n = int(round(p * len(ids)))
    chosen = np.asarray(ids)[order[:n]]
    st = oc.place(chosen)
    return chosen, st


def random_tables(n_obj, n_seq, max_blocks, seed):
    g = W.rng(seed, 102)
    n_blocks = g.integers(0, max_blocks + 1, size=n_seq).astype(np.int32)
    n_blocks[0] = max_blocks                     # one full row
    table = g.integers(0, n_obj, size=(n_seq, max_blocks)).astype(np.int32)   # duplicates allowed
    sdb = np.concatenate([[0], np.cumsum(n_blocks)[:-1]]).astype(np.uint64)
    return table, n_blocks, sdb, int(n_blocks.sum())


def check_tags(oc, dst, plane, layer, table, n_blocks, sdb, seed, chunk):
    for s in range(table.shape[0]):
        for j in range(n_blocks[s]):
            d = int(sdb[s]) + j
            assert W.check_tag(dst[d * chunk:(d + 1) * chunk], seed, W.CLS_KV, plane, layer, int(table[s, j])), \
                (plane, layer, s, j)


# ---- self-describing payload: no reference buffer at all --------------------------------------------------

@pytest.mark.parametrize("p_cache", [0.0, 0.3, 0.6, 1.0])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_fetch_kv_every_destination_word_names_its_request(p_cache, seed):
    chunk = 48
    oc, ids, _ = make_kv(n_layers=3, chunk=chunk, n_obj=40, n_cache=40, seed=seed)
    place_fraction(oc, ids, p_cache, seed)
    table, n_blocks, sdb, cap = random_tables(40, 5, 9, seed)
    for layer in range(3):
        k, v, miss, counts = oc.fetch_kv(layer, table, n_blocks, sdb, cap)
        check_tags(oc, k, 0, layer, table, n_blocks, sdb, seed, chunk)
        check_tags(oc, v, 1, layer, table, n_blocks, sdb, seed, chunk)
        assert counts["n_requests"] == cap and counts["n_invalid"] == 0 and counts["n_lost"] == 0


# ---- tier independence (Section 3.1) ----------------------------------------------------------------------

def test_fetch_is_identical_for_every_residency_assignment():
    results = {}
    for seed in (0, 1, 2):
        for p in (0.0, 0.3, 0.6, 1.0):
            oc, ids, _ = make_kv(n_layers=2, chunk=256, n_obj=64, n_cache=64, seed=seed, mode=W.FILL_NORMAL)
            place_fraction(oc, ids, p, seed + 7)
            table, n_blocks, sdb, cap = random_tables(64, 6, 11, seed)
            k, v, miss, counts = oc.fetch_kv(1, table, n_blocks, sdb, cap)
            kp, vp, _, _ = oc.fetch_kv(1, table, n_blocks, sdb, cap, plain=True)
            assert np.array_equal(k, kp) and np.array_equal(v, vp)
            results.setdefault(seed, []).append((k.copy(), v.copy(), counts))
    for seed, rs in results.items():
        for k, v, _ in rs[1:]:
            assert np.array_equal(k, rs[0][0]) and np.array_equal(v, rs[0][1])
        assert rs[0][2]["n_cache"] == 0 and rs[-1][2]["n_host"] == 0        # p = 0 and p = 1


# ---- library cross-checks ---------------------------------------------------------------------------------

def test_fetch_equals_numpy_take_on_the_host_plane():
    oc, ids, hs = make_kv(n_layers=2, chunk=128, n_obj=50, n_cache=20, seed=3, mode=W.FILL_NORMAL)
    place_fraction(oc, ids, 0.4, 3)
    table, n_blocks, sdb, cap = random_tables(50, 4, 10, 3)
    for layer in range(2):
        k, v, _, _ = oc.fetch_kv(layer, table, n_blocks, sdb, cap)
        flat = np.concatenate([table[s, :n_blocks[s]] for s in range(4)])
        for plane, got in ((0, k), (1, v)):
            want = np.take(oc.plane(O.HOST, plane)[layer], hs[flat], axis=0).reshape(-1)
            assert np.array_equal(got, want)


def test_torch_index_select_reproduces_the_gather():
    import torch
    oc, ids, hs = make_kv(n_layers=1, chunk=96, n_obj=30, n_cache=30, seed=4, mode=W.FILL_NORMAL)
    place_fraction(oc, ids, 1.0, 4)
    table, n_blocks, sdb, cap = random_tables(30, 3, 7, 4)
    k, _, _, _ = oc.fetch_kv(0, table, n_blocks, sdb, cap)
    flat = np.concatenate([table[s, :n_blocks[s]] for s in range(3)])
    slots = np.array([oc.lookup(b)[1] for b in flat])
    want = torch.index_select(torch.from_numpy(oc.plane(O.CACHE, 0)[0].copy()), 0, torch.from_numpy(slots))
    assert np.array_equal(k, want.numpy().reshape(-1))


def test_all_cached_identity_table_is_one_memcpy():
    n = 24
    oc, ids, _ = make_kv(n_layers=2, chunk=64, n_obj=n, n_cache=n, seed=5, mode=W.FILL_NORMAL)
    st = oc.place(ids)                                    # in id order: lowest free slot == id
    assert (st == O.OK).all()
    table = np.arange(n, dtype=np.int32).reshape(1, n)
    k, v, miss, counts = oc.fetch_kv(1, table, np.array([n], np.int32), np.array([0], np.uint64), n)
    assert np.array_equal(k, oc.plane(O.CACHE, 0)[1].reshape(-1))
    assert np.array_equal(v, oc.plane(O.CACHE, 1)[1].reshape(-1))
    assert miss.size == 0 and counts["n_cache"] == n


# ---- brute force on tiny inputs against an independent model ----------------------------------------------

def test_brute_force_three_blocks_all_tables_residencies_and_revocations():
    """3 blocks, 1 layer, every order of the table, every subset placed, every subset then revoked.
    Model: a dict block -> bytes (the value never changes) and a dict block -> 'H'/'C'."""
    chunk = 16
    for perm in itertools.permutations(range(3)):
        for placed in itertools.product([0, 1], repeat=3):
            for revoked in itertools.product([0, 1], repeat=3):
                oc = OracleClass(1, 2, chunk, 3, 3, 3, 0, poison=True)
                ids = oc.register(3, [2, 0, 1], O.HOST)
                value = {}
                for b in range(3):
                    kb = np.full(chunk, 10 + b, np.uint8); vb = np.full(chunk, 20 + b, np.uint8)
                    oc.set_object(b, kb, vb)
                    value[b] = (kb, vb)
                where = {b: "H" for b in range(3)}
                oc.place([b for b in range(3) if placed[b]])
                for b in range(3):
                    if placed[b]: where[b] = "C"
                oc.revoke([b for b in range(3) if revoked[b]])
                for b in range(3):
                    if revoked[b]: where[b] = "H"
                table = np.array([perm], dtype=np.int32)
                k, v, miss, counts = oc.fetch_kv(0, table, np.array([3], np.int32), np.array([0], np.uint64), 3)
                for j, b in enumerate(perm):
                    assert np.array_equal(k[j * chunk:(j + 1) * chunk], value[b][0])
                    assert np.array_equal(v[j * chunk:(j + 1) * chunk], value[b][1])
                assert sorted(miss) == [j for j, b in enumerate(perm) if where[b] == "H"]
                assert counts["n_cache"] == sum(1 for b in perm if where[b] == "C")
                for b in range(3):
                    assert oc.lookup(b)[0] == (O.CACHE if where[b] == "C" else O.HOST)
                    assert oc.lookup(b)[2] == placed[b] + (placed[b] and revoked[b])
                oc.close()


# ---- round trips (Sections 5.1-5.2) ------------------------------------------------------------------------

def test_evict_of_fetched_bytes_is_identity_and_evict_of_new_bytes_is_returned():
    chunk = 80
    oc, ids, _ = make_kv(n_layers=2, chunk=chunk, n_obj=32, n_cache=20, seed=6, mode=W.FILL_NORMAL)
    place_fraction(oc, ids, 0.5, 6)
    perm = W.rng(6, 1).permutation(32).astype(np.int32)
    table = perm.reshape(4, 8)
    nb = np.full(4, 8, np.int32); sdb = (np.arange(4) * 8).astype(np.uint64)
    before = [oc.fetch_kv(l, table, nb, sdb, 32)[:2] for l in range(2)]
    host_before = [oc.plane(O.HOST, p).copy() for p in range(2)]
    cache_before = [oc.plane(O.CACHE, p).copy() for p in range(2)]
    for l in range(2):
        oc.evict(l, table.reshape(-1), before[l][0], before[l][1], np.arange(32), 32)
    for p in range(2):
        assert np.array_equal(oc.plane(O.HOST, p), host_before[p])
        assert np.array_equal(oc.plane(O.CACHE, p), cache_before[p])
    # new bytes
    g = W.rng(6, 2)
    yk = g.integers(0, 256, size=32 * chunk, dtype=np.uint8); yv = g.integers(0, 256, size=32 * chunk, dtype=np.uint8)
    oc.evict(1, table.reshape(-1), yk, yv, np.arange(32), 32)
    k, v, _, _ = oc.fetch_kv(1, table, nb, sdb, 32)
    assert np.array_equal(k, yk) and np.array_equal(v, yv)
    k0, v0, _, _ = oc.fetch_kv(0, table, nb, sdb, 32)      # the other layer is untouched
    assert np.array_equal(k0, before[0][0]) and np.array_equal(v0, before[0][1])
    # every copy of a cached object stays identical to its host copy
    for b in range(32):
        t, slot, _, hs = oc.lookup(b)
        if t == O.CACHE:
            for p in range(2):
                assert np.array_equal(oc.plane(O.CACHE, p)[:, slot], oc.plane(O.HOST, p)[:, hs])
    # a revoked object is then served, with the new bytes, from the host
    cached = [b for b in range(32) if oc.lookup(b)[0] == O.CACHE]
    oc.revoke(cached)
    k, v, miss, _ = oc.fetch_kv(1, table, nb, sdb, 32)
    assert np.array_equal(k, yk) and np.array_equal(v, yv) and miss.size == 32


def test_evict_all_layers_layout_and_duplicate_rejection():
    chunk, L = 32, 3
    oc, ids, _ = make_kv(n_layers=L, chunk=chunk, n_obj=10, n_cache=10, seed=7)
    oc.place([1, 4])
    stride = 6
    g = W.rng(7, 3)
    sk = g.integers(0, 256, size=L * stride * chunk, dtype=np.uint8)
    sv = g.integers(0, 256, size=L * stride * chunk, dtype=np.uint8)
    ev = np.array([4, 7, 1], np.uint32); sb = np.array([5, 0, 2], np.uint64)
    oc.evict(-1, ev, sk, sv, sb, stride)
    for l in range(L):
        table = ev.astype(np.int32).reshape(1, 3)
        k, v, _, _ = oc.fetch_kv(l, table, np.array([3], np.int32), np.array([0], np.uint64), 3)
        for j in range(3):
            o = (l * stride + int(sb[j])) * chunk
            assert np.array_equal(k[j * chunk:(j + 1) * chunk], sk[o:o + chunk])
            assert np.array_equal(v[j * chunk:(j + 1) * chunk], sv[o:o + chunk])
    snap = [oc.plane(O.HOST, p).copy() for p in range(2)]
    with pytest.raises(OracleError) as e:
        oc.evict(0, [2, 3, 2], sk, sv, [0, 1, 2], stride)
    assert e.value.code == O.EINVAL
    with pytest.raises(OracleError) as e:
        oc.evict(0, [2], sk, sv, [stride], stride)
    assert e.value.code == O.EINVAL
    with pytest.raises(OracleError) as e:
        oc.evict(0, [99], sk, sv, [0], stride)
    assert e.value.code == O.ENOENT
    for p in range(2):
        assert np.array_equal(oc.plane(O.HOST, p), snap[p])


# ---- revocation (Section 3.2) -----------------------------------------------------------------------------

@pytest.mark.parametrize("poison", [False, True])
def test_revocation_falls_back_to_host_and_grows_the_miss_set_exactly(poison):
    chunk = 64
    oc, ids, _ = make_kv(n_layers=2, chunk=chunk, n_obj=48, n_cache=48, seed=8, poison=poison, mode=W.FILL_NORMAL)
    placed, _ = place_fraction(oc, ids, 0.7, 8)
    table, n_blocks, sdb, cap = random_tables(48, 5, 12, 8)
    k0, v0, miss0, c0 = oc.fetch_kv(0, table, n_blocks, sdb, cap)
    R = placed[W.rng(8, 9).permutation(placed.size)[:placed.size // 3]]
    slots = [oc.lookup(b)[1] for b in R]
    gens = [oc.lookup(b)[2] for b in R]
    oc.revoke(R)
    assert oc.revoked_log == [int(b) for b in R]              # callbacks, in order, once each
    for b, g in zip(R, gens):
        assert oc.lookup(b)[:3] == (O.HOST, -1, g + 1)
    if poison:
        for s in slots:
            assert (oc.plane(O.CACHE, 0)[:, s] == O.POISON).all() and (oc.plane(O.CACHE, 1)[:, s] == O.POISON).all()
    k1, v1, miss1, c1 = oc.fetch_kv(0, table, n_blocks, sdb, cap)
    assert np.array_equal(k0, k1) and np.array_equal(v0, v1)
    grown = set(miss1) - set(miss0)
    want = {s * table.shape[1] + j for s in range(table.shape[0]) for j in range(n_blocks[s])
            if table[s, j] in set(int(b) for b in R)}
    assert grown == want and set(miss0) <= set(miss1)
    assert c1["n_host"] == c0["n_host"] + len(want) and c1["n_cache"] == c0["n_cache"] - len(want)
    # revoking again, or revoking host objects, is a no-op with no callback
    oc.revoke(R)
    assert len(oc.revoked_log) == len(R)
    # freed slots are reused lowest first
    st = oc.place(R[:3])
    assert (st == O.OK).all()
    assert sorted(oc.lookup(b)[1] for b in R[:3]) == sorted(slots)[:3]
    assert [oc.lookup(b)[2] for b in R[:3]] == [g + 2 for g in gens[:3]]


def test_miss_list_is_exactly_the_host_and_lost_requests_in_request_order():
    oc, ids, _ = make_kv(n_layers=1, chunk=32, n_obj=30, n_cache=30, seed=9)
    place_fraction(oc, ids, 0.5, 9)
    table, n_blocks, sdb, cap = random_tables(30, 4, 8, 9)
    _, _, miss, counts = oc.fetch_kv(0, table, n_blocks, sdb, cap)
    want = [s * 8 + j for s in range(4) for j in range(n_blocks[s]) if oc.lookup(table[s, j])[0] in (O.HOST, O.NONE)]
    assert list(miss) == want and counts["n_host"] == len(want)


# ---- placement (Sections 3.2, 4.3) ------------------------------------------------------------------------

def test_place_takes_lowest_free_slot_copies_the_host_bytes_and_reports_enospc():
    oc, ids, hs = make_kv(n_layers=2, chunk=32, n_obj=12, n_cache=4, seed=10, mode=W.FILL_NORMAL)
    st = oc.place([7, 3, 9])
    assert list(st) == [O.OK] * 3
    assert [oc.lookup(b)[:3] for b in (7, 3, 9)] == [(O.CACHE, 0, 1), (O.CACHE, 1, 1), (O.CACHE, 2, 1)]
    for b in (7, 3, 9):
        for p in range(2):
            assert np.array_equal(oc.plane(O.CACHE, p)[:, oc.lookup(b)[1]], oc.plane(O.HOST, p)[:, hs[b]])
    st = oc.place([3, 5, 6, 6])                  # already cached -> OK no-op; one slot left; then full
    assert list(st) == [O.OK, O.OK, O.ENOSPC, O.ENOSPC]
    assert oc.lookup(3)[:3] == (O.CACHE, 1, 1) and oc.lookup(5)[:3] == (O.CACHE, 3, 1)
    assert oc.lookup(6)[:3] == (O.HOST, -1, 0)
    oc.revoke([3])
    assert list(oc.place([6])) == [O.OK] and oc.lookup(6)[:3] == (O.CACHE, 1, 1)
    with pytest.raises(OracleError) as e:
        oc.place([0, 500])
    assert e.value.code == O.ENOENT and oc.lookup(0)[0] == O.HOST


def test_place_from_a_copy_in_device_memory_writes_those_bytes_and_never_touches_the_host():
    """Section 3.2: the allocation only allocates, every copy is explicit - so the new cache-tier copy may be filled from
    wherever the application holds the bytes.  Closed form: slot bytes == the named source bytes, layer by layer."""
    oc, ids, hs = make_kv(n_layers=2, chunk=32, n_obj=12, n_cache=4, seed=13, mode=W.FILL_NORMAL)
    stride = 5
    g = W.rng(13, 200)
    src = [g.integers(0, 256, size=(2, stride, 32), dtype=np.uint8) for _ in range(2)]      # unlike any host bytes
    host_before = [oc.plane(O.HOST, p).copy() for p in range(2)]
    st = oc.place_from([7, 3, 9], src[0], src[1], [4, 0, 2], stride)
    assert list(st) == [O.OK] * 3
    assert [oc.lookup(b)[:3] for b in (7, 3, 9)] == [(O.CACHE, 0, 1), (O.CACHE, 1, 1), (O.CACHE, 2, 1)]
    for b, blk in ((7, 4), (3, 0), (9, 2)):
        for p in range(2):
            for l in range(2):
                assert np.array_equal(oc.plane(O.CACHE, p)[l, oc.lookup(b)[1]], src[p][l, blk]), (b, p, l)
    assert all(np.array_equal(oc.plane(O.HOST, p), host_before[p]) for p in range(2))
    # a fetch is served from the cache-tier copy while it exists, and from the host copy after revocation
    table, nb, sdb = np.array([[3, 7, 5]], np.int32), np.array([3], np.int32), np.array([0], np.uint64)
    k, v, miss, counts = oc.fetch_kv(1, table, nb, sdb, 3)
    assert np.array_equal(k[:32], src[0][1, 0]) and np.array_equal(v[32:64], src[1][1, 4]) and list(miss) == [2]
    assert np.array_equal(k[64:], host_before[0][1, hs[5]])
    oc.revoke([3, 7])
    k, v, miss, counts = oc.fetch_kv(1, table, nb, sdb, 3)
    assert np.array_equal(k[:32], host_before[0][1, hs[3]]) and np.array_equal(v[32:64], host_before[1][1, hs[7]])
    # statuses as for place: no-op for what is already in HBM (nothing written), one slot... then full; errors change nothing
    cache_before = [oc.plane(O.CACHE, p).copy() for p in range(2)]
    st = oc.place_from([9, 5, 6, 1, 2], src[0], src[1], [1, 1, 3, 0, 4], stride)
    assert list(st) == [O.OK, O.OK, O.OK, O.OK, O.ENOSPC]
    assert oc.lookup(9)[:3] == (O.CACHE, 2, 1) and np.array_equal(oc.plane(O.CACHE, 0)[:, 2], cache_before[0][:, 2])
    assert [oc.lookup(b)[:2] for b in (5, 6, 1)] == [(O.CACHE, 0), (O.CACHE, 1), (O.CACHE, 3)]
    assert np.array_equal(oc.plane(O.CACHE, 1)[0, 3], src[1][0, 0]) and oc.lookup(2)[:3] == (O.HOST, -1, 0)
    for bad_ids, bad_blk, code in (([0, 500], [0, 0], O.ENOENT), ([0, 4], [0, stride], O.EINVAL)):
        with pytest.raises(OracleError) as e:
            oc.place_from(bad_ids, src[0], src[1], bad_blk, stride)
        assert e.value.code == code and oc.lookup(0)[0] == O.HOST
    oc.close()


def test_place_from_the_host_bytes_is_place():
    """Special case that reduces to the pinned routine: a source holding exactly the host copies leaves the same
    directory and the same cache tier as orc_place - with equal-size slots and with best-fit segments."""
    for shared in (False, True):
        pools = [O.SegPool(22 * 64, 64) if shared else None for _ in range(2)]       # four objects of 5 granules, 2 to spare
        a, ids, hs = make_kv(n_layers=3, chunk=48, n_obj=10, n_cache=3, seed=14, segpool=pools[0])
        b, _, _ = make_kv(n_layers=3, chunk=48, n_obj=10, n_cache=3, seed=14, segpool=pools[1])
        order = [4, 8, 1, 4, 6, 0]                                    # a repeat; more than fits either way
        st_a = a.place(order)
        blk = W.rng(14, 201).permutation(12)[:len(order)]
        src = [np.zeros((3, 12, 48), np.uint8) for _ in range(2)]
        for i, obj in enumerate(order):
            for p in range(2):
                src[p][:, blk[i]] = b.plane(O.HOST, p)[:, hs[obj]]
        st_b = b.place_from(order, src[0], src[1], blk, 12)
        assert list(st_a) == list(st_b) and O.ENOSPC in st_a and list(st_a).count(O.OK) >= 4
        assert [a.lookup(i) for i in ids] == [b.lookup(i) for i in ids]
        if shared:
            assert np.array_equal(pools[0].mem(), pools[1].mem()) and pools[0].free_runs() == pools[1].free_runs()
        else:
            assert all(np.array_equal(a.plane(O.CACHE, p), b.plane(O.CACHE, p)) for p in range(2))
        a.close(); b.close()
        for g in pools:
            if g:
                g.close()


def test_fetch_never_changes_the_directory_or_any_tier():
    oc, ids, _ = make_kv(n_layers=2, chunk=32, n_obj=20, n_cache=8, n_local=3, seed=11)
    place_fraction(oc, ids, 0.4, 11)
    snap_dir = [oc.lookup(b) for b in range(20)]
    snap = [oc.plane(w, p).copy() for w in (O.HOST, O.CACHE, O.LOCAL) for p in range(2)]
    table, n_blocks, sdb, cap = random_tables(20, 4, 6, 11)
    oc.fetch_kv(1, table, n_blocks, sdb, cap)
    assert snap_dir == [oc.lookup(b) for b in range(20)]
    for a, (w, p) in zip(snap, [(w, p) for w in (O.HOST, O.CACHE, O.LOCAL) for p in range(2)]):
        assert np.array_equal(a, oc.plane(w, p))


# ---- local tier, demotion, lossy objects ------------------------------------------------------------------

def test_local_objects_append_evict_demote_then_place():
    chunk, L = 64, 2
    oc, ids, hs = make_kv(n_layers=L, chunk=chunk, n_obj=6, n_cache=4, n_local=2, seed=12, extra_host=8)
    free = sorted(set(range(oc.n_slots[O.HOST])) - set(int(h) for h in hs))
    tail = oc.register(2, free[:2], O.LOCAL)
    assert [oc.lookup(t)[:2] for t in tail] == [(O.LOCAL, 0), (O.LOCAL, 1)]
    with pytest.raises(OracleError) as e:
        oc.register(1, free[2:3], O.LOCAL)                         # local pool full
    assert e.value.code == O.ENOSPC
    with pytest.raises(OracleError) as e:
        oc.register(1, free[:1], O.HOST)                           # host slot taken
    assert e.value.code == O.EINVAL
    rows = {}
    for t in tail:
        for p in range(2):
            for l in range(L):
                for r in range(4):
                    d = W.rng(12, int(t), p, l, r).integers(0, 256, size=16, dtype=np.uint8)
                    oc.write_local(t, p, l, r * 16, d)
                    rows[(int(t), p, l, r)] = d
    table = np.array([[0, int(tail[0])], [int(tail[1]), 3]], np.int32)
    nb = np.array([2, 2], np.int32); sdb = np.array([0, 2], np.uint64)
    k, v, miss, counts = oc.fetch_kv(1, table, nb, sdb, 4)
    assert counts["n_local"] == 2 and counts["n_host"] == 2 and list(miss) == [0, 3]
    want_k = np.concatenate([rows[(int(tail[0]), 0, 1, r)] for r in range(4)])
    assert np.array_equal(k[chunk:2 * chunk], want_k)
    # write back + leave local HBM: source is the local pool itself
    oc.evict(-1, tail, oc.plane(O.LOCAL, 0), oc.plane(O.LOCAL, 1), [0, 1], oc.n_slots[O.LOCAL], O.EVICT_DEMOTE)
    assert [oc.lookup(t)[:3] for t in tail] == [(O.HOST, -1, 1), (O.HOST, -1, 1)]
    k2, v2, miss2, _ = oc.fetch_kv(1, table, nb, sdb, 4)
    assert np.array_equal(k, k2) and np.array_equal(v, v2) and list(miss2) == [0, 1, 2, 3]
    assert list(oc.place(tail)) == [O.OK, O.OK]
    k3, v3, miss3, _ = oc.fetch_kv(1, table, nb, sdb, 4)
    assert np.array_equal(k, k3) and np.array_equal(v, v3) and list(miss3) == [0, 3]
    fresh = oc.register(1, free[2:3], O.LOCAL)                      # the local slot is free again
    assert oc.lookup(fresh[0])[:2] == (O.LOCAL, 0)
    with pytest.raises(OracleError):                                 # demote needs all layers
        oc.evict(0, fresh, oc.plane(O.LOCAL, 0)[0], oc.plane(O.LOCAL, 1)[0], [0], 2, O.EVICT_DEMOTE)


def test_invalid_requests_are_skipped_and_counted():
    oc, ids, _ = make_kv(n_layers=1, chunk=32, n_obj=8, n_cache=8, seed=13)
    table = np.array([[0, -1, 2, 99], [3, 4, 5, 6]], np.int32)
    nb = np.array([4, 9], np.int32)                                  # 9 is clamped to max_blocks = 4
    sdb = np.array([0, 4], np.uint64)
    k = np.full(6 * 32, 0xEE, np.uint8); v = np.full(6 * 32, 0xEE, np.uint8)
    k, v, miss, counts = oc.fetch_kv(0, table, nb, sdb, 6, dst_k=k, dst_v=v)
    assert counts == dict(n_requests=8, n_local=0, n_cache=0, n_host=4, n_lost=0, n_invalid=4)
    assert list(miss) == [0, 2, 4, 5]
    for d in (1, 3):
        assert (k[d * 32:(d + 1) * 32] == 0xEE).all()
    assert W.check_tag(k[5 * 32:6 * 32], 13, W.CLS_KV, 0, 0, 4)


# ---- experts (Section 4.3) --------------------------------------------------------------------------------

def make_experts(n_layers=3, E=10, chunk=96, n_cache=12, n_local_per_layer=2, seed=0, lossy_local=False, segpool=None):
    n = n_layers * E
    oc = OracleClass(1, 1, chunk, n, n, 0 if segpool else n_cache, n_layers * n_local_per_layer, poison=True,
                     segpool=segpool)
    hs = W.rng(seed, 110).permutation(n)
    local = np.zeros(n, bool)
    for l in range(n_layers):
        local[l * E + W.rng(seed, 111, l).permutation(E)[:n_local_per_layer]] = True
    # registration is in id order, so tier changes run by run
    ids = []
    i = 0
    while i < n:
        j = i
        while j < n and local[j] == local[i]:
            j += 1
        ids.extend(oc.register(j - i, hs[i:j], O.LOCAL if local[i] else O.HOST))
        i = j
    assert ids == list(range(n))
    so = np.full(n, W.NO_OBJECT, np.uint32); so[hs] = np.arange(n)
    W.fill_array(oc.plane(O.HOST, 0), so, seed, W.CLS_EXPERT, 0, W.FILL_TAG)
    lo = np.full(oc.n_slots[O.LOCAL], W.NO_OBJECT, np.uint32)
    for b in np.nonzero(local)[0]:
        lo[oc.lookup(b)[1]] = b
    W.fill_array(oc.plane(O.LOCAL, 0), lo, seed, W.CLS_EXPERT, 0, W.FILL_TAG)
    oc.adopt(np.arange(n))
    return oc, local


def test_expert_fetch_union_ranks_and_bytes():
    E, chunk, seed = 10, 96, 3
    oc, local = make_experts(E=E, chunk=chunk, seed=seed)
    host_only = [b for b in range(3 * E) if not local[b]]
    oc.place(host_only[::2])
    g = W.rng(seed, 5)
    for layer in range(3):
        topk = g.integers(0, E, size=(7, 2)).astype(np.int32)
        staging, kind, where, miss, counts = oc.fetch_experts(layer, E, topk, E)
        U = sorted(set(int(e) for e in topk.reshape(-1)))
        assert [e for e in range(E) if kind[e] != O.UNSELECTED] == U
        rank = 0
        want_miss = []
        for e in U:
            b = layer * E + e
            t, slot, _, _ = oc.lookup(b)
            if t == O.LOCAL:
                assert kind[e] == O.IN_PLACE and where[e] == slot
                assert W.check_tag(oc.plane(O.LOCAL, 0)[0, slot], seed, W.CLS_EXPERT, 0, 0, b)
            else:
                assert kind[e] == O.STAGED and where[e] == rank
                assert W.check_tag(staging[rank * chunk:(rank + 1) * chunk], seed, W.CLS_EXPERT, 0, 0, b)
                if t == O.HOST:
                    want_miss.append(e)
                rank += 1
        assert list(miss) == want_miss
        assert counts["n_requests"] == len(U) and counts["n_local"] == sum(local[layer * E + e] for e in U)
        assert (staging[rank * chunk:] == 0).all()                 # nothing beyond the used staging slots


def test_expert_fetch_staging_overflow_invalid_ids_and_revocation():
    E, chunk, seed = 6, 32, 4
    oc, local = make_experts(n_layers=1, E=E, chunk=chunk, n_cache=6, n_local_per_layer=1, seed=seed)
    non_local = [e for e in range(E) if not local[e]]
    oc.place(non_local)
    topk = np.array([[0, 1], [2, 3], [4, 5], [-1, 6]], np.int32)
    staging, kind, where, miss, counts = oc.fetch_experts(0, E, topk, 3)
    assert counts["n_invalid"] == 2 + (len(non_local) - 3) and counts["n_cache"] == 3 and miss.size == 0
    assert [kind[e] for e in non_local] == [O.STAGED] * 3 + [O.OVERFLOW] * (len(non_local) - 3)
    s_before, *_ = oc.fetch_experts(0, E, topk, E)
    oc.revoke(non_local[1:3])
    s_after, kind, where, miss, counts = oc.fetch_experts(0, E, topk, E)
    assert np.array_equal(s_before, s_after) and list(miss) == non_local[1:3] and counts["n_host"] == 2


def test_lossy_object_is_lost_after_revocation_and_leaves_dst_untouched():
    """A lossy object has no host copy: leaving local HBM it can only go to the cache tier, and a revocation there
    loses it (Section 3.1: the application tolerates the loss and reconstructs)."""
    chunk = 32
    oc = OracleClass(2, 2, chunk, 6, 4, 2, 3, poison=True)
    a, a2, a3 = oc.register(3, None, O.LOCAL)
    with pytest.raises(OracleError):
        oc.register(1, None, O.HOST)                           # a lossy object needs a copy somewhere
    b = oc.register(1, [0], O.HOST)[0]
    rows = {}
    for obj in (a, a2, a3):
        for p in range(2):
            for l in range(2):
                rows[(obj, p, l)] = W.rng(15, int(obj), p, l).integers(0, 256, size=chunk, dtype=np.uint8)
                oc.write_local(obj, p, l, 0, rows[(obj, p, l)])
    oc.set_object(b, np.full(2 * chunk, 9, np.uint8), np.full(2 * chunk, 8, np.uint8))
    assert list(oc.place([a, b])) == [O.OK, O.OK] and oc.lookup(a)[0] == O.LOCAL      # local stays local; b takes slot 0
    with pytest.raises(OracleError) as e:                       # one cache slot left, two lossy objects to take in
        oc.evict(-1, [a, a2], oc.plane(O.LOCAL, 0), oc.plane(O.LOCAL, 1), [0, 1], 3, O.EVICT_DEMOTE)
    assert e.value.code == O.ENOSPC and oc.lookup(a)[:2] == (O.LOCAL, 0) and oc.lookup(a2)[:2] == (O.LOCAL, 1)
    oc.evict(-1, [a], oc.plane(O.LOCAL, 0), oc.plane(O.LOCAL, 1), [0], 3, O.EVICT_DEMOTE)
    assert oc.lookup(a) == (O.CACHE, 1, 1, -1)
    table = np.array([[int(a), int(b), int(a2)]], np.int32)
    nb, sdb = np.array([3], np.int32), np.array([0], np.uint64)
    for l in range(2):
        k, v, miss, counts = oc.fetch_kv(l, table, nb, sdb, 3)
        assert np.array_equal(k[:chunk], rows[(a, 0, l)]) and np.array_equal(v[:chunk], rows[(a, 1, l)])
        assert np.array_equal(k[2 * chunk:], rows[(a2, 0, l)])
        assert counts["n_cache"] == 2 and counts["n_local"] == 1 and miss.size == 0
    oc.revoke([a, b])
    assert oc.revoked_log == [int(a), int(b)]
    assert oc.lookup(a)[:3] == (O.NONE, -1, 2) and oc.lookup(b)[:3] == (O.HOST, -1, 2)
    k = np.full(3 * chunk, 0xEE, np.uint8); v = np.full(3 * chunk, 0xEE, np.uint8)
    k, v, miss, counts = oc.fetch_kv(0, table, nb, sdb, 3, dst_k=k, dst_v=v)
    assert (k[:chunk] == 0xEE).all() and (v[:chunk] == 0xEE).all()                   # lost: destination untouched
    assert (k[chunk:2 * chunk] == 9).all() and counts["n_lost"] == 1 and counts["n_host"] == 1 and list(miss) == [0, 1]
    assert list(oc.place([a])) == [O.ELOST]
    with pytest.raises(OracleError) as e:
        oc.evict(0, [a], k, v, [0], 3)
    assert e.value.code == O.ELOST
    # reconstruction: the lost object comes back into the lowest free local slot (a left slot 0 when it was demoted)
    for bad, code in (([b], O.EINVAL), ([a2], O.EINVAL), ([a, a], O.EINVAL), ([77], O.ENOENT)):
        with pytest.raises(OracleError) as e:
            oc.restore(bad)
        assert e.value.code == code and oc.lookup(a)[:3] == (O.NONE, -1, 2)
    oc.restore([a])
    assert oc.lookup(a) == (O.LOCAL, 0, 3, -1)
    rebuilt = {(p, l): W.rng(16, p, l).integers(0, 256, size=chunk, dtype=np.uint8) for p in range(2) for l in range(2)}
    for (p, l), row in rebuilt.items():
        oc.write_local(a, p, l, 0, row)
    for l in range(2):
        k, v, miss, counts = oc.fetch_kv(l, table, nb, sdb, 3)
        kp, vp, _, _ = oc.fetch_kv(l, table, nb, sdb, 3, plain=True)
        assert np.array_equal(k[:chunk], rebuilt[(0, l)]) and np.array_equal(v[:chunk], rebuilt[(1, l)])
        assert np.array_equal(k, kp) and np.array_equal(v, vp) and counts["n_lost"] == 0 and counts["n_local"] == 2


def test_restore_is_all_or_nothing_when_local_hbm_is_full():
    oc = OracleClass(1, 1, 16, 6, 1, 4, 2, poison=False)
    x, y = oc.register(2, None, O.LOCAL)
    for obj in (x, y):
        oc.write_local(obj, 0, 0, 0, np.full(16, int(obj) + 1, np.uint8))
    oc.evict(-1, [x, y], oc.plane(O.LOCAL, 0), None, [0, 1], 2, O.EVICT_DEMOTE)
    oc.revoke([x, y])
    z = oc.register(1, None, O.LOCAL)[0]                        # takes local slot 0: one slot left for two lost objects
    with pytest.raises(OracleError) as e:
        oc.restore([x, y])
    assert e.value.code == O.ENOSPC and oc.lookup(x)[0] == O.NONE and oc.lookup(y)[0] == O.NONE
    oc.restore([y])
    assert oc.lookup(y)[:3] == (O.LOCAL, 1, 3) and oc.lookup(z)[:2] == (O.LOCAL, 0)
    with pytest.raises(OracleError) as e:                       # the restored object owns its slot: local HBM is full
        oc.register(1, None, O.LOCAL)
    assert e.value.code == O.ENOSPC


# ---- random operation sequences: the invariants hold after every step ------------------------------------

@pytest.mark.parametrize("seed", range(6))
def test_random_operation_sequences_keep_tiered_and_plain_fetch_equal(seed):
    chunk, L, n = 32, 2, 24
    oc, ids, _ = make_kv(n_layers=L, chunk=chunk, n_obj=n, n_cache=9, n_local=0, seed=seed, poison=True,
                         mode=W.FILL_NORMAL)
    g = W.rng(seed, 200)
    model_tier = {b: O.HOST for b in range(n)}
    for step in range(60):
        op = g.integers(0, 4)
        sub = g.permutation(n)[:g.integers(1, 8)].astype(np.uint32)
        if op == 0:
            st = oc.place(sub)
            for b, s in zip(sub, st):
                if s == O.OK: model_tier[int(b)] = O.CACHE
            assert sum(1 for t in model_tier.values() if t == O.CACHE) <= 9
        elif op == 1:
            oc.revoke(sub)
            for b in sub: model_tier[int(b)] = O.HOST
        elif op == 2:
            layer = int(g.integers(-1, L))
            nl = L if layer < 0 else 1
            sk = g.integers(0, 256, size=nl * sub.size * chunk, dtype=np.uint8)
            sv = g.integers(0, 256, size=nl * sub.size * chunk, dtype=np.uint8)
            oc.evict(layer, sub, sk, sv, g.permutation(sub.size), sub.size)
        table, n_blocks, sdb, cap = random_tables(n, 3, 7, seed * 1000 + step)
        for layer in range(L):
            k, v, miss, counts = oc.fetch_kv(layer, table, n_blocks, sdb, cap)
            kp, vp, _, _ = oc.fetch_kv(layer, table, n_blocks, sdb, cap, plain=True)
            assert np.array_equal(k, kp) and np.array_equal(v, vp)
        for b in range(n):
            assert oc.lookup(b)[0] == model_tier[b]
        used = sorted(oc.lookup(b)[1] for b in range(n) if model_tier[b] == O.CACHE)
        assert len(set(used)) == len(used)                           # no two objects share a slot


def test_threads_do_not_change_the_result():
    oc, ids, _ = make_kv(n_layers=1, chunk=256, n_obj=200, n_cache=120, seed=14, mode=W.FILL_NORMAL)
    place_fraction(oc, ids, 0.6, 14)
    table, n_blocks, sdb, cap = random_tables(200, 8, 40, 14)
    a = oc.fetch_kv(0, table, n_blocks, sdb, cap, threads=1)
    b = oc.fetch_kv(0, table, n_blocks, sdb, cap, threads=4)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]) and list(a[2]) == list(b[2]) and a[3] == b[3]


# ---- head-major working layout ---------------------------------------------------------------------------------

@pytest.mark.parametrize("heads,bt,hb", [(8, 16, 256), (3, 4, 48), (1, 16, 32), (5, 1, 16)])
def test_head_major_fetch_is_the_transpose_of_the_token_major_fetch(heads, bt, hb):
    chunk = heads * bt * hb
    oc, ids, _ = make_kv(n_layers=2, chunk=chunk, n_obj=30, n_cache=20, seed=21, mode=W.FILL_NORMAL)
    place_fraction(oc, ids, 0.5, 21)
    g = W.rng(21, 1)
    n_seq, max_blocks = 3, 6
    nb = np.array([6, 2, 4], np.int32)
    table = g.integers(0, 30, size=(n_seq, max_blocks)).astype(np.int32)
    cap = np.array([7, 2, 5], np.uint32)                   # room beyond the current length stays untouched
    sdb = np.array([0, 7, 9], np.uint64)
    total = 14
    for layer in range(2):
        k_tm, v_tm, miss_tm, c_tm = oc.fetch_kv(layer, table, nb, sdb, total)
        k_hm, v_hm, miss_hm, c_hm = oc.fetch_kv_head_major(layer, table, nb, sdb, cap, total, heads, bt)
        assert list(miss_tm) == list(miss_hm) and c_tm == c_hm
        for tm, hm in ((k_tm, k_hm), (v_tm, v_hm)):
            for s in range(n_seq):
                lo, hi = int(sdb[s]) * chunk, (int(sdb[s]) + int(cap[s])) * chunk
                a = tm[lo:hi].reshape(int(cap[s]) * bt, heads, hb)            # [token][head][bytes]
                b = hm[lo:hi].reshape(heads, int(cap[s]) * bt, hb)            # [head][token][bytes]
                assert np.array_equal(np.transpose(a, (1, 0, 2)), b)


def test_head_major_fetch_rejects_what_does_not_fit():
    heads, bt, hb = 2, 4, 16
    chunk = heads * bt * hb
    oc, ids, _ = make_kv(n_layers=1, chunk=chunk, n_obj=10, n_cache=10, seed=22)
    table = np.array([[0, 1, 2, 3], [4, 5, 6, 99]], np.int32)
    nb = np.array([4, 4], np.int32)
    k = np.full(8 * chunk, 0xEE, np.uint8); v = np.full(8 * chunk, 0xEE, np.uint8)
    # sequence 0 has room for 3 of its 4 blocks; sequence 1's region would end beyond the destination
    k, v, miss, counts = oc.fetch_kv_head_major(0, table, nb, np.array([0, 5], np.uint64), np.array([3, 4], np.uint32), 8,
                                                heads, bt, dst_k=k, dst_v=v)
    assert counts["n_requests"] == 8 and counts["n_invalid"] == 5 and counts["n_host"] == 3
    assert (k[3 * chunk:] == 0xEE).all()
    with pytest.raises(OracleError):
        oc.fetch_kv_head_major(0, table, nb, np.array([0, 4], np.uint64), np.array([4, 4], np.uint32), 8, 3, bt)


# ---- variable-size segments shared by both classes, best-fit allocation (Section 3.3) ----------------------------

def bitmap_model(used, need):
    """The definition on a granule bitmap: list the maximal free runs; the shortest one that fits, the lowest of equals."""
    runs, i, n = [], 0, len(used)
    while i < n:
        if used[i]:
            i += 1
            continue
        j = i
        while j < n and not used[j]:
            j += 1
        runs.append((j - i, i))
        i = j
    fits = [r for r in runs if r[0] >= need]
    return (min(fits)[1] if fits else -1), sorted((o, l) for l, o in runs)


def test_best_fit_worked_example():
    """16 granules; after A B C D E fill the pool and A, C, E are freed the free runs are (0,5) (7,2) (12,4):
    first-fit, worst-fit and best-fit each answer the next requests differently."""
    g = O.SegPool(16 * 32, 32)
    assert [g.alloc(n) for n in (5, 2, 2, 3, 4)] == [0, 5, 7, 9, 12] and g.free_runs() == [] and g.alloc(1) == -1
    g.free(0, 5); g.free(7, 2); g.free(12, 4)
    assert g.free_runs() == [(0, 5), (7, 2), (12, 4)]
    assert g.alloc(2) == 7                       # the exact fit, not the first (0) or the largest (0) run
    assert g.alloc(3) == 12                      # the run of 4 leaves 1 behind, the run of 5 would leave 2
    assert g.free_runs() == [(0, 5), (15, 1)]
    assert g.alloc(1) == 15 and g.alloc(6) == -1 and g.alloc(5) == 0 and g.free_runs() == []
    g.free(9, 3); g.free(7, 2)                   # joins the run after it
    assert g.free_runs() == [(7, 5)]
    g.free(5, 2)                                 # joins the run after it again
    g.free(15, 1)                                # a run of its own
    assert g.free_runs() == [(5, 7), (15, 1)]
    g.free(12, 3)                                # closes the gap: joins both neighbours
    assert g.free_runs() == [(5, 11)]
    g.free(0, 5)
    assert g.free_runs() == [(0, 16)] and g.alloc(0) == -1
    g.close()


@pytest.mark.parametrize("seed", range(5))
def test_best_fit_agrees_with_the_bitmap_definition_on_random_sequences(seed):
    n = 97
    g = O.SegPool(n * 16, 16)
    used = np.zeros(n, bool)
    live = []
    r = W.rng(seed, 130)
    n_failed = 0
    for _ in range(600):
        if live and r.random() < 0.45:
            off, ln = live.pop(int(r.integers(len(live))))
            g.free(off, ln)
            used[off:off + ln] = False
        else:
            need = int(r.integers(1, 13))
            want, _ = bitmap_model(used, need)
            got = g.alloc(need)
            assert got == want, (seed, need)
            if got >= 0:
                used[got:got + need] = True
                live.append((got, need))
            else:
                n_failed += 1
        assert g.free_runs() == bitmap_model(used, 1)[1]
    assert n_failed > 5
    for off, ln in live:
        g.free(off, ln)
    assert g.free_runs() == [(0, n)]
    g.close()


def segment_bytes(pool, oc, slot, plane, layer):
    o = slot * pool.granule + (layer * oc.n_planes + plane) * oc.chunk_bytes
    return pool.mem()[o:o + oc.chunk_bytes]


def test_two_classes_share_one_segment_pool():
    """KV blocks (3 layers x 2 planes x 48 B = 288 B -> 5 granules of 64 B, 32 B of slack) and experts (400 B -> 7
    granules) draw from one pool: layout inside a segment, fragmentation, ENOSPC for the large class while the small
    one still fits, exact poisoning, and fetches that do not care."""
    pool = O.SegPool(44 * 64, 64)
    kv, ids, _ = make_kv(n_layers=3, chunk=48, n_obj=12, seed=20, poison=True, segpool=pool)
    ex, local = make_experts(n_layers=2, E=6, chunk=400, seed=21, segpool=pool)
    host_experts = [int(e) for e in np.nonzero(~local)[0]]
    # interleave: K0 K1 X0 K2 X1 K3 -> offsets 0 5 10 17 22 29, 34 of 44 granules used
    order = [(kv, 0), (kv, 1), (ex, host_experts[0]), (kv, 2), (ex, host_experts[1]), (kv, 3)]
    offs = []
    for c, i in order:
        assert list(c.place([i])) == [O.OK]
        offs.append(c.lookup(i)[1])
    assert offs == [0, 5, 10, 17, 22, 29] and pool.free_runs() == [(34, 10)]
    for b in range(4):                                               # [layer][plane][chunk] inside the segment
        for l in range(3):
            for p in range(2):
                assert W.check_tag(segment_bytes(pool, kv, kv.lookup(b)[1], p, l), 20, W.CLS_KV, p, l, b)
    for e in host_experts[:2]:
        assert W.check_tag(segment_bytes(pool, ex, ex.lookup(e)[1], 0, 0), 21, W.CLS_EXPERT, 0, 0, e)
    # fragment: revoke K1 (5 @ 5) and K2 (5 @ 17): 20 granules free, the longest run is 10 -> one expert fits, not two
    kv.revoke([1, 2])
    assert pool.free_runs() == [(5, 5), (17, 5), (34, 10)]
    m = pool.mem()
    assert (m[5 * 64:5 * 64 + 288] == O.POISON).all() and (m[5 * 64 + 288:10 * 64] == 0).all()   # the object, not the slack
    assert list(ex.place(host_experts[2:4])) == [O.OK, O.ENOSPC] and ex.lookup(host_experts[2])[1] == 34
    assert pool.free_runs() == [(5, 5), (17, 5), (41, 3)]
    assert list(kv.place([5, 6, 7])) == [O.OK, O.OK, O.ENOSPC]       # exact fits, lowest first; 3 granules are too few
    assert (kv.lookup(5)[1], kv.lookup(6)[1]) == (5, 17) and pool.free_runs() == [(41, 3)]
    # fetches resolve through the shared pool and equal the tier-free definition
    table = np.array([[0, 5, 1, 6, 3, 7, 2]], np.int32)
    nb, sdb = np.array([7], np.int32), np.array([0], np.uint64)
    for l in range(3):
        k, v, miss, counts = kv.fetch_kv(l, table, nb, sdb, 7)
        kp, vp, _, _ = kv.fetch_kv(l, table, nb, sdb, 7, plain=True)
        assert np.array_equal(k, kp) and np.array_equal(v, vp) and counts["n_cache"] == 4 and list(miss) == [2, 5, 6]
        check_tags(kv, k, 0, l, table, nb, sdb, 20, 48)
        check_tags(kv, v, 1, l, table, nb, sdb, 20, 48)
    in_cache = [e for e in host_experts[:3] if e < 6]                # layer 0's experts are objects 0..5
    assert in_cache
    topk = np.array([in_cache], np.int32)
    st, kind, where, miss, counts = ex.fetch_experts(0, 6, topk, 6)
    assert counts["n_cache"] == len(in_cache) and counts["n_host"] == 0
    for r, e in enumerate(sorted(in_cache)):
        assert W.check_tag(st[r * 400:(r + 1) * 400], 21, W.CLS_EXPERT, 0, 0, e)
    # everything revoked: the pool is one run again
    kv.revoke(list(range(12))); ex.revoke(list(range(12)))
    assert pool.free_runs() == [(0, 44)]
    kv.close(); ex.close(); pool.close()


def test_lossy_demotion_into_segments_is_all_or_nothing():
    pool = O.SegPool(5 * 64, 64)                                     # room for two objects of 2 granules, not three
    oc = OracleClass(1, 2, 64, 6, 2, 0, 3, poison=True, segpool=pool)
    a, b, c = oc.register(3, None, O.LOCAL)
    for obj in (a, b, c):
        for p in range(2):
            oc.write_local(obj, p, 0, 0, np.full(64, 10 * int(obj) + p + 1, np.uint8))
    lk, lv = oc.plane(O.LOCAL, 0), oc.plane(O.LOCAL, 1)
    with pytest.raises(OracleError) as e:
        oc.evict(-1, [a, b, c], lk, lv, [0, 1, 2], 3, O.EVICT_DEMOTE)
    assert e.value.code == O.ENOSPC and pool.free_runs() == [(0, 5)] and oc.lookup(a)[:2] == (O.LOCAL, 0)
    oc.evict(-1, [b, a], lk, lv, [1, 0], 3, O.EVICT_DEMOTE)
    assert oc.lookup(b)[:2] == (O.CACHE, 0) and oc.lookup(a)[:2] == (O.CACHE, 2) and pool.free_runs() == [(4, 1)]
    m = pool.mem()
    assert (m[0:64] == 11).all() and (m[64:128] == 12).all() and (m[128:192] == 1).all() and (m[192:256] == 2).all()
    oc.revoke([b])
    assert oc.lookup(b)[0] == O.NONE and pool.free_runs() == [(0, 2), (4, 1)] and (m[0:128] == O.POISON).all()
    oc.close(); pool.close()
