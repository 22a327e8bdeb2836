"""CPU-only checks of the HIP library: it loads, exports exactly what include/harvest.h declares, its structs have
the layout the binding assumes, and its host-side logic (directory mirror, slot allocators, argument validation,
callback order) agrees with the oracle's directory under random operation sequences.  No kernel is launched: the
context is created with HARVEST_FLAG_NO_DEVICE."""
import os
import re
import subprocess
import ctypes

import numpy as np
import pytest

import oracle as O
import workloads as W
from paper_2602_00328_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "harvest.h")


def test_library_exports_every_declared_symbol_and_nothing_is_undeclared():
    text = open(HEADER).read()
    declared = set(re.findall(r"\b(harvest_[a-z_]+)\s*\(", text)) - {"harvest_revoke_cb"}
    assert declared == set(B.SYMBOLS), (declared ^ set(B.SYMBOLS))
    out = subprocess.check_output(["nm", "-D", "--defined-only", B.LIB_PATH], text=True)
    exported = {l.split()[-1] for l in out.splitlines() if " T " in l and "harvest_" in l}
    assert declared <= exported, declared - exported


def test_process_holds_exactly_one_hip_runtime():
    mapped = {l.split()[-1] for l in open("/proc/self/maps") if "libamdhip64" in l}
    assert len(mapped) == 1, mapped


def test_struct_layouts_match_the_header(tmp_path):
    src = tmp_path / "sz.c"
    src.write_text('#include <stdio.h>\n#include "harvest.h"\nint main(void){printf("%zu %zu %zu %zu %zu %zu\\n",'
                   'sizeof(harvest_class_config),sizeof(harvest_config),sizeof(harvest_fetch_counts),'
                   'sizeof(harvest_stats_t),sizeof(harvest_profile_t),offsetof(harvest_config,gather_wg_per_cu));return 0;}\n')
    exe = tmp_path / "sz"
    subprocess.check_call(["gcc", "-I", os.path.join(ROOT, "include"), "-o", str(exe), str(src)])
    got = [int(x) for x in subprocess.check_output([str(exe)], text=True).split()]
    want = [ctypes.sizeof(B.harvest_class_config), ctypes.sizeof(B.harvest_config),
            ctypes.sizeof(B.harvest_fetch_counts), ctypes.sizeof(B.harvest_stats_t),
            ctypes.sizeof(B.harvest_profile_t), B.harvest_config.gather_wg_per_cu.offset]
    assert got == want


def test_status_codes_agree_with_the_oracle_where_they_mean_the_same():
    assert (B.OK, B.EINVAL, B.ENOSPC, B.ENOENT, B.ELOST) == (O.OK, O.EINVAL, O.ENOSPC, O.ENOENT, O.ELOST)
    assert (B.HOST, B.CACHE, B.LOCAL, B.NONE) == (O.HOST, O.CACHE, O.LOCAL, O.NONE)
    assert B.lib.harvest_strerror(B.ENOSPC) == b"no free slot"


def spec(n_layers=2, n_planes=2, chunk=64, max_objects=40, n_host=48, n_cache=9, n_local=4, n_experts=0):
    return B.ClassSpec(n_layers, n_planes, chunk, max_objects, n_host, n_cache, n_local, n_experts)


def test_create_rejects_bad_configurations():
    for bad in (spec(chunk=40), spec(n_planes=3), spec(max_objects=0)):
        with pytest.raises(B.HarvestError) as e:
            B.Harvest(kv=bad, flags=B.FLAG_NO_DEVICE)
        assert e.value.code == B.EINVAL
    with pytest.raises(B.HarvestError):
        B.Harvest(flags=B.FLAG_NO_DEVICE)                                  # no class at all
    with pytest.raises(B.HarvestError):
        B.Harvest(expert=spec(n_layers=1, n_planes=1, n_experts=0), flags=B.FLAG_NO_DEVICE)
    h = B.Harvest(kv=spec(), flags=B.FLAG_NO_DEVICE)
    with pytest.raises(B.HarvestError) as e:
        h.register(B.EXPERT, 1, [0])                                       # class not configured
    assert e.value.code == B.ENOENT
    h.close()


def test_data_calls_refuse_to_run_without_a_device():
    h = B.Harvest(kv=spec(), expert=spec(n_layers=1, n_planes=1, n_experts=4), flags=B.FLAG_NO_DEVICE)
    rc = B.lib.harvest_fetch_kv(h.h, 0, None, None, 1, 1, None, None, None, 1, None)
    assert rc == B.ENODEV
    rc = B.lib.harvest_fetch_experts(h.h, 0, None, 1, 1, None, 0, None, None)
    assert rc == B.ENODEV
    assert B.lib.harvest_fetch_info(h.h, None, None, None, 0, None) == B.ENODEV
    assert B.lib.harvest_release_stream(h.h, None) == B.ENODEV
    h.close()


@pytest.mark.parametrize("seed", range(8))
def test_host_logic_matches_the_oracle_directory_under_random_operations(seed):
    sp = spec()
    h = B.Harvest(kv=sp, flags=B.FLAG_NO_DEVICE)
    oc = O.OracleClass(sp.n_layers, sp.n_planes, sp.chunk_bytes, sp.max_objects, sp.n_host_slots, sp.n_cache_slots,
                       sp.n_local_slots)
    g = W.rng(seed, 300)
    free_host = list(g.permutation(sp.n_host_slots))
    dummy = np.zeros(sp.n_layers * 8 * sp.chunk_bytes, np.uint8)

    def both(fo, fh):
        eo = eh = None
        try:
            ro = fo()
        except O.OracleError as e:
            ro, eo = None, e.code
        try:
            rh = fh()
        except B.HarvestError as e:
            rh, eh = None, e.code
        assert eo == eh, (eo, eh)
        return ro, rh

    for step in range(120):
        n = oc.n_objects
        op = int(g.integers(0, 6))
        if op == 0 and free_host:                                            # register
            k = int(g.integers(1, 4))
            hs = [int(free_host.pop()) for _ in range(min(k, len(free_host)))]
            tier = O.LOCAL if g.random() < 0.4 else O.HOST
            if tier == O.LOCAL and g.random() < 0.3:                       # lossy objects: no host slot
                free_host.extend(hs)
                ro, rh = both(lambda: oc.register(1, None, tier), lambda: h.register(B.KV, 1, None, tier))
                if ro is not None:
                    assert np.array_equal(ro, rh)
                continue
            if g.random() < 0.1:
                hs[0] = int(g.integers(-2, sp.n_host_slots + 2))            # maybe invalid or taken
            ro, rh = both(lambda: oc.register(len(hs), hs, tier), lambda: h.register(B.KV, len(hs), hs, tier))
            if ro is not None:
                assert np.array_equal(ro, rh)
            else:
                free_host.extend(hs[1:])
        elif n:
            ids = g.integers(0, n + (1 if g.random() < 0.05 else 0), size=int(g.integers(1, 6))).astype(np.uint32)
            if op == 1 and g.random() < 0.5:
                ro, rh = both(lambda: oc.place(ids), lambda: h.place(B.KV, ids))
                if ro is not None:
                    assert np.array_equal(ro, rh)
            elif op == 1:                                                   # the same decisions when the bytes come from a device copy
                sb = g.integers(0, 8 + (1 if g.random() < 0.1 else 0), size=ids.size).astype(np.uint64)
                ro, rh = both(lambda: oc.place_from(ids, dummy, dummy, sb, 8), lambda: h.place_from(B.KV, ids, None, None, sb, 8))
                if ro is not None:
                    assert np.array_equal(ro, rh)
            elif op == 2:
                n0, m0 = len(oc.revoked_log), len(h.revoked_log)
                both(lambda: oc.revoke(ids), lambda: h.revoke(B.KV, ids))
                assert oc.revoked_log[n0:] == [i for _c, i in h.revoked_log[m0:]]
            elif op in (3, 4):
                layer = int(g.integers(-1, sp.n_layers))
                flags = O.EVICT_DEMOTE if (op == 4 and layer < 0) else 0
                sb = g.integers(0, 8 + (1 if g.random() < 0.05 else 0), size=ids.size).astype(np.uint64)
                both(lambda: oc.evict(layer, ids, dummy, dummy, sb, 8, flags),
                     lambda: h.evict(B.KV, layer, ids, None, None, sb, 8, flags))
            elif g.random() < 0.7:
                both(lambda: oc.restore(ids[:2]), lambda: h.restore(B.KV, ids[:2]))       # mostly EINVAL: rarely all lost
                lost = [i for i in range(n) if oc.lookup(i)[0] == O.NONE][:2]
                if lost:
                    both(lambda: oc.restore(lost), lambda: h.restore(B.KV, lost))
            else:
                bad = int(n + 3)
                both(lambda: oc.lookup(bad), lambda: h.lookup(B.KV, bad))
        for i in range(oc.n_objects):
            assert oc.lookup(i) == h.lookup(B.KV, i), (step, i)
    st = h.stats()
    in_cache = sum(1 for i in range(oc.n_objects) if oc.lookup(i)[0] == O.CACHE)
    in_local = sum(1 for i in range(oc.n_objects) if oc.lookup(i)[0] == O.LOCAL)
    assert st.cache_slots_in_use[B.KV] == in_cache and st.local_slots_in_use[B.KV] == in_local
    h.close()
    oc.close()


def test_lossy_objects_host_logic():
    h = B.Harvest(kv=spec(n_cache=1), flags=B.FLAG_NO_DEVICE)
    a, a2 = h.register(B.KV, 2, None, B.LOCAL)
    with pytest.raises(B.HarvestError):
        h.register(B.KV, 1, None, B.HOST)
    with pytest.raises(B.HarvestError) as e:                       # one cache slot, two lossy objects
        h.evict(B.KV, -1, [a, a2], None, None, [0, 1], 4, B.EVICT_DEMOTE)
    assert e.value.code == B.ENOSPC and h.lookup(B.KV, a)[0] == B.LOCAL
    h.evict(B.KV, -1, [a], None, None, [0], 4, B.EVICT_DEMOTE)
    assert h.lookup(B.KV, a) == (B.CACHE, 0, 1, -1)
    h.revoke(B.KV, [a])
    assert h.lookup(B.KV, a)[:3] == (B.NONE, -1, 2) and h.revoked_log == [(B.KV, int(a))]
    assert list(h.place(B.KV, [a])) == [B.ELOST]
    with pytest.raises(B.HarvestError) as e:
        h.evict(B.KV, 0, [a], None, None, [0], 4)
    assert e.value.code == B.ELOST
    h.close()


# ---- shared cache pool: best-fit segments for both classes (Section 3.3) -----------------------------------------

def test_create_rejects_bad_shared_pools():
    kv = spec(n_cache=0)
    for kw in (dict(shared_cache_bytes=4096, shared_granule=100), dict(shared_cache_bytes=4096, shared_granule=128),
               dict(shared_cache_bytes=4096 + 256, shared_granule=512), dict(shared_cache_bytes=0, shared_granule=512)):
        with pytest.raises(B.HarvestError) as e:
            B.Harvest(kv=kv, flags=B.FLAG_NO_DEVICE, **kw)
        assert e.value.code == B.EINVAL, kw
    h = B.Harvest(kv=kv, flags=B.FLAG_NO_DEVICE, shared_cache_bytes=8192)        # default granule: 4096
    st = h.stats()
    assert (st.shared_granules_free, st.shared_free_runs, st.shared_longest_free_run) == (2, 1, 2)
    h.close()


@pytest.mark.parametrize("seed", range(8))
def test_shared_pool_host_logic_matches_the_oracle_under_random_operations(seed):
    """KV objects of 3 granules (some of them lossy) and expert objects of 5 compete for 41 granules: every status, every
    directory entry and the free runs must agree with the oracle after every operation."""
    G = 256
    kv = spec(n_layers=3, chunk=128, max_objects=30, n_host=30, n_cache=0, n_local=5)
    ex = spec(n_layers=1, n_planes=1, chunk=5 * G - 16, max_objects=16, n_host=16, n_cache=0, n_local=0, n_experts=8)
    h = B.Harvest(kv=kv, expert=ex, flags=B.FLAG_NO_DEVICE, shared_cache_bytes=41 * G, shared_granule=G)
    pool = O.SegPool(41 * G, G)
    oc = {B.KV: O.OracleClass(3, 2, 128, 30, 30, 0, 5, segpool=pool),
          B.EXPERT: O.OracleClass(1, 1, 5 * G - 16, 16, 16, 0, 0, segpool=pool)}
    g = W.rng(seed, 310)
    free_host = {B.KV: list(g.permutation(30)), B.EXPERT: list(g.permutation(16))}
    dummy = np.zeros(3 * 8 * 5 * G, np.uint8)
    n_enospc = 0

    def both(fo, fh):
        eo = eh = None
        try:
            ro = fo()
        except O.OracleError as e:
            ro, eo = None, e.code
        try:
            rh = fh()
        except B.HarvestError as e:
            rh, eh = None, e.code
        assert eo == eh, (eo, eh)
        return ro, rh, eo

    for step in range(260):
        cls = B.KV if g.random() < 0.6 else B.EXPERT
        c = oc[cls]
        n = c.n_objects
        op = int(g.integers(0, 5))
        if op == 0 and (free_host[cls] or cls == B.KV):
            if cls == B.KV and g.random() < 0.35:                            # a lossy block in local HBM
                ro, rh, _ = both(lambda: c.register(1, None, O.LOCAL), lambda: h.register(cls, 1, None, B.LOCAL))
            elif free_host[cls]:
                hs = [int(free_host[cls].pop())]
                ro, rh, _ = both(lambda: c.register(1, hs, O.HOST), lambda: h.register(cls, 1, hs, B.HOST))
            else:
                continue
            if ro is not None:
                assert np.array_equal(ro, rh)
        elif n:
            ids = np.unique(g.integers(0, n, size=int(g.integers(1, 5)))).astype(np.uint32)
            g.shuffle(ids)
            if op in (1, 2):
                if g.random() < 0.5:
                    ro, rh, _ = both(lambda: c.place(ids), lambda: h.place(cls, ids))
                else:
                    sb = g.integers(0, 8, size=ids.size).astype(np.uint64)
                    ro, rh, _ = both(lambda: c.place_from(ids, dummy, dummy, sb, 8),
                                     lambda: h.place_from(cls, ids, None, None, sb, 8))
                assert np.array_equal(ro, rh)
                n_enospc += int((ro == O.ENOSPC).sum())
            elif op == 3:
                n0, m0 = len(c.revoked_log), len(h.revoked_log)
                both(lambda: c.revoke(ids), lambda: h.revoke(cls, ids))
                assert c.revoked_log[n0:] == [i for k, i in h.revoked_log[m0:] if k == cls]
            else:
                sb = np.arange(ids.size, dtype=np.uint64)
                _, _, err = both(lambda: c.evict(-1, ids, dummy, dummy, sb, 8, O.EVICT_DEMOTE),
                                 lambda: h.evict(cls, -1, ids, None, None, sb, 8, B.EVICT_DEMOTE))
                n_enospc += err == O.ENOSPC
        for k in oc:
            for i in range(oc[k].n_objects):
                assert oc[k].lookup(i) == h.lookup(k, i), (step, k, i)
        runs = pool.free_runs()
        st = h.stats()
        assert (st.shared_free_runs, st.shared_granules_free) == (len(runs), sum(l for _, l in runs)), step
        assert st.shared_longest_free_run == max([l for _, l in runs], default=0)
    assert n_enospc > 0
    in_cache = {k: sum(1 for i in range(oc[k].n_objects) if oc[k].lookup(i)[0] == O.CACHE) for k in oc}
    assert [st.cache_slots_in_use[k] for k in (B.KV, B.EXPERT)] == [in_cache[B.KV], in_cache[B.EXPERT]]
    h.close()
    for c in oc.values():
        c.close()
    pool.close()


def test_the_papers_three_calls():
    """harvest_alloc / harvest_free / harvest_register_cb (Section 3.2) against the oracle's place and revoke."""
    sp = spec(n_cache=2)
    h = B.Harvest(kv=sp, flags=B.FLAG_NO_DEVICE)
    oc = O.OracleClass(sp.n_layers, sp.n_planes, sp.chunk_bytes, sp.max_objects, sp.n_host_slots, 2, sp.n_local_slots)
    ids = h.register(B.KV, 4, [5, 6, 7, 8], B.HOST)
    oc.register(4, [5, 6, 7, 8], O.HOST)
    want = [int(oc.place([i])[0]) for i in ids]
    got = [h.alloc(B.KV, i) for i in ids]
    assert got == want == [B.OK, B.OK, B.ENOSPC, B.ENOSPC]
    for i in ids:
        assert oc.lookup(i) == h.lookup(B.KV, i)
    h.register_cb(B.KV, ids[1], enabled=False)                  # object 1 loses its callback
    h.free(B.KV, ids[0])                                        # given back by the application: no callback
    oc.revoke([ids[0]])
    assert h.revoked_log == [] and oc.lookup(ids[0]) == h.lookup(B.KV, ids[0]) == (O.HOST, -1, 2, 5)
    h.revoke(B.KV, [ids[1]]); oc.revoke([ids[1]])
    assert h.revoked_log == [] and oc.lookup(ids[1]) == h.lookup(B.KV, ids[1])
    assert h.alloc(B.KV, ids[2]) == B.OK and h.alloc(B.KV, ids[3]) == B.OK      # the freed slots are taken again
    oc.place([ids[2], ids[3]])
    h.register_cb(B.KV, ids[2])
    h.revoke(B.KV, [ids[2], ids[3]]); oc.revoke([ids[2], ids[3]])
    assert h.revoked_log == [(B.KV, int(ids[2])), (B.KV, int(ids[3]))]
    for i in ids:
        assert oc.lookup(i) == h.lookup(B.KV, i)
    with pytest.raises(B.HarvestError) as e:
        h.free(B.KV, 99)
    assert e.value.code == B.ENOENT
    with pytest.raises(B.HarvestError) as e:
        h.register_cb(B.KV, 99)
    assert e.value.code == B.ENOENT
    h.close(); oc.close()
