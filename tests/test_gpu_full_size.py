"""GPU parity at the real shapes of the benchmark's configs (32 KiB KV chunks at 32K-128K-token contexts, 150 MiB and
16.5 MiB experts), in the launch configuration bench.py times.  The only reduction is the number of model layers
materialised in the pools (per-step shapes - blocks per layer, expert size - are what the kernels see and stay real);
for KV the oracle materialises one layer and every fetch of that layer is compared in full."""
import sys

import numpy as np
import pytest

import workloads as W
from workloads import scenarios as S
import parity as P

pytestmark = pytest.mark.gpu


def say(msg):
    from conftest import live
    live(msg)


def _full_compare_step(t, every=10):
    return t % every == 0


def test_config2_long_context_decode_200_steps_real_shapes():
    """Config 2 as stated: 200 decode steps, step t gathers layer t mod 32 for all four sequences (12 045 blocks at the
    start, 0.74 GiB of payload per step) and appends one token to each.  All 32 layers are materialised on both sides.
    Every step's K and V destinations are compared through a position-dependent checksum (the HIP side's computed on
    the device, so nothing but counters and the miss list crosses PCIe), counts and miss list exactly, and every tenth
    step byte for byte.  The cache tier keeps K and V of a block side by side, as bench.py's default run does."""
    L, steps = 32, 200
    say(f"config 2 at real shapes, {L} layers materialised, {steps} steps")
    wl = W.kv_decode(seed=0, n_layers=L, n_steps=steps)
    assert int(sum(len(t) for t in wl.tables)) > 12000 and wl.shape.chunk_bytes == 32768
    eo, eh = P.make_engines(wl, hip_kwargs=dict(cache_planes_adjacent=True))
    eo.threads = 8
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        assert np.array_equal(ro.place_status, rh.place_status)
        full = 0
        for t in range(steps):
            layer = t % L
            if _full_compare_step(t):
                got = rh.fetch(layer)
                P.assert_kv_equal(ro.fetch(layer), got, f"config 2 step {t}")
                full += 1
                say(f"  step {t}: layer {layer}, {got[3]['n_requests']} blocks compared byte for byte")
            else:
                got = rh.fetch(layer, digest=True)
                want = ro.fetch(layer, digest=True)
                assert want[0] == got[0] and want[1] == got[1], f"config 2 step {t}: checksums of K / V differ"
                assert want[3] == got[3] and np.array_equal(want[2], got[2]), f"config 2 step {t}: counts / miss list"
            ro.append(t); rh.append(t)
        assert full == 20 and got[3]["n_cache"] > 8000 and got[3]["n_host"] > 3000
        assert sum(len(t) for t in rh.tables) > int(sum(len(t) for t in wl.tables)) + 40      # tails rolled over
        P.assert_dirs_equal(eo, eh, S.KV, wl.n_objects)
    finally:
        eh.close(); eo.close()


def test_config3_phi_shaped_experts_real_size():
    say("config 3: 150 MiB experts, 2 layers materialised")
    ex = W.expert_offload(seed=0, shape=W.ExpertShape(n_layers=2))
    assert ex.shape.chunk_bytes == 150 * 2**20
    eo, eh = P.make_engines(ex_wl=ex)
    try:
        xo, xh = S.ExpertRun(eo, ex), S.ExpertRun(eh, ex)
        assert np.array_equal(xo.place_status, xh.place_status)
        for t in range(2):
            for layer in range(2):
                say(f"  step {t} layer {layer}")
                P.assert_experts_equal(xo.fetch(t, layer), xh.fetch(t, layer), f"config 3 step {t} layer {layer}")
    finally:
        eh.close(); eo.close()


def test_config4_qwen_shaped_experts_lru_real_size():
    say("config 4: 16.5 MiB experts, LRU cache tier, 2 layers materialised")
    ex = W.expert_lru(seed=0, shape=W.ExpertShape(n_layers=2, n_experts=60, d_model=2048, d_ff=1408))
    assert ex.shape.chunk_bytes == 17301504 and ex.lru_capacity == 24
    eo, eh = P.make_engines(ex_wl=ex, poison=True)
    try:
        xo, xh = S.ExpertRun(eo, ex), S.ExpertRun(eh, ex)
        hits = 0
        for t in range(3):
            for layer in range(2):
                say(f"  step {t} layer {layer}")
                a, b = xo.fetch(t, layer), xh.fetch(t, layer)
                P.assert_experts_equal(a, b, f"config 4 step {t} layer {layer}")
                hits += b[4]["n_cache"]
                from_staging = t >= 1                    # the second half fills the cache tier from the staging buffer
                ua, ub = xo.lru_update(t, layer, from_staging), xh.lru_update(t, layer, from_staging)
                assert ua[0] == ub[0] and ua[1] == ub[1] and ua[2] == ub[2] and np.array_equal(ua[3], ub[3])
        assert hits >= 2 * 2 * 20
        P.assert_dirs_equal(eo, eh, S.EXPERT, ex.n_objects)
    finally:
        eh.close(); eo.close()


@pytest.mark.parametrize("two_streams,steps", [(True, 500), (False, 60)], ids=["two-streams-500-steps", "one-stream-60-steps"])
def test_config5_revocation_stress_real_shapes(two_streams, steps):
    """Config 5 as stated: config 2's KV decode (2 layers materialised, real block counts) on one stream and config 3's
    expert fetch (1 layer of 16 experts of 150 MiB) on another, 500 steps; at t = 10, 20, ... a seeded quarter of the live
    cache-tier allocations of each class is revoked while both fetches of the step are in flight (poisoning on), at
    t = 5 mod 10 the revoked objects are placed again.  Every step's fetched bytes - K, V, staged experts - are compared
    with the oracle's through checksums, and byte for byte on every tenth step, which includes every revocation step.
    The one-stream variant runs both classes on the same stream (the wrapper's default)."""
    say(f"config 5: KV (2 layers) + experts (1 layer), {steps} steps, two streams {two_streams}, revocations in flight")
    wl = W.kv_decode(seed=0, n_layers=2, n_steps=steps)
    ex = W.expert_offload(seed=0, shape=W.ExpertShape(n_layers=1))
    eo, eh = P.make_engines(wl, ex, poison=True, two_streams=two_streams)
    eo.threads = 8
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        xo, xh = S.ExpertRun(eo, ex), S.ExpertRun(eh, ex)
        n_revocations = 0
        for t in range(steps):
            layer = t % 2
            revoke_now = t % 10 == 0 and t > 0
            full = _full_compare_step(t)
            ha, hx = rh.fetch_begin(layer), xh.fetch_begin(t, 0)
            if revoke_now:                                            # while both fetches are in flight
                rk_o, rk_h = ro.revoke_quarter(t), rh.revoke_quarter(t)
                rx_o, rx_h = xo.revoke_quarter(t), xh.revoke_quarter(t)
                assert np.array_equal(rk_o[0], rk_h[0]) and rk_o[1] == rk_h[1]
                assert np.array_equal(rx_o[0], rx_h[0]) and rx_o[1] == rx_h[1]
                n_revocations += 1
                say(f"  step {t}: revoked {len(rk_o[0])} KV blocks and {len(rx_o[0])} experts with fetches in flight")
            # the oracle fetches after the revocation: the bytes must not depend on when the fetch resolved (the counts
            # may: a fetch that overlaps a revocation may still have been served from the slot)
            if full:
                b, y = eh.fetch_end(ha), eh.fetch_end(hx)
                P.assert_kv_equal(ro.fetch(layer), b, f"config 5 kv step {t}", counts=not revoke_now)
                P.assert_experts_equal(xo.fetch(t, 0), y, f"config 5 experts step {t}", counts=not revoke_now)
            else:
                b, y = eh.fetch_end(ha, digest=True), eh.fetch_end(hx, digest=True)
                a, x = ro.fetch(layer, digest=True), xo.fetch(t, 0, digest=True)
                assert a[0] == b[0] and a[1] == b[1], f"config 5 step {t}: checksums of K / V differ"
                assert a[3] == b[3] and np.array_equal(a[2], b[2]), f"config 5 step {t}: KV counts / miss list"
                assert x[0] == y[0], f"config 5 step {t}: checksum of the staged experts differs"
                assert np.array_equal(np.where(x[1] >= 3, 0, x[1]), y[1]) and np.array_equal(x[2][y[1] > 0], y[2][y[1] > 0])
                assert x[4] == y[4] and np.array_equal(x[3], y[3]), f"config 5 step {t}: expert counts / miss list"
            if t % 10 == 5:
                assert np.array_equal(ro.replace_revoked(), rh.replace_revoked())
                assert np.array_equal(xo.replace_revoked(), xh.replace_revoked())
            ro.append(t); rh.append(t)
            if t % 50 == 49:
                say(f"  step {t} done")
        assert n_revocations == (steps - 1) // 10
        P.assert_dirs_equal(eo, eh, S.KV, wl.n_objects)
        P.assert_dirs_equal(eo, eh, S.EXPERT, ex.n_objects)
    finally:
        eh.close(); eo.close()


def test_revocation_drains_fetches_that_are_still_queued():
    """Three fetches of ~4.5 ms each are queued back to back, then a quarter of the cache tier is revoked at once, with
    poisoning on, and other blocks are placed into the freed slots.  The last gather starts milliseconds after the
    revocation was requested: only the drain (Section 3.2: work in flight on the region finishes before it is freed)
    keeps it from reading poisoned or re-used slots."""
    say("drain ordering")
    wl = W.kv_decode(seed=5, n_layers=3, n_steps=1)
    eo, eh = P.make_engines(wl, poison=True, cache_slack=0)
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        want = [ro.fetch(layer) for layer in range(3)]
        handles = [rh.fetch_begin(layer) for layer in range(3)]           # ~13 ms of queued work
        ids_o, called_o = ro.revoke_quarter(0)
        ids_h, called_h = rh.revoke_quarter(0)                            # returns only after the drain
        assert np.array_equal(ids_o, ids_h) and called_o == called_h and len(ids_h) > 1500
        host_only = [b for b in range(wl.n_closed) if not wl.resident[b]][:len(ids_h)]
        st_o, st_h = eo.place(S.KV, host_only), eh.place(S.KV, host_only)  # re-use the freed slots for other blocks
        assert np.array_equal(st_o, st_h) and (st_h == 0).all()
        for layer in range(3):
            P.assert_kv_equal(want[layer], eh.fetch_end(handles[layer]), f"queued fetch {layer}", counts=False)
        for layer in range(3):                                            # and the new residency serves the same bytes
            a, b = ro.fetch(layer), rh.fetch(layer)
            P.assert_kv_equal(a, b, f"after re-use, layer {layer}")
            assert np.array_equal(a[0], want[layer][0]) and np.array_equal(a[1], want[layer][1])
    finally:
        eh.close(); eo.close()


def test_shared_cache_pool_real_shapes():
    """32 KiB KV chunks (2 layers materialised: 128 KiB objects) and 150 MiB experts carved best-fit from one pool that
    holds 80 % of what the placement draw asks for; a revocation round, other objects into the holes, re-placement."""
    say("shared cache pool at real shapes")
    wl = W.kv_decode(seed=0, n_layers=2, n_steps=12)
    ex = W.expert_offload(seed=0, shape=W.ExpertShape(n_layers=1))
    kv_obj = 2 * 2 * wl.shape.chunk_bytes
    demand = int(wl.resident.sum()) * kv_obj + int((ex.tier0 == 1).sum()) * ex.shape.chunk_bytes
    pool = int(0.8 * demand) // 4096 * 4096
    eo, eh = P.make_engines(wl, ex, poison=True, two_streams=True, shared_cache_bytes=pool)
    try:
        xo, xh = S.ExpertRun(eo, ex), S.ExpertRun(eh, ex)
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        assert np.array_equal(ro.place_status, rh.place_status) and np.array_equal(xo.place_status, xh.place_status)
        assert (xh.place_status == 0).all() and (rh.place_status != 0).any()
        for t in range(12):
            layer = t % 2
            say(f"  step {t}")
            ha, hx = rh.fetch_begin(layer), xh.fetch_begin(t, 0)
            P.assert_kv_equal(ro.fetch(layer), eh.fetch_end(ha), f"shared real kv step {t}")
            P.assert_experts_equal(xo.fetch(t, 0), eh.fetch_end(hx), f"shared real experts step {t}")
            if t == 4:
                a, b = ro.revoke_quarter(t), rh.revoke_quarter(t)
                assert np.array_equal(a[0], b[0]) and a[1] == b[1]
                a, b = xo.revoke_quarter(t), xh.revoke_quarter(t)
                assert np.array_equal(a[0], b[0]) and a[1] == b[1]
                other = [b for b in range(wl.n_closed)
                         if eo.lookup(S.KV, b)[0] == S.HOST and b not in ro.pending_replace][:1500]
                st_o, st_h = eo.place(S.KV, other), eh.place(S.KV, other)      # blocks move into the experts' holes
                assert np.array_equal(st_o, st_h) and (st_h == 0).sum() > 1000
                for r in (ro, rh):
                    r.live |= {int(i) for i, st in zip(other, st_o) if st == 0}
            if t == 8:
                st_x = xo.replace_revoked()
                assert np.array_equal(st_x, xh.replace_revoked()) and np.array_equal(ro.replace_revoked(), rh.replace_revoked())
                say(f"  re-placement statuses of the experts: {list(st_x)}")
            ro.append(t); rh.append(t)
        P.assert_dirs_equal(eo, eh, S.KV, wl.n_objects)
        P.assert_dirs_equal(eo, eh, S.EXPERT, ex.n_objects)
        st = eh.h.stats()
        runs = eo.shared_free_runs()
        assert st.shared_free_runs == len(runs) and st.shared_granules_free == sum(l for _, l in runs)
    finally:
        eh.close(); eo.close()


def test_config2_at_its_maximum_lengths():
    """All four sequences at the upper end of the length range (131 072 tokens): 32 768 blocks, 2 GiB of payload per
    fetch - the largest single fetch the configuration can ask for."""
    say("config 2, maximum lengths")
    wl = W.kv_decode(seed=1, n_layers=1, min_len=131072, max_len=131072, n_steps=2)
    assert int(sum(len(t) for t in wl.tables)) == 4 * 8192 + 4
    eo, eh = P.make_engines(wl)
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        for t in range(2):
            got = rh.fetch(0)
            say(f"  step {t}: comparing {got[3]['n_requests']} blocks")
            P.assert_kv_equal(ro.fetch(0), got, f"maximum lengths step {t}")
            ro.append(t); rh.append(t)
        assert got[3]["n_requests"] == 32772 and got[3]["n_cache"] > 20000 and got[3]["n_host"] > 8000
    finally:
        eh.close(); eo.close()
