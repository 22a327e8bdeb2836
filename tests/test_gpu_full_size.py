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
    print(msg, flush=True)
    sys.stdout.flush()


def test_config2_long_context_decode_real_shapes():
    L, check_layer, steps = 4, 1, 34
    say(f"config 2 at real per-step shapes, {L} layers materialised, oracle on layer {check_layer}")
    wl = W.kv_decode(seed=0, n_layers=L, n_steps=steps)
    assert int(sum(len(t) for t in wl.tables)) > 12000 and wl.shape.chunk_bytes == 32768
    eo, eh = P.make_engines(wl, kv_layers=[check_layer])
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        assert np.array_equal(ro.place_status, rh.place_status)
        compared = 0
        for t in range(steps):
            layer = t % L
            got = rh.fetch(layer)
            if layer == check_layer:
                say(f"  step {t}: comparing {got[3]['n_requests']} blocks")
                P.assert_kv_equal(ro.fetch(layer), got, f"config 2 step {t}")
                compared += 1
            ro.append(t); rh.append(t)
        assert compared >= 8 and got[3]["n_cache"] > 8000 and got[3]["n_host"] > 3000
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


def test_config5_revocation_stress_real_shapes_two_streams():
    say("config 5: config 2 KV (2 layers) on one stream + config 3 experts (1 layer) on another, revocations in flight")
    wl = W.kv_decode(seed=0, n_layers=2, n_steps=26)
    ex = W.expert_offload(seed=0, shape=W.ExpertShape(n_layers=1))
    eo, eh = P.make_engines(wl, ex, poison=True, two_streams=True)
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        xo, xh = S.ExpertRun(eo, ex), S.ExpertRun(eh, ex)
        for t in range(26):
            layer = t % 2
            revoke_now = t % 10 == 0 and t > 0
            ha, hx = rh.fetch_begin(layer), xh.fetch_begin(t, 0)
            if revoke_now:                                            # while both fetches are in flight
                rk_o, rk_h = ro.revoke_quarter(t), rh.revoke_quarter(t)
                rx_o, rx_h = xo.revoke_quarter(t), xh.revoke_quarter(t)
                assert np.array_equal(rk_o[0], rk_h[0]) and rk_o[1] == rk_h[1]
                assert np.array_equal(rx_o[0], rx_h[0]) and rx_o[1] == rx_h[1]
                say(f"  step {t}: revoked {len(rk_o[0])} KV blocks and {len(rx_o[0])} experts with fetches in flight")
            b, y = eh.fetch_end(ha), eh.fetch_end(hx)
            if t % 2 == 0 or revoke_now:                              # compare every other step in full (1.5 GiB each)
                # the oracle fetches after the revocation: bytes must not depend on when the fetch resolved
                a, x = ro.fetch(layer), xo.fetch(t, 0)
                P.assert_kv_equal(a, b, f"config 5 kv step {t}", counts=not revoke_now)
                P.assert_experts_equal(x, y, f"config 5 experts step {t}", counts=not revoke_now)
            if t % 10 == 5:
                assert np.array_equal(ro.replace_revoked(), rh.replace_revoked())
                assert np.array_equal(xo.replace_revoked(), xh.replace_revoked())
            ro.append(t); rh.append(t)
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
