"""Shared helpers of the parity tests: build an oracle engine and a HIP engine over the same workload, compare what
they return, byte for byte."""
import numpy as np

import workloads as W
from workloads import scenarios as S


def make_engines(kv_wl=None, ex_wl=None, poison=False, two_streams=False, kv_layers=None, cache_slack=0,
                 local_slack=0, hip_kwargs=None, kv_spec=None, ex_spec=None, shared_cache_bytes=0, shared_granule=0):
    """shared_cache_bytes > 0: both classes carve their cache tier from one pool of that size (best-fit segments)."""
    from oracle.engine import OracleEngine
    from workloads.hip_engine import HipEngine
    shared = shared_cache_bytes > 0
    kv = kv_spec or (S.kv_spec(kv_wl, cache_slack, local_slack, shared=shared) if kv_wl is not None else None)
    ex = ex_spec or (S.expert_spec(ex_wl, shared=shared) if ex_wl is not None else None)
    eo = OracleEngine(kv=kv, expert=ex, poison=poison, kv_layers=kv_layers, shared_cache_bytes=shared_cache_bytes,
                      shared_granule=shared_granule)
    eh = HipEngine(kv=kv, expert=ex, poison=poison, two_streams=two_streams, shared_cache_bytes=shared_cache_bytes,
                   shared_granule=shared_granule, **(hip_kwargs or {}))
    return eo, eh


def assert_shared_pools_equal(eo, eh, what=""):
    a, b = eo.shared_plane(), eh.shared_plane()
    assert a.shape == b.shape
    assert np.array_equal(a, b), f"{what}: shared cache pool differs: {first_diff(a, b)}"
    st = eh.h.stats()
    runs = eo.shared_free_runs()
    assert st.shared_free_runs == len(runs) and st.shared_granules_free == sum(l for _, l in runs), what
    assert st.shared_longest_free_run == max([l for _, l in runs], default=0), what


def first_diff(a, b):
    d = np.nonzero(a != b)[0]
    return None if d.size == 0 else (int(d[0]), int(a[d[0]]), int(b[d[0]]), int(d.size))


def assert_kv_equal(o, h, what, counts=True):
    ko, vo, mo, co = o
    kh, vh, mh, ch = h
    assert ko.shape == kh.shape, what
    assert np.array_equal(ko, kh), f"{what}: K differs (first byte, oracle, hip, n): {first_diff(ko, kh)}"
    if vo is not None:
        assert np.array_equal(vo, vh), f"{what}: V differs (first byte, oracle, hip, n): {first_diff(vo, vh)}"
    if counts:
        assert co == ch, f"{what}: counts {co} != {ch}"
        assert np.array_equal(mo, mh), f"{what}: miss lists differ"


def assert_experts_equal(o, h, what, counts=True):
    oo, kind_o, where_o, mo, co = o
    oh, kind_h, where_h, mh, ch = h
    assert len(oo) == len(oh)
    for e, (a, b) in enumerate(zip(oo, oh)):
        assert (a is None) == (b is None), f"{what}: expert {e} presence differs"
        if a is not None:
            assert np.array_equal(a, b), f"{what}: expert {e} bytes differ: {first_diff(a, b)}"
    # oracle kinds 3 (overflow) and 4 (lost) both surface as a NULL pointer
    assert np.array_equal(np.where(kind_o >= 3, 0, kind_o), kind_h), f"{what}: kinds {kind_o} vs {kind_h}"
    if counts:
        sel = kind_h > 0
        assert np.array_equal(where_o[sel], where_h[sel]), f"{what}: staging ranks / local slots differ"
        assert co == ch, f"{what}: counts {co} != {ch}"
        assert np.array_equal(mo, mh), f"{what}: miss lists differ"


def assert_dirs_equal(eo, eh, cls, n, what=""):
    for i in range(n):
        assert eo.lookup(cls, i) == eh.lookup(cls, i), f"{what}: directory entry {i}: {eo.lookup(cls, i)} != {eh.lookup(cls, i)}"


def assert_tiers_equal(eo, eh, cls, n_planes, tiers=(S.HOST, S.CACHE, S.LOCAL), what=""):
    for tier in tiers:
        for p in range(n_planes):
            a, b = eo.tier_plane(cls, tier, p), eh.tier_plane(cls, tier, p)
            if a.size == 0 and b.size == 0:
                continue
            assert a.shape == b.shape
            assert np.array_equal(a, b), f"{what}: tier {tier} plane {p} differs: {first_diff(a.reshape(-1), b.reshape(-1))}"


def smoke():
    """One tiny pass of every entry point on cuda:0 against the oracle."""
    wl = W.kv_decode(seed=3, n_layers=2, n_seq=3, min_len=40, max_len=90, n_steps=20, fill_mode=W.FILL_TAG)
    ex = W.expert_offload(seed=3, shape=W.ExpertShape(n_layers=2, n_experts=8, d_model=32, d_ff=50), n_tokens=6,
                          fill_mode=W.FILL_TAG)
    for general in (False, True):              # the one-kernel form small tables take, then the general path
        eo, eh = make_engines(wl, ex, poison=True, hip_kwargs=dict(general_fetch=general))
        try:
            ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
            xo, xh = S.ExpertRun(eo, ex), S.ExpertRun(eh, ex)
            for t in range(20):
                assert_kv_equal(ro.step(t), rh.step(t), f"smoke kv step {t}")
                assert_experts_equal(xo.fetch(t, t % 2), xh.fetch(t, t % 2), f"smoke experts step {t}")
                if t == 10:
                    assert ro.revoke_quarter(t)[1] == rh.revoke_quarter(t)[1]
                    assert xo.revoke_quarter(t)[1] == xh.revoke_quarter(t)[1]
                if t == 15:
                    assert np.array_equal(ro.replace_revoked(), rh.replace_revoked())
                    assert np.array_equal(xo.replace_revoked(), xh.replace_revoked())
            assert_dirs_equal(eo, eh, S.KV, wl.n_objects, "smoke")
            assert_tiers_equal(eo, eh, S.KV, 2, what="smoke")
        finally:
            eh.close()
            eo.close()


def streams_run_independently(dev, a, b, ms=30.0):
    """True if work on stream b completes while stream a is still busy: a sleeping kernel of about `ms` on a, a tiny fill
    on b.  False when the device runs the two streams one after the other (HIP has a few hardware queues - 4 here - and
    streams that map to the same one take turns)."""
    import torch
    torch.cuda.synchronize()
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(a):
        t0.record(); torch.cuda._sleep(20_000_000); t1.record()
    torch.cuda.synchronize()
    cycles = int(20_000_000 * ms / max(t0.elapsed_time(t1), 1e-3))
    flag = torch.zeros(64, dtype=torch.uint8, device=dev)
    still = torch.cuda.Event()
    with torch.cuda.stream(a):
        torch.cuda._sleep(cycles); still.record()
    with torch.cuda.stream(b):
        flag.fill_(1)
    b.synchronize()
    independent = not still.query()
    torch.cuda.synchronize()
    return independent, cycles
