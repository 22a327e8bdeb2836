"""The harness drivers run against the oracle alone (no GPU): with the self-describing tag payload every fetched
chunk names the block it must be, so these runs check drivers and oracle together against the workload definition."""
import numpy as np
import pytest

import workloads as W
from workloads import scenarios as S
from oracle.engine import OracleEngine


def check_kv_tags(wl, run, out, layer, skip_tails=True):
    k, v, miss, counts = out
    chunk = wl.shape.chunk_bytes
    for s, t in enumerate(run.tables):
        blocks = t[:-1] if (wl.has_tails and skip_tails) else t
        for j, b in enumerate(blocks):
            d = int(run.seq_dst_block[s]) + j
            assert W.check_tag(k[d * chunk:(d + 1) * chunk], wl.seed, W.CLS_KV, 0, layer, b), (s, j, b)
            assert W.check_tag(v[d * chunk:(d + 1) * chunk], wl.seed, W.CLS_KV, 1, layer, b), (s, j, b)


def test_tiny_config_on_the_oracle():
    wl = W.kv_tiny(0, fill_mode=W.FILL_TAG)
    e = OracleEngine(kv=S.kv_spec(wl))
    run = S.KVRun(e, wl)
    assert (run.place_status == 0).all() and len(run.live) == 614
    out = run.fetch(0)
    check_kv_tags(wl, run, out, 0)
    assert out[3]["n_requests"] == 256 and out[3]["n_cache"] + out[3]["n_host"] == 256
    slots = sorted(e.lookup(S.KV, b)[1] for b in run.live)
    assert slots == list(range(614))
    assert any(e.lookup(S.KV, b)[1] != b for b in run.live)
    e.close()


def test_decode_steps_on_the_oracle():
    wl = W.kv_decode(seed=2, n_layers=2, n_seq=3, min_len=100, max_len=400, n_steps=40, fill_mode=W.FILL_TAG)
    e = OracleEngine(kv=S.kv_spec(wl))
    run = S.KVRun(e, wl)
    n0 = [len(t) for t in run.tables]
    first_tails = [t[-1] for t in run.tables]
    for t in range(40):
        layer = t % 2
        out = run.fetch(layer)
        # blocks closed at step 0 still carry their tag; blocks closed later carry appended rows
        k = out[0]
        chunk = wl.shape.chunk_bytes
        for s in range(3):
            for j in range(n0[s] - 1):
                d = int(run.seq_dst_block[s]) + j
                assert W.check_tag(k[d * chunk:(d + 1) * chunk], wl.seed, W.CLS_KV, 0, layer, run.tables[s][j])
        assert out[3]["n_local"] == 3 and out[3]["n_invalid"] == 0
        run.append(t)
    assert [len(t) for t in run.tables] == [n + len(f) for n, f in zip(n0, wl.future_blocks)]
    # a tail that was closed holds, row by row, what was there at step 0 and then the appended rows
    s = 0
    tail = first_tails[s]
    assert e.lookup(S.KV, tail)[0] in (S.HOST, S.CACHE)
    table = np.array([[tail]], np.int32)
    k, v, _, _ = e.fetch_kv(1, table, np.array([1], np.int32), np.array([0], np.uint64), 1)
    rb, bt = wl.shape.row_bytes, wl.shape.block_tokens
    start = int(wl.seq_lens[s]) % bt
    base = W.chunk(wl.seed, W.CLS_KV, 0, 1, tail, wl.shape.chunk_bytes, W.FILL_TAG)
    assert np.array_equal(k[:start * rb], base[:start * rb])
    for r in range(start, bt):
        rows = W.append_rows(wl, r - start, s)
        assert np.array_equal(k[r * rb:(r + 1) * rb], rows[0, 1])
        assert np.array_equal(v[r * rb:(r + 1) * rb], rows[1, 1])
    e.close()


def test_expert_configs_on_the_oracle():
    sh = W.ExpertShape(n_layers=3, n_experts=16, d_model=16, d_ff=20)
    ex = W.expert_offload(seed=1, shape=sh, n_tokens=64, fill_mode=W.FILL_TAG)
    e = OracleEngine(expert=S.expert_spec(ex))
    run = S.ExpertRun(e, ex)
    for t in range(3):
        for layer in range(3):
            out, kind, where, miss, counts = run.fetch(t, layer)
            U = sorted(set(int(x) for x in ex.routing(t, layer).reshape(-1)))
            assert [i for i in range(16) if out[i] is not None] == U
            for i in U:
                assert W.check_tag(out[i], ex.seed, W.CLS_EXPERT, 0, 0, layer * 16 + i)
            assert counts["n_local"] == sum(1 for i in U if ex.tier0[layer, i] == 2)
            assert counts["n_cache"] == sum(1 for i in U if ex.tier0[layer, i] == 1)
    e.close()


@pytest.mark.parametrize("from_staging", [False, True])
def test_lru_policy_keeps_capacity_and_hits_after_warm_up(from_staging):
    sh = W.ExpertShape(n_layers=2, n_experts=60, d_model=16, d_ff=12)
    ex = W.expert_lru(seed=1, shape=sh, n_tokens=32, top_k=4, fill_mode=W.FILL_TAG)
    e = OracleEngine(expert=S.expert_spec(ex), poison=True)
    run = S.ExpertRun(e, ex)
    hits = []
    for t in range(5):
        for layer in range(2):
            out, kind, where, miss, counts = run.fetch(t, layer)
            for i in range(60):
                if out[i] is not None:
                    assert W.check_tag(out[i], ex.seed, W.CLS_EXPERT, 0, 0, layer * 60 + i)
            hits.append(counts["n_cache"])
            run.lru_update(t, layer, from_staging=from_staging)
            in_cache = [i for i in range(60) if e.lookup(S.EXPERT, layer * 60 + i)[0] == S.CACHE]
            assert len(in_cache) == min(24, len(run.lru[layer].members())) and set(in_cache) == run.lru[layer].members()
    assert hits[0] == 0 and hits[1] == 0 and sum(hits[2:]) > 0
    e.close()


def test_placing_from_the_staging_buffer_leaves_the_state_placing_from_the_host_leaves():
    """An expert the fetch has just staged holds its host bytes, so filling the cache tier from the staging buffer must
    end in the same directory and the same cache-tier bytes as filling it over PCIe."""
    sh = W.ExpertShape(n_layers=2, n_experts=60, d_model=16, d_ff=12)
    ex = W.expert_lru(seed=2, shape=sh, n_tokens=32, top_k=4)
    engines = [OracleEngine(expert=S.expert_spec(ex), poison=True) for _ in range(2)]
    runs = [S.ExpertRun(e, ex, n_staging=40) for e in engines]                 # 40 slots: some steps overflow the staging buffer
    for t in range(4):
        for layer in range(2):
            outs = [r.fetch(t, layer) for r in runs]
            ranks = runs[1].staged_ranks(t, layer)                             # what the harness works out on the host ...
            kind, where = outs[1][1], outs[1][2]                               # ... is what the fetch did
            assert ranks == {e: int(where[e]) for e in range(60) if kind[e] == 2}
            assert all((a is None) == (b is None) and (a is None or np.array_equal(a, b)) for a, b in zip(*[o[0] for o in outs]))
            ups = [r.lru_update(t, layer, from_staging=k == 1) for k, r in enumerate(runs)]
            assert ups[0][0] == ups[1][0] and ups[0][2] == ups[1][2] and np.array_equal(ups[0][3], ups[1][3])
    a, b = engines
    assert [a.lookup(S.EXPERT, i) for i in range(ex.n_objects)] == [b.lookup(S.EXPERT, i) for i in range(ex.n_objects)]
    assert np.array_equal(a.tier_plane(S.EXPERT, S.CACHE), b.tier_plane(S.EXPERT, S.CACHE))
    for e in engines:
        e.close()


def test_revocation_schedule_on_the_oracle():
    wl = W.kv_decode(seed=3, n_layers=1, n_seq=2, min_len=300, max_len=600, n_steps=30, fill_mode=W.FILL_TAG)
    e = OracleEngine(kv=S.kv_spec(wl), poison=True)
    run = S.KVRun(e, wl)
    for t in range(30):
        before = len(run.live)
        if t % 10 == 0 and t > 0:
            ids, called = run.revoke_quarter(t)
            assert len(ids) == round(0.25 * before) and called == [int(i) for i in ids]
            assert all(e.lookup(S.KV, i)[0] == S.HOST for i in ids)
        if t % 10 == 5:
            st = run.replace_revoked()
            assert (st == 0).all()
        out = run.step(t)
        check_kv_tags(wl, run, (out[0], out[1], None, None), 0) if t == 0 else None
    e.close()


def test_both_classes_in_one_shared_cache_pool_on_the_oracle():
    """KV blocks and experts compete for one tight segment pool: some placements fail, revocations fragment it,
    and every fetched chunk still names its block (Section 3.1: what the cache tier holds changes no result)."""
    wl = W.kv_decode(seed=6, n_layers=2, n_seq=3, min_len=200, max_len=500, n_steps=40, fill_mode=W.FILL_TAG)
    ex = W.expert_offload(seed=6, shape=W.ExpertShape(n_layers=2, n_experts=8, d_model=32, d_ff=50), n_tokens=8,
                          fill_mode=W.FILL_TAG)
    kv_bytes = 2 * 2 * wl.shape.chunk_bytes
    demand = int(wl.resident.sum()) * kv_bytes + int((ex.tier0 == 1).sum()) * ex.shape.chunk_bytes
    G = 1024
    pool_bytes = (int(0.7 * demand) // G) * G
    e = OracleEngine(kv=S.kv_spec(wl, shared=True), expert=S.expert_spec(ex, shared=True), poison=True,
                     shared_cache_bytes=pool_bytes, shared_granule=G)
    run, xr = S.KVRun(e, wl), S.ExpertRun(e, ex)
    assert (run.place_status == 0).sum() > 10
    assert (np.concatenate([run.place_status, xr.place_status]) == -2).any()        # the pool is too small for all
    for t in range(40):
        layer = t % 2
        check_kv_tags(wl, run, run.fetch(layer), layer)
        st, kind, where, miss, counts = xr.fetch(t, layer)
        assert counts["n_invalid"] == 0 and counts["n_lost"] == 0
        if t % 10 == 0 and t:
            run.revoke_quarter(t); xr.revoke_quarter(t)
        if t % 10 == 5:
            xr.replace_revoked(); run.replace_revoked()
    runs = e.shared_free_runs()
    used = pool_bytes // G - sum(l for _, l in runs)
    kv_g, ex_g = -(-kv_bytes // G), -(-ex.shape.chunk_bytes // G)
    assert used == len(run.live) * kv_g + len(xr.live) * ex_g
    e.close()
