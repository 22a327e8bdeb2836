"""A KV fetch recorded into a HIP graph: the graph's launch parameters never change, the residency directory in device
memory does.  Every replay - with eager placements, revocations, evictions and synchronisations between them - must
deliver exactly what an eager fetch and the oracle deliver for the residency of that moment."""
import sys

import numpy as np
import pytest
import torch

import workloads as W
from workloads import scenarios as S
import parity as P

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("general,adjacent", [(True, False), (True, True), (False, False)],
                         ids=["general path", "general path, K|V adjacent in the cache tier", "one-kernel path"])
def test_captured_fetch_follows_residency_changes_across_replays(general, adjacent):
    """Once through resolve, compaction and the two gathers, once through the single kernel that serves small tables
    (this one has 1 125 cells)."""
    print("graph capture", flush=True)
    wl = W.kv_decode(seed=11, n_layers=2, n_seq=3, min_len=2000, max_len=6000, p_cache=0.6, n_steps=1)
    eo, eh = P.make_engines(wl, poison=True, cache_slack=64,
                            hip_kwargs=dict(general_fetch=general, cache_planes_adjacent=adjacent))
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        dev = eh.dev
        table, nb = rh.table_arrays()
        d_table = torch.from_numpy(table).to(dev)
        d_nb = torch.from_numpy(nb).to(dev)
        d_sdb = torch.from_numpy(rh.seq_dst_block.view(np.int64)).to(dev)
        chunk = wl.shape.chunk_bytes
        dst = [torch.zeros(rh.cap * chunk, dtype=torch.uint8, device=dev) for _ in range(2)]
        s = torch.cuda.Stream(dev)
        with torch.cuda.stream(s):                     # once outside capture: allocates this stream's scratch
            eh.h.fetch_kv(1, d_table, d_nb, dst[0], dst[1], d_sdb, rh.cap)
        s.synchronize()
        g = torch.cuda.CUDAGraph()
        some_host_block = next(b for b in range(wl.n_closed) if eh.lookup(S.KV, b)[0] == S.HOST)
        before = eh.lookup(S.KV, some_host_block)
        with torch.cuda.graph(g, stream=s):
            with pytest.raises(Exception) as e:            # directory edits cannot be recorded: refused, nothing changes
                eh.h.place(S.KV, [some_host_block])
            assert e.value.code == -1
            with pytest.raises(Exception) as e:            # and a revocation could not drain
                eh.h.revoke(S.KV, [int(next(iter(rh.live)))])
            assert e.value.code == -1
            eh.h.fetch_kv(1, d_table, d_nb, dst[0], dst[1], d_sdb, rh.cap)
        assert eh.lookup(S.KV, some_host_block) == before

        def replay_and_check(what):
            for t in dst:
                t.zero_()
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            with torch.cuda.stream(s):
                counts, miss, n_miss = eh.h.fetch_info(miss_cap=table.size)
            got = (dst[0].cpu().numpy(), dst[1].cpu().numpy(), np.sort(miss), counts)
            P.assert_kv_equal(ro.fetch(1), got, what)
            P.assert_kv_equal(rh.fetch(1), got, what + " (eager)")            # eager work between the replays
            return counts

        c0 = replay_and_check("replay 1")
        c1 = replay_and_check("replay 2 (unchanged)")
        assert c0 == c1
        ids_o, _ = ro.revoke_quarter(1)
        ids_h, _ = rh.revoke_quarter(1)
        assert np.array_equal(ids_o, ids_h) and len(ids_h) > 50
        c2 = replay_and_check("replay 3 (a quarter revoked, slots poisoned)")
        assert c2["n_host"] > c1["n_host"] and c2["n_cache"] < c1["n_cache"]
        host_only = [b for b in range(wl.n_closed) if eh.lookup(S.KV, b)[0] == S.HOST][:40]
        assert np.array_equal(eo.place(S.KV, host_only), eh.place(S.KV, host_only))
        c3 = replay_and_check("replay 4 (other blocks placed into the freed slots)")
        assert c3["n_cache"] == c2["n_cache"] + sum(1 for b in host_only if b in set(table[:, :].reshape(-1).tolist()))
        # new bytes through the write-back path, then replay again
        ev = np.array(sorted(set(int(b) for b in table[0, :8])), np.uint32)
        gk = W.rng(11, 7).integers(0, 256, size=ev.size * chunk, dtype=np.uint8)
        gv = W.rng(11, 8).integers(0, 256, size=ev.size * chunk, dtype=np.uint8)
        for e in (eo, eh):
            e.evict(S.KV, 1, ev, gk, gv, np.arange(ev.size), ev.size)
        replay_and_check("replay 5 (after a write-back)")
        assert np.array_equal(ro.replace_revoked(), rh.replace_revoked())
        replay_and_check("replay 6 (revoked blocks placed again)")
    finally:
        eh.close(); eo.close()


def test_captured_expert_fetch_follows_residency_changes_across_replays():
    """The same for the expert fetch: routing ids, staging buffer and pointer table are fixed in the graph; which experts
    come from the cache tier and which from the host is read from the directory at every replay."""
    print("graph capture, experts", flush=True)
    ex = W.expert_offload(seed=12, shape=W.ExpertShape(n_layers=3, n_experts=16, d_model=64, d_ff=100), n_tokens=64)
    eo, eh = P.make_engines(None, ex, poison=True)
    try:
        xo, xh = S.ExpertRun(eo, ex), S.ExpertRun(eh, ex)
        dev, sp, layer, n_staging = eh.dev, eh.spec[S.EXPERT], 1, 16
        topk = ex.routing(0, layer)
        d_topk = torch.from_numpy(np.ascontiguousarray(topk, dtype=np.int32)).to(dev)
        staging = torch.zeros(n_staging * sp.chunk_bytes, dtype=torch.uint8, device=dev)
        ptrs = torch.zeros(sp.n_experts, dtype=torch.int64, device=dev)
        s = torch.cuda.Stream(dev)
        with torch.cuda.stream(s):                     # once outside capture: allocates this stream's scratch
            eh.h.fetch_experts(layer, d_topk, staging, n_staging, ptrs)
        s.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            eh.h.fetch_experts(layer, d_topk, staging, n_staging, ptrs)

        def replay_and_check(what):
            staging.fill_(0x5A)
            ptrs.zero_()
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            with torch.cuda.stream(s):
                got = eh.fetch_end(("experts", staging, n_staging, ptrs, d_topk))
            P.assert_experts_equal(eo.fetch_experts(layer, topk, n_staging), got, what)
            P.assert_experts_equal(eh.fetch_experts(layer, topk, n_staging), got, what + " (eager)")
            return got[4]

        c1 = replay_and_check("replay 1")
        in_cache = [i for i in range(layer * 16, layer * 16 + 16) if eh.lookup(S.EXPERT, i)[0] == S.CACHE]
        assert len(in_cache) >= 2
        gone = in_cache[:len(in_cache) // 2 + 1]
        assert eo.revoke(S.EXPERT, gone) == eh.revoke(S.EXPERT, gone) == gone
        c2 = replay_and_check("replay 2 (cached experts revoked, slots poisoned)")
        assert c2["n_host"] > c1["n_host"] or not set(gone) & {layer * 16 + int(e) for e in np.unique(topk)}
        on_host = [i for i in range(layer * 16, layer * 16 + 16) if eh.lookup(S.EXPERT, i)[0] == S.HOST]
        assert np.array_equal(eo.place(S.EXPERT, on_host), eh.place(S.EXPERT, on_host))
        replay_and_check("replay 3 (every host expert of the layer placed, as far as slots last)")
        replay_and_check("replay 4 (unchanged)")
    finally:
        eh.close(); eo.close()
