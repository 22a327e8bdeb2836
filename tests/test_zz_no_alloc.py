"""harvest_fetch_kv_static - the KV fetch for callers that cannot allocate - against harvest_fetch_kv, the entry point
it is a variant of: same requests, same bytes, same counts, same miss list; and against the oracle.  Two calls in a row
on one stream, the second with a smaller block table, because every call shares the GPU's one fixed scratch array and
finds the previous call's contents in it."""
import sys

import numpy as np
import pytest
import torch

import workloads as W
from workloads import scenarios as S
import parity as P

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _device_args(eh, run, n_seq_used=None, max_blocks_used=None):
    """The table arrays of a decode state on the device; optionally cut down to fewer sequences / columns."""
    table, nb = run.table_arrays()
    sdb = run.seq_dst_block.copy()
    if n_seq_used is not None:
        table, nb, sdb = table[:n_seq_used], nb[:n_seq_used], sdb[:n_seq_used]
    if max_blocks_used is not None:
        table = np.ascontiguousarray(table[:, :max_blocks_used])
        nb = np.minimum(nb, max_blocks_used).astype(np.int32)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(eh.dev)
    return table, nb, sdb, d(table), d(nb), d(sdb.view(np.int64))


def _compare_one(eh, eo, layer, args, cap, what, stream=None):
    table, nb, sdb, d_table, d_nb, d_sdb = args
    sp = eh.spec[S.KV]
    n_cells = table.size
    fill = 0x3C
    new = lambda: [torch.full((cap * sp.chunk_bytes,), fill, dtype=torch.uint8, device=eh.dev) for _ in range(2)]
    dst_a, dst_b = new(), new()
    info = torch.full((8,), -1, dtype=torch.int32, device=eh.dev)
    miss = torch.full((max(1, n_cells),), -1, dtype=torch.int32, device=eh.dev)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    eh.h.fetch_kv_static(layer, d_table, d_nb, dst_a[0], dst_a[1], d_sdb, cap, info, miss, stream=stream)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before, f"{what}: device memory in use changed across the call"
    # the entry point it is a variant of, on the same inputs
    eh.h.fetch_kv(layer, d_table, d_nb, dst_b[0], dst_b[1], d_sdb, cap)
    counts, miss_b, n_miss = eh.h.fetch_info(miss_cap=max(1, n_cells))
    for p in range(2):
        assert torch.equal(dst_a[p], dst_b[p]), f"{what}: plane {p} differs from harvest_fetch_kv"
    got = info.cpu().numpy()
    want = [counts["n_requests"], counts["n_local"], counts["n_cache"], counts["n_host"], counts["n_lost"],
            counts["n_invalid"], n_miss, 0]
    assert list(got) == want, f"{what}: info {list(got)} != {want}"
    m = miss.cpu().numpy()[:n_miss]
    assert np.array_equal(m, np.sort(m)), f"{what}: miss list not in request order"
    assert np.array_equal(m.astype(np.uint32), np.sort(miss_b)), f"{what}: miss lists differ"
    # and the oracle
    ko, vo, mo, co = eo.fetch_kv(layer, table, nb, sdb, cap)
    ko, vo = ko.copy(), vo.copy()
    # the oracle's destination starts zeroed, this one with a fill byte: compare where a request wrote
    ka, va = dst_a[0].cpu().numpy(), dst_a[1].cpu().numpy()
    written = np.zeros(cap, bool)
    for s in range(table.shape[0]):
        written[int(sdb[s]):int(sdb[s]) + int(nb[s])] = True
    wb = np.repeat(written, sp.chunk_bytes)
    assert np.array_equal(ka[wb], ko[wb]) and np.array_equal(va[wb], vo[wb]), f"{what}: differs from the oracle"
    assert (ka[~wb] == fill).all() and (va[~wb] == fill).all(), f"{what}: bytes outside the requests were written"
    assert co == counts and np.array_equal(mo, np.sort(miss_b))
    return counts


@pytest.mark.parametrize("general", [False, True], ids=["one-kernel", "general"])
def test_static_fetch_matches_fetch_kv_on_two_calls_in_a_row(general):
    say(f"fetch without allocation, general path {general}")
    # 3 sequences of 900-2600 blocks: more than 4096 cells, so the first call takes resolve + compaction + two gathers
    wl = W.kv_decode(seed=61, n_layers=2, n_seq=3, min_len=16000, max_len=42000, p_cache=0.65, n_steps=4)
    eo, eh = P.make_engines(wl, poison=True, hip_kwargs=dict(general_fetch=general))
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        for t in range(2):
            ro.append(t); rh.append(t)
        big = _device_args(eh, rh)
        assert big[0].size > 4096
        c = _compare_one(eh, eo, 1, big, rh.cap, "first call (large table)")
        assert c["n_cache"] > 1000 and c["n_host"] > 500 and c["n_local"] == 3
        # second call: a smaller input - fewer sequences, shorter rows (a ragged tail: 37 columns)
        small = _device_args(eh, rh, n_seq_used=2, max_blocks_used=37)
        c = _compare_one(eh, eo, 0, small, rh.cap, "second call (small table)")
        assert c["n_requests"] == 74
        # third: large again, other layer, after a revocation (the fixed scratch held the small call's lists)
        a, b = ro.revoke_quarter(0), rh.revoke_quarter(0)
        assert np.array_equal(a[0], b[0])
        _compare_one(eh, eo, 0, big, rh.cap, "third call (after a revocation)")
        # an empty table
        empty = _device_args(eh, rh, n_seq_used=0)
        info = torch.full((8,), -1, dtype=torch.int32, device=eh.dev)
        eh.h.fetch_kv_static(0, empty[3].reshape(0, 5), empty[4], torch.zeros(16, dtype=torch.uint8, device=eh.dev),
                             torch.zeros(16, dtype=torch.uint8, device=eh.dev), empty[5], 0, info, None)
        torch.cuda.synchronize()
        assert list(info.cpu().numpy()) == [0] * 8
    finally:
        eh.close(); eo.close()


def test_static_fetch_refuses_tables_beyond_its_fixed_scratch():
    from paper_2602_00328_amd import binding as B
    say("fetch without allocation: size limit")
    wl = W.kv_decode(seed=62, n_layers=1, n_seq=2, min_len=64, max_len=100, n_steps=1)
    eo, eh = P.make_engines(wl)
    try:
        S.KVRun(eo, wl); rh = S.KVRun(eh, wl)
        n_seq, max_blocks = 257, 256                         # 65 792 cells > 65 536
        d_table = torch.zeros((n_seq, max_blocks), dtype=torch.int32, device=eh.dev)
        d_nb = torch.zeros(n_seq, dtype=torch.int32, device=eh.dev)
        d_sdb = torch.zeros(n_seq, dtype=torch.int64, device=eh.dev)
        dst = torch.zeros(rh.cap * wl.shape.chunk_bytes, dtype=torch.uint8, device=eh.dev)
        with pytest.raises(B.HarvestError) as e:
            eh.h.fetch_kv_static(0, d_table, d_nb, dst, dst.clone(), d_sdb, rh.cap)
        assert e.value.code == B.E2BIG
        # exactly at the limit it is served
        d_table = torch.zeros((256, 256), dtype=torch.int32, device=eh.dev)
        eh.h.fetch_kv_static(0, d_table, d_nb[:256], dst, dst.clone(), d_sdb[:256], rh.cap)
        torch.cuda.synchronize()
    finally:
        eh.close(); eo.close()


def test_static_fetch_serves_four_streams_and_a_released_state_goes_to_the_next():
    from paper_2602_00328_amd import binding as B
    say("fetch without allocation: four streams per context, release")
    wl = W.kv_decode(seed=64, n_layers=1, n_seq=2, min_len=3000, max_len=6000, p_cache=0.6, n_steps=1)
    eo, eh = P.make_engines(wl, hip_kwargs=dict(general_fetch=True))
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        args = _device_args(eh, rh)
        streams = [torch.cuda.Stream(eh.dev) for _ in range(5)]
        for st in streams[:4]:
            with torch.cuda.stream(st):
                _compare_one(eh, eo, 0, args, rh.cap, "one of four streams", stream=st)
        table, nb, sdb, d_table, d_nb, d_sdb = args
        dst = [torch.zeros(rh.cap * eh.spec[S.KV].chunk_bytes, dtype=torch.uint8, device=eh.dev) for _ in range(2)]
        with pytest.raises(B.HarvestError) as e:
            eh.h.fetch_kv_static(0, d_table, d_nb, dst[0], dst[1], d_sdb, rh.cap, stream=streams[4])
        assert e.value.code == B.EBUSY
        eh.h.release_stream(streams[1])                    # its fixed state is free again ...
        with pytest.raises(B.HarvestError) as e:
            eh.h.release_stream(streams[1])
        assert e.value.code == B.ENOENT
        with torch.cuda.stream(streams[4]):                # ... and the fifth stream takes it
            _compare_one(eh, eo, 0, args, rh.cap, "fifth stream after a release", stream=streams[4])
        with torch.cuda.stream(streams[3]):                # the state that moved into the gap still serves its stream
            _compare_one(eh, eo, 0, args, rh.cap, "fourth stream after the release", stream=streams[3])
        with pytest.raises(B.HarvestError) as e:
            eh.h.fetch_kv_static(0, d_table, d_nb, dst[0], dst[1], d_sdb, rh.cap, stream=streams[1])
        assert e.value.code == B.EBUSY
    finally:
        eh.close(); eo.close()


def test_static_fetch_recorded_into_a_graph_with_no_earlier_call_on_the_stream():
    say("fetch without allocation: graph capture on a fresh stream")
    wl = W.kv_decode(seed=63, n_layers=2, n_seq=3, min_len=9000, max_len=30000, p_cache=0.6, n_steps=2)
    eo, eh = P.make_engines(wl, poison=True)
    try:
        ro, rh = S.KVRun(eo, wl), S.KVRun(eh, wl)
        args = _device_args(eh, rh)
        table, nb, sdb, d_table, d_nb, d_sdb = args
        sp = eh.spec[S.KV]
        dst = [torch.zeros(rh.cap * sp.chunk_bytes, dtype=torch.uint8, device=eh.dev) for _ in range(2)]
        info = torch.zeros(8, dtype=torch.int32, device=eh.dev)
        stream = torch.cuda.Stream(eh.dev)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            eh.h.fetch_kv_static(1, d_table, d_nb, dst[0], dst[1], d_sdb, rh.cap, info, None,
                                 stream=torch.cuda.current_stream())
        for rep in range(3):
            for t in dst:
                t.zero_()
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            ko, vo, mo, co = ro.fetch(1)
            assert np.array_equal(dst[0].cpu().numpy(), ko) and np.array_equal(dst[1].cpu().numpy(), vo), f"replay {rep}"
            assert list(info.cpu().numpy()[:6]) == [co["n_requests"], co["n_local"], co["n_cache"], co["n_host"],
                                                    co["n_lost"], co["n_invalid"]]
            if rep == 0:                       # residency changes between replays; the recorded fetch follows it
                a, b = ro.revoke_quarter(0), rh.revoke_quarter(0)
                assert np.array_equal(a[0], b[0])
            if rep == 1:
                assert np.array_equal(ro.replace_revoked(), rh.replace_revoked())
    finally:
        eh.close(); eo.close()
