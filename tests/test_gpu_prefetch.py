"""Double-buffered expert prefetch through the C ABI: while the compute stream consumes layer l's experts from one
staging buffer, the library's fetch stream fills the other with layer l+1's (Section 4.3: transfers for the next
micro-batch overlap the computation of the current one).  Every consumed buffer must hold exactly what the oracle's
fetch of that layer holds, with revocations (+ poisoning) and re-placements happening while fetches are in flight."""
import numpy as np
import pytest
import torch

import workloads as W
from workloads import scenarios as S
import parity as P

pytestmark = pytest.mark.gpu
IN_PLACE, STAGED = 1, 2


def test_double_buffered_prefetch_against_layer_by_layer_oracle_fetches():
    from paper_2602_00328_amd import binding as B
    print("prefetch ring", flush=True)
    L, E = 6, 16
    sh = W.ExpertShape(n_layers=L, n_experts=E, d_model=96, d_ff=100)
    ex = W.expert_offload(seed=31, shape=sh, n_tokens=64)
    eo, eh = P.make_engines(ex_wl=ex, poison=True)
    pf = None
    try:
        xo, xh = S.ExpertRun(eo, ex), S.ExpertRun(eh, ex)
        chunk = sh.chunk_bytes
        pf = B.Prefetcher(eh.h, n_staging_slots=E)
        with pytest.raises(B.HarvestError) as e:
            pf.acquire()
        assert e.value.code == B.EBUSY
        with pytest.raises(B.HarvestError) as e:
            pf.release()
        assert e.value.code == B.EINVAL
        compute = torch.cuda.Stream()
        local = eh.h.dev_plane(S.EXPERT, S.LOCAL, 0)
        n_steps = 4
        work = [(t, l) for t in range(n_steps) for l in range(L)]
        topk = {w: torch.from_numpy(ex.routing(*w)).to(eh.dev) for w in work}
        torch.cuda.synchronize()
        consumed = []                                   # (staging copy, pointer copy, base address of the buffer used)
        pf.issue(work[0][1], topk[work[0]])
        for i, w in enumerate(work):
            if i + 1 < len(work):
                pf.issue(work[i + 1][1], topk[work[i + 1]])       # the next layer's fetch runs beside this layer's use
            if i == 0:
                with pytest.raises(B.HarvestError) as e:          # two fetches issued, none released
                    pf.issue(0, topk[work[0]])
                assert e.value.code == B.EBUSY
            st, pt = pf.acquire(compute)
            with torch.cuda.stream(compute):                      # the consumer: reads every staged byte and pointer
                consumed.append((st.clone(), pt.clone(), st.data_ptr()))
            pf.release(compute)
            if i == 7:                                            # revoke with a fetch in flight, poison on
                a, b = xo.revoke_quarter(1), xh.revoke_quarter(1)
                assert np.array_equal(a[0], b[0]) and a[1] == b[1] and len(a[0]) > 0
            if i == 13:
                assert np.array_equal(xo.replace_revoked(), xh.replace_revoked())
        counts, miss, n_miss = pf.fetch_info(miss_cap=E)          # synchronises the fetch stream: the last layer's fetch
        with pytest.raises(B.HarvestError) as e:                  # the ring's stream is the ring's to release
            eh.h.release_stream(pf.stream)
        assert e.value.code == B.EINVAL
        torch.cuda.synchronize()
        # the oracle, layer by layer, for the residency at the end (bytes do not depend on residency; pointers of
        # staged experts depend only on the routed set)
        for i, w in enumerate(work):
            out_o, kind_o, where_o, miss_o, counts_o = xo.fetch(*w)
            st, pt, base = consumed[i]
            st, pt = st.cpu().numpy(), pt.cpu().numpy()
            for e in range(E):
                if kind_o[e] == STAGED:
                    r = int(where_o[e])
                    assert int(pt[e]) == base + r * chunk, (w, e)
                    assert np.array_equal(st[r * chunk:(r + 1) * chunk], out_o[e]), (w, e)
                elif kind_o[e] == IN_PLACE:
                    assert int(pt[e]) == local.data_ptr() + int(where_o[e]) * chunk, (w, e)
                else:
                    assert int(pt[e]) == 0, (w, e)
            if i == len(work) - 1:
                assert counts == counts_o and np.array_equal(np.sort(miss), miss_o)
        assert {c[2] for c in consumed} == {pf.staging[0].data_ptr(), pf.staging[1].data_ptr()}
        left_open = B.Prefetcher(eh.h, n_staging_slots=2)          # never closed: the context takes it down with it
        left_open.issue(0, topk[work[0]])
    finally:
        if pf is not None:
            pf.close()
        eh.close(); eo.close()
