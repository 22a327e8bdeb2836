"""Writes tests/golden/fetch_digests.json: SHA-256 digests of what a few seeded scenarios deliver, computed with the
CPU oracle only.  The paper prints no worked example of the fetch (no input / output pair to store), so these are
regression values of the pinned oracle on the seeded generators, not values of the paper: they hold the oracle, the
generators and the harness drivers still, and give the HIP path fixed numbers to hit.

    python tests/golden/make_golden.py          # rewrites the file; run it only when a change to the oracle's
                                                 # arithmetic or to a generator is intended and justified

`digests(make_engine)` is the scenario script; the tests call it with the oracle (CPU) and with the HIP engine (GPU).
"""
import hashlib
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workloads as W                      # noqa: E402
from workloads import scenarios as S       # noqa: E402

PATH = os.path.join(HERE, "fetch_digests.json")


def sha(*arrays):
    h = hashlib.sha256()
    for a in arrays:
        if a is None:
            h.update(b"\x00none")
        else:
            a = np.ascontiguousarray(a)
            h.update(str(a.dtype).encode() + str(a.shape).encode())
            h.update(a.tobytes())
    return h.hexdigest()


def kv_digest(out):
    k, v, miss, counts = out
    return {"k": sha(k), "v": sha(v), "miss": sha(np.sort(miss).astype(np.uint32)), "counts": counts}


def expert_digest(out):
    blobs, kind, where, miss, counts = out
    present = np.array([b is not None for b in blobs])
    kind = np.asarray(kind, np.int32)
    served = (kind == 1) | (kind == 2)                  # used in place / staged; everything else has no pointer
    return {"bytes": sha(*[b for b in blobs if b is not None]), "present": sha(present),
            "kind": sha(np.where(served, kind, 0)), "where": sha(np.where(served, np.asarray(where, np.int64), -1)),
            "miss": sha(np.sort(miss).astype(np.uint32)), "counts": counts}


def directory_digest(e, cls, n):
    return sha(np.array([e.lookup(cls, i) for i in range(n)], np.int64))


def digests(make_engine):
    """make_engine(kv=..., expert=..., poison=..., shared_cache_bytes=..., shared_granule=...) -> engine."""
    out = {}
    # 1. the tiny KV configuration: fetch, write the fetched bytes back, fetch again
    wl = W.kv_tiny(0)
    e = make_engine(kv=S.kv_spec(wl))
    run = S.KVRun(e, wl)
    first = run.fetch(0)
    out["tiny_kv"] = {"fetch": kv_digest(first), "directory": directory_digest(e, S.KV, wl.n_closed)}
    e.close()
    # 2. decode steps with appends, tail write-backs and placements
    wl = W.kv_decode(seed=2, n_layers=3, n_seq=4, min_len=500, max_len=2000, n_steps=40)
    e = make_engine(kv=S.kv_spec(wl))
    run = S.KVRun(e, wl)
    steps = {}
    for t in range(40):
        o = run.step(t)
        if t in (0, 13, 39):
            steps[str(t)] = kv_digest(o)
    out["decode_small"] = {"steps": steps, "directory": directory_digest(e, S.KV, wl.n_objects)}
    e.close()
    # 3. experts with revocation and re-placement, poison on
    ex = W.expert_offload(seed=3, shape=W.ExpertShape(n_layers=4, n_experts=16, d_model=64, d_ff=100), n_tokens=32)
    e = make_engine(expert=S.expert_spec(ex), poison=True)
    xr = S.ExpertRun(e, ex)
    steps = {}
    for t in range(6):
        for layer in range(4):
            o = xr.fetch(t, layer)
            if (t, layer) in ((0, 0), (2, 3), (5, 1)):
                steps[f"{t}.{layer}"] = expert_digest(o)
        if t == 1:
            xr.revoke_quarter(t)
        if t == 3:
            xr.replace_revoked()
    out["experts_small"] = {"steps": steps, "directory": directory_digest(e, S.EXPERT, ex.n_objects)}
    e.close()
    # 4. both classes in one tight shared cache pool (best-fit segments)
    wl = W.kv_decode(seed=6, n_layers=2, n_seq=3, min_len=200, max_len=500, n_steps=12)
    ex = W.expert_offload(seed=6, shape=W.ExpertShape(n_layers=2, n_experts=8, d_model=32, d_ff=50), n_tokens=8)
    demand = int(wl.resident.sum()) * 4 * wl.shape.chunk_bytes + int((ex.tier0 == 1).sum()) * ex.shape.chunk_bytes
    e = make_engine(kv=S.kv_spec(wl, shared=True), expert=S.expert_spec(ex, shared=True), poison=True,
                    shared_cache_bytes=int(0.7 * demand) // 1024 * 1024, shared_granule=1024)
    xr, run = S.ExpertRun(e, ex), S.KVRun(e, wl)
    steps = {}
    for t in range(12):
        layer = t % 2
        a, b = run.fetch(layer), xr.fetch(t, layer)
        if t in (0, 7, 11):
            steps[str(t)] = {"kv": kv_digest(a), "experts": expert_digest(b)}
        if t == 4:
            run.revoke_quarter(t); xr.revoke_quarter(t)
        if t == 8:
            xr.replace_revoked(); run.replace_revoked()
        run.append(t)
    out["shared_pool"] = {"steps": steps, "pool": sha(e.shared_plane()),
                          "kv_directory": directory_digest(e, S.KV, wl.n_objects),
                          "expert_directory": directory_digest(e, S.EXPERT, ex.n_objects)}
    e.close()
    # 5. head-major working layout, fp8-sized elements
    shape = W.KVShape(n_layers=2, block_tokens=16, n_kv_heads=4, head_dim=64, elt_bytes=1)
    wl = W.kv_decode(seed=12, n_seq=3, min_len=300, max_len=900, n_steps=1, shape=shape)
    e = make_engine(kv=S.kv_spec(wl))
    run = S.KVRun(e, wl)
    table, nb = run.table_arrays()
    caps = np.array([len(t) + len(f) for t, f in zip(wl.tables, wl.future_blocks)], np.uint32)
    o = e.fetch_kv_head_major(1, table, nb, run.seq_dst_block, caps, run.cap, 4, 16, dst_fill=0x5A)
    out["head_major"] = kv_digest(o)
    e.close()
    return out


def main():
    from oracle.engine import OracleEngine
    d = digests(lambda **kw: OracleEngine(**kw))
    with open(PATH, "w") as f:
        json.dump(d, f, indent=1, sort_keys=True)
        f.write("\n")
    print(f"wrote {PATH}")


if __name__ == "__main__":
    main()
