"""Stored digests (tests/golden/fetch_digests.json, written by tests/golden/make_golden.py from the oracle alone): the
oracle must still produce them (CPU), and the HIP path must hit the same numbers (GPU)."""
import importlib.util
import json
import os

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
G = importlib.util.module_from_spec(spec)
spec.loader.exec_module(G)


def stored():
    with open(G.PATH) as f:
        return json.load(f)


def compare(got, want, path=""):
    assert type(got) is type(want), path
    if isinstance(want, dict):
        assert sorted(got) == sorted(want), path
        for k in want:
            compare(got[k], want[k], f"{path}/{k}")
    else:
        assert got == want, f"{path}: {got} != {want}"


def test_oracle_still_produces_the_stored_digests():
    from oracle.engine import OracleEngine
    compare(G.digests(lambda **kw: OracleEngine(**kw)), stored())


@pytest.mark.gpu
def test_hip_path_produces_the_stored_digests():
    from workloads.hip_engine import HipEngine
    print("golden digests", flush=True)
    compare(G.digests(lambda **kw: HipEngine(**kw)), stored())
