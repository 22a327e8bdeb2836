"""The seeded input generators: determinism, the structure the configs ask for, regenerable chunks."""
import numpy as np
import pytest

import workloads as W


def test_chunks_regenerate_and_differ_by_every_key_field():
    a = W.chunk(0, W.CLS_KV, 0, 3, 17, 4096)
    assert np.array_equal(a, W.chunk(0, W.CLS_KV, 0, 3, 17, 4096))
    for other in (W.chunk(1, W.CLS_KV, 0, 3, 17, 4096), W.chunk(0, W.CLS_EXPERT, 0, 3, 17, 4096),
                  W.chunk(0, W.CLS_KV, 1, 3, 17, 4096), W.chunk(0, W.CLS_KV, 0, 4, 17, 4096),
                  W.chunk(0, W.CLS_KV, 0, 3, 18, 4096)):
        assert not np.array_equal(a, other)
    pool = np.zeros((5, 7, 4096), np.uint8)
    so = np.array([9, W.NO_OBJECT, 17, 3, 4, 5, 6], np.uint32)
    W.fill_array(pool, so, 0, W.CLS_KV, 0)
    assert np.array_equal(pool[3, 2], a) and (pool[:, 1] == 0).all()


def test_normal_fill_is_bf16_standard_normal():
    x = W.chunk(0, W.CLS_KV, 0, 0, 0, 1 << 20).view(np.uint16)
    f = (x.astype(np.uint32) << 16).view(np.float32)
    assert abs(f.mean()) < 0.01 and abs(f.std() - 1.0) < 0.01
    assert abs(np.mean(np.abs(f) < 1.0) - 0.6827) < 0.005
    y = W.chunk(0, W.CLS_EXPERT, 0, 0, 0, 1 << 20, sigma=0.02).view(np.uint16)
    g = (y.astype(np.uint32) << 16).view(np.float32)
    assert abs(g.std() - 0.02) < 0.0003


def test_tag_words_describe_themselves():
    t = W.chunk(5, W.CLS_EXPERT, 0, 2, 77, 160, W.FILL_TAG).view(np.uint32).reshape(-1, 4)
    assert (t[:, 0] == (1 << 28 | 2)).all() and (t[:, 1] == 77).all() and list(t[:, 2]) == list(range(10))
    assert W.check_tag(t.view(np.uint8).reshape(-1), 5, W.CLS_EXPERT, 0, 2, 77)
    assert not W.check_tag(t.view(np.uint8).reshape(-1), 5, W.CLS_EXPERT, 0, 2, 78)


def test_kv_tiny_matches_the_config():
    w = W.kv_tiny(0)
    assert w.n_seq == 16 and all(len(t) == 16 for t in w.tables) and w.shape.chunk_bytes == 32768
    allb = np.concatenate(w.tables)
    assert len(set(allb)) == 256 and allb.max() < 1024
    assert w.resident.sum() == 614 and w.place_order.size == 614 and set(w.place_order) == set(np.nonzero(w.resident)[0])
    assert not np.array_equal(w.place_order, np.sort(w.place_order))          # slots become a permutation, not identity
    w2 = W.kv_tiny(0)
    assert all(np.array_equal(a, b) for a, b in zip(w.tables, w2.tables)) and np.array_equal(w.resident, w2.resident)


def test_kv_decode_matches_the_config():
    w = W.kv_decode(0)
    assert w.n_seq == 4 and ((w.seq_lens >= 32768) & (w.seq_lens <= 131072)).all()
    nb = w.n_blocks()
    assert all(nb[s] == w.seq_lens[s] // 16 + 1 for s in range(4))
    ids = np.concatenate(w.tables + w.future_blocks)
    assert sorted(ids) == list(range(w.n_objects))
    C = w.n_closed
    assert [int(t[-1]) for t in w.tables] == [C + s for s in range(4)]
    assert all((w.seq_lens[s] + 200) // 16 + 1 == nb[s] + len(w.future_blocks[s]) for s in range(4))
    opened = sorted((int(b), s) for s in range(4) for b in w.future_blocks[s])
    assert [b for b, _ in opened] == list(range(C + 4, w.n_objects))      # numbered in opening order
    assert abs(w.resident.mean() - 0.7) < 0.02
    assert set(w.place_order) == set(np.nonzero(w.resident[:C])[0])
    assert sorted(w.host_slot) == list(range(w.n_objects)) and not np.array_equal(w.host_slot, np.arange(w.n_objects))


def test_zipf_routing_draws_distinct_experts_with_the_stated_popularity():
    w = W.expert_offload(0)
    assert (w.tier0 == 2).sum(axis=1).tolist() == [2] * 32
    frac = (w.tier0 == 1).sum() / (32 * 14)
    assert abs(frac - 0.5) < 0.08
    counts = np.zeros(16)
    unions = []
    for step in range(40):
        for layer in (0, 5):
            r = w.routing(step, layer)
            assert r.shape == (64, 2) and (r[:, 0] != r[:, 1]).all() and r.min() >= 0 and r.max() < 16
            unions.append(len(set(r.reshape(-1))))
            inv = np.argsort(w.rank_to_expert[layer])          # expert -> rank
            np.add.at(counts, inv[r[:, 0]], 1)
    p = np.arange(1, 17) ** -1.1
    p /= p.sum()
    assert np.abs(counts / counts.sum() - p).max() < 0.02       # first draw follows rank^-1.1
    assert 14.5 < np.mean(unions) <= 16
    assert np.array_equal(w.routing(3, 1), W.expert_offload(0).routing(3, 1))


def test_many_small_experts_config():
    w = W.expert_lru(0)
    assert w.shape.chunk_bytes == 3 * 2048 * 1408 * 2 and w.lru_capacity == 24 and w.n_objects == 1440
    r = w.routing(0, 0)
    assert r.shape == (256, 4) and all(len(set(row)) == 4 for row in r)


def test_lru_matches_a_list_based_brute_force():
    g = W.rng(0, 77)
    trace = g.integers(0, 5, size=200)
    lru = W.LRU(3)
    lst = []                                                    # most recent last
    for x in trace:
        lru.touch(int(x))
        if x in lst:
            lst.remove(x)
        lst.append(x)
        lst = lst[-3:]
        assert lru.members() == set(int(v) for v in lst)


def test_revoke_draw_is_a_quarter_and_order_independent():
    a = W.revoke_draw(0, 10, 0, {5, 1, 9, 3, 7, 11, 13, 15})
    b = W.revoke_draw(0, 10, 0, [15, 13, 11, 9, 7, 5, 3, 1])
    assert a.size == 2 and np.array_equal(a, b)


# ---- the checksum long runs compare outputs with ---------------------------------------------------------------

def _digest_by_definition(buf):
    """The definition in digest.c, in Python integers."""
    from workloads import digest as D
    x = [int(v) for v in buf.view(np.uint64)]
    w = [int(v) for v in D.weights()]
    mask = (1 << 64) - 1
    total = 0
    for p in range((len(x) + D.M - 1) // D.M):
        s = sum(x[p * D.M + j] * w[j] for j in range(min(D.M, len(x) - p * D.M))) & mask
        total = (total + int(D.piece_factors(p + 1)[p]) * s) & mask
    return total


@pytest.mark.parametrize("n_bytes", [8, 4096, 8 * 65536, 8 * 65536 + 8, 8 * (2 * 65536 + 1234)])
def test_digest_on_host_and_as_tensor_operations_follow_the_definition(n_bytes):
    import torch
    from workloads.digest import digest
    buf = W.rng(9, n_bytes).integers(0, 256, size=n_bytes, dtype=np.uint8)
    want = _digest_by_definition(buf)
    assert digest(buf) == want
    assert digest(torch.from_numpy(buf)) == want


def test_digest_notices_single_bytes_and_moved_blocks():
    from workloads.digest import digest
    buf = W.rng(10).integers(0, 256, size=64 * 32768, dtype=np.uint8)
    d0 = digest(buf)
    one = buf.copy(); one[1234567] ^= 1
    assert digest(one) != d0
    swapped = buf.copy().reshape(64, 32768)
    swapped[[3, 41]] = swapped[[41, 3]]                      # two blocks delivered to each other's place
    assert digest(swapped.reshape(-1)) != d0
    shifted = np.roll(buf, 16)
    assert digest(shifted) != d0
    assert digest(buf.copy()) == d0
