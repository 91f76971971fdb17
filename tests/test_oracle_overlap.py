"""Pins for the oracle's cross-layer overlap (paper App. A): independent set arithmetic."""
import numpy as np
import pytest


def _rows(rng, nq, k, Lk, fill):
    idx = np.full((nq, k), -1, dtype=np.int32)
    for t in range(nq):
        n = int(fill[t])
        idx[t, :n] = np.sort(rng.choice(Lk, size=n, replace=False))
    return idx


def test_overlap_matches_python_sets(oracle):
    rng = np.random.default_rng(11)
    nq, k, Lk, n = 37, 24, 90, 5
    fill = rng.integers(0, k + 1, size=nq)
    layers = [_rows(rng, nq, k, Lk, fill if l != 3 else rng.integers(0, k + 1, size=nq)) for l in range(n)]
    ov, inter, sizes = oracle.topk_overlap(layers, Lk)
    for i in range(n):
        assert sizes[i] == sum(len(set(r[r >= 0])) for r in layers[i])
        for j in range(n):
            want = sum(len(set(a[a >= 0]) & set(b[b >= 0])) for a, b in zip(layers[i], layers[j]))
            assert inter[i, j] == want
            if sizes[i]:
                assert ov[i, j] == pytest.approx(want / float(sizes[i]), rel=0, abs=1e-15)


def test_overlap_closed_forms(oracle):
    nq, k, Lk = 6, 16, 200
    base = np.tile(np.arange(k, dtype=np.int32), (nq, 1))
    shifted = [base + s for s in (0, 1, 5, 16, 40)]           # windows {s..s+k-1}: overlap with window 0 is max(k-s,0)
    ov, inter, sizes = oracle.topk_overlap(shifted, Lk)
    assert np.all(sizes == nq * k)
    for a, sa in enumerate((0, 1, 5, 16, 40)):
        for b, sb in enumerate((0, 1, 5, 16, 40)):
            assert inter[a, b] == nq * max(k - abs(sa - sb), 0)
    assert np.allclose(np.diag(ov), 1.0)
    assert np.array_equal(inter, inter.T)                       # equal set sizes => symmetric


def test_overlap_ignores_padding_order_and_out_of_range(oracle):
    rng = np.random.default_rng(3)
    Lk, k = 50, 8
    a = np.array([[4, 9, 11, -1, -1, 30, 49, -1]], dtype=np.int32)
    b = np.array([[49, 77, 4, -1, 12, 11, -5, 1000]], dtype=np.int32)     # 77 and 1000 are >= Lk: not members
    ov, inter, sizes = oracle.topk_overlap([a, b, a[:, ::-1].copy()], Lk)
    assert list(sizes) == [5, 4, 5]
    assert inter[0, 1] == 3 and inter[1, 0] == 3               # {4, 11, 49}
    assert inter[0, 2] == 5 and ov[0, 2] == 1.0                # order inside a row is irrelevant
    assert ov[1, 0] == 0.75


def test_overlap_of_shared_layers_is_one(oracle):
    """A Shared layer inherits the index tensor of its Full layer: overlap 1 inside a sharing block."""
    rng = np.random.default_rng(5)
    nq, k, Lk = 9, 12, 64
    f0 = _rows(rng, nq, k, Lk, np.full(nq, k))
    f1 = _rows(rng, nq, k, Lk, np.full(nq, k))
    mask = oracle.pattern_from_string("FSSFS")
    used = [f0, f0, f0, f1, f1]
    ov, _, _ = oracle.topk_overlap(used, Lk)
    for i in range(5):
        for j in range(5):
            same = oracle.source_layer(mask, i) == oracle.source_layer(mask, j)
            assert (ov[i, j] == 1.0) == same or (not same and ov[i, j] < 1.0)
