"""Pins for the oracle's top-k (O3): library sorts, argmax, closed-form rows, invariants."""
import numpy as np
import torch

import synth


def _bits(x):
    return synth.bits(torch.as_tensor(x, dtype=torch.float32).to(torch.bfloat16))


def test_topk_row_vs_lexsort(oracle):
    rng = np.random.default_rng(2)
    for n, k in [(50, 7), (50, 50), (50, 64), (1, 1), (300, 32)]:
        # few distinct values => many ties, including at the k-th boundary
        sc = rng.integers(0, 6, size=n).astype(np.float64) - 2.0
        r = oracle.topk_row(sc, n, k)
        order = np.lexsort((np.arange(n), -sc))          # score desc, then position asc
        m = min(n, k)
        assert np.array_equal(r["idx"][:m], order[:m])
        assert np.all(r["idx"][m:] == -1)
        assert np.array_equal(r["sel"][:m], sc[order[:m]])
        assert r["kth"] == sc[order[m - 1]]
        assert r["next"] == (sc[order[m]] if n > m else -np.inf)
        assert np.isclose(r["mean_abs"], np.abs(sc).mean())


def test_topk_k1_is_first_argmax(oracle):
    sc = np.array([0.5, 3.0, -1.0, 3.0, 2.0])
    r = oracle.topk_row(sc, 5, 1)
    assert r["idx"][0] == int(np.argmax(sc)) == 1      # numpy argmax returns the first maximum


def test_topk_all_equal_row_selects_lowest_positions(oracle):
    r = oracle.topk_row(np.zeros(100), 100, 16)
    assert np.array_equal(r["idx"], np.arange(16))
    assert r["kth"] == 0.0 and r["next"] == 0.0


def test_topk_monotone_rows(oracle):
    inc = np.arange(40, dtype=np.float64)
    assert np.array_equal(oracle.topk_row(inc, 40, 5)["idx"], [39, 38, 37, 36, 35])
    assert np.array_equal(oracle.topk_row(-inc, 40, 5)["idx"], [0, 1, 2, 3, 4])
    # only the visible prefix competes
    assert np.array_equal(oracle.topk_row(inc, 10, 3)["idx"], [9, 8, 7])


def test_indexer_topk_short_rows_select_every_causal_position(oracle):
    # L <= k: every visible key is selected, the rest is -1
    rng = np.random.default_rng(4)
    B, L, H, d, k = 2, 20, 3, 8, 32
    q, kk = rng.standard_normal((B, L, H, d)), rng.standard_normal((B, L, d))
    w = rng.uniform(0, 1, (B, L, H)).astype(np.float32)
    r = oracle.indexer_topk(_bits(q), _bits(kk), w, 0, k)
    for b in range(B):
        for t in range(L):
            got = r["idx"][b, t]
            assert sorted(got[: t + 1].tolist()) == list(range(t + 1))
            assert np.all(got[t + 1:] == -1)
            assert r["next"][b, t] == -np.inf


def test_indexer_topk_invariants_and_torch_topk(oracle):
    rng = np.random.default_rng(6)
    B, Tq, Lk, H, d, k, p0 = 2, 24, 40, 4, 16, 8, 16
    q, kk = rng.standard_normal((B, Tq, H, d)), rng.standard_normal((B, Lk, d))
    w = rng.uniform(0, 1, (B, Tq, H)).astype(np.float32)
    r = oracle.indexer_topk(_bits(q), _bits(kk), w, p0, k)
    sc = oracle.indexer_scores(_bits(q), _bits(kk), w, p0)
    for b in range(B):
        for i in range(Tq):
            nv = min(Lk, p0 + i + 1)
            n = min(nv, k)
            idx = r["idx"][b, i]
            sel = idx[:n]
            assert np.all(idx[n:] == -1)
            assert len(set(sel.tolist())) == n and sel.min() >= 0 and sel.max() < nv
            rest = np.setdiff1d(np.arange(nv), sel)
            if rest.size:
                assert sc[b, i, sel].min() >= sc[b, i, rest].max()
                assert r["next"][b, i] == sc[b, i, rest].max()
            assert r["kth"][b, i] == sc[b, i, sel].min()
            # library top-k on the same scores: same value multiset (ties may permute positions)
            tv = torch.topk(torch.from_numpy(sc[b, i, :nv]), n).values.numpy()
            assert np.array_equal(np.sort(tv), np.sort(sc[b, i, sel]))
            assert np.array_equal(r["sel"][b, i, :n], sc[b, i, sel])


def test_indexer_topk_rows_subset_matches_full(oracle):
    rng = np.random.default_rng(7)
    B, L, H, d, k = 1, 30, 2, 8, 4
    q, kk = rng.standard_normal((B, L, H, d)), rng.standard_normal((B, L, d))
    w = rng.uniform(0, 1, (B, L, H)).astype(np.float32)
    full = oracle.indexer_topk(_bits(q), _bits(kk), w, 0, k)
    rows = [0, 3, 17, 29]
    sub = oracle.indexer_topk(_bits(q), _bits(kk), w, 0, k, rows=rows)
    assert np.array_equal(sub["idx"][0], full["idx"][0, rows])
    assert np.array_equal(sub["kth"][0], full["kth"][0, rows])


def test_positive_row_scaling_of_w_keeps_indices(oracle):
    rng = np.random.default_rng(9)
    B, L, H, d, k = 1, 40, 4, 16, 6
    q, kk = rng.standard_normal((B, L, H, d)), rng.standard_normal((B, L, d))
    w = rng.uniform(0, 1, (B, L, H)).astype(np.float32)
    a = oracle.indexer_topk(_bits(q), _bits(kk), w, 0, k)["idx"]
    b = oracle.indexer_topk(_bits(q), _bits(kk), (w * np.float32(4.0)), 0, k)["idx"]
    assert np.array_equal(a, b)
