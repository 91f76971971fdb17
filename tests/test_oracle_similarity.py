"""Pins for the oracle's output-similarity measure and exhaustive pattern search (paper App. C)."""
import numpy as np
import pytest
import torch

import synth


def _bf16(x):
    return synth.bits(torch.from_numpy(np.asarray(x, dtype=np.float32)).to(torch.bfloat16))


def test_cosine_matches_numpy_on_random_rows(oracle):
    rng = np.random.default_rng(2)
    a, b = rng.standard_normal((13, 96)).astype(np.float32), rng.standard_normal((13, 96)).astype(np.float32)
    A, B = _bf16(a), _bf16(b)
    af = torch.from_numpy(A.view(np.int16)).view(torch.bfloat16).double().numpy()
    bf = torch.from_numpy(B.view(np.int16)).view(torch.bfloat16).double().numpy()
    want = (af * bf).sum(1) / (np.linalg.norm(af, axis=1) * np.linalg.norm(bf, axis=1))
    mean, per = oracle.cosine_rows(A, B)
    assert np.allclose(per, want, rtol=0, atol=1e-14)
    assert mean == pytest.approx(want.mean(), abs=1e-14)


def test_cosine_special_cases(oracle):
    e = np.eye(4, 8, dtype=np.float32)
    A = _bf16(np.stack([e[0], e[1], 3 * e[2], np.zeros(8), np.zeros(8), e[3] + e[0]]))
    B = _bf16(np.stack([e[0], e[2], -5 * e[2], np.zeros(8), e[1], e[3] - e[0]]))
    mean, per = oracle.cosine_rows(A, B)
    # same, orthogonal, opposite (any scale), both zero, one zero, orthogonal sums
    assert list(per) == [1.0, 0.0, -1.0, 1.0, 0.0, 0.0]
    assert mean == pytest.approx(1.0 / 6.0, abs=1e-15)
    assert oracle.cosine_rows(A, A)[0] == 1.0


def test_pattern_total_and_exhaustive_search_closed_forms(oracle):
    N = 7
    S = np.zeros((N, N))
    blocks = [0, 0, 0, 3, 3, 5, 5]                          # block heads 0, 3, 5
    for l in range(N):
        for j in range(l):
            S[l, j] = 1.0 if blocks[l] == blocks[j] else 0.1
    # three Full layers: the block heads, every Shared layer sits in its head's block
    best, arg = oracle.pattern_search_exhaustive(S, 3)
    assert arg == [[True, False, False, True, False, True, False]] and best == pytest.approx(4.0)
    assert oracle.pattern_total(S, arg[0]) == pytest.approx(4.0)
    # all Full: nothing is shared; one Full: everybody reads layer 0
    assert oracle.pattern_search_exhaustive(S, N)[0] == 0.0
    assert oracle.pattern_search_exhaustive(S, 1)[0] == pytest.approx(S[1:, 0].sum())
    # the paper's uniform pattern is one of the candidates, so the optimum is never below it
    rng = np.random.default_rng(4)
    R = np.tril(rng.random((9, 9)), -1)
    for m in (2, 3, 5):
        best, arg = oracle.pattern_search_exhaustive(R, m)
        assert all(sum(p) == m and p[0] for p in arg)
        uni = [False] * 9
        for l in range(0, 9, -(-9 // m)):
            uni[l] = True
        if sum(uni) == m:
            assert best >= oracle.pattern_total(R, uni) - 1e-12
