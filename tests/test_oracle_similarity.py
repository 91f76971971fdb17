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


# ---- pins of similarity_matrix / pattern_loss_forward that share nothing with their own cosine ----
# Construction: one head, Q = 0 (uniform attention over the selected rows) and one-hot value rows
# V[s] = e_s, so a layer's output under the index set A is (1/|A|) * sum_{s in A} e_s and the cosine of
# the outputs under two sets A, B is |A & B| / sqrt(|A| |B|): plain set arithmetic.

def _onehot_layer(Lk, Tq, d=64):
    Q = np.zeros((1, Tq, 1, d), dtype=np.float32)
    KV = np.zeros((1, Lk, 2 * d), dtype=np.float32)
    KV[0, :, :d] = np.random.default_rng(Lk).standard_normal((Lk, d))   # keys: irrelevant under Q = 0
    for s in range(Lk):
        KV[0, s, d + s] = 1.0                                             # values: e_s
    return {"Q": _bf16(Q), "KV": _bf16(KV)}


def _set_cos(A, B):
    A, B = set(A), set(B)
    if not A and not B:
        return 1.0
    if not A or not B:
        return 0.0
    return len(A & B) / np.sqrt(len(A) * len(B))


def test_similarity_matrix_on_orthogonal_values_is_set_overlap(oracle):
    Lk, Tq, k = 10, 4, 4
    layers = [_onehot_layer(Lk, Tq) for _ in range(3)]
    rows = [  # per layer, per token: selected positions (-1 = empty slot)
        [[0, 1, 2, 3], [4, 5, -1, -1], [-1, -1, -1, -1], [9, -1, -1, -1]],
        [[0, 1, 2, 3], [5, 6, 7, -1], [-1, -1, -1, -1], [1, 2, -1, -1]],
        [[3, 2, 8, 9], [4, 5, -1, -1], [0, -1, -1, -1], [9, 8, 7, 6]],
    ]
    idx = [np.array(r, dtype=np.int32)[None] for r in rows]
    S = oracle.similarity_matrix(layers, idx, 64, 64, 1.0)
    # by hand, layer 1 against 0: tokens (1, 1/sqrt(6), both empty = 1, 0) -> mean 0.60206...
    assert S[1, 0] == pytest.approx((1.0 + 1.0 / np.sqrt(6.0) + 1.0 + 0.0) / 4.0, abs=1e-12)
    # layer 2 against 0: (2/4, 1, non-empty vs empty = 0, 1/sqrt(4)) ; against 1: (2/4, 1/sqrt(6), 0, 0)
    assert S[2, 0] == pytest.approx((0.5 + 1.0 + 0.0 + 0.5) / 4.0, abs=1e-12)
    assert S[2, 1] == pytest.approx((0.5 + 1.0 / np.sqrt(6.0) + 0.0 + 0.0) / 4.0, abs=1e-12)
    for i in range(3):
        for j in range(i):
            want = np.mean([_set_cos([s for s in rows[i][t] if s >= 0], [s for s in rows[j][t] if s >= 0]) for t in range(Tq)])
            assert S[i, j] == pytest.approx(want, abs=1e-12)
        assert S[i, i] == 1.0 and np.all(S[i, i + 1:] == 0.0)
    # identical index tensors: exactly 1, whatever the values are
    cfg = synth.config("c0", Tq=40, Lk=40, k_sel=8, n_layers=2)
    ls = [synth.bits_layer(l) for l in synth.stack_layers(cfg)]
    same = np.sort(np.random.default_rng(1).integers(0, 40, (1, 40, 8)).astype(np.int32), -1)
    assert oracle.similarity_matrix(ls, [same, same.copy()], cfg["d_v"], cfg["v_off"], 0.125)[1, 0] == pytest.approx(1.0, abs=1e-15)


def test_similarity_matrix_agrees_with_the_row_cosine_routine(oracle):
    # the C routine cosine_rows (pinned above against numpy and special cases) on the attention
    # oracle's outputs rounded to bf16: the rounding moves a cosine by well under 1e-3
    cfg = synth.config("c0", Tq=64, Lk=64, k_sel=8, n_layers=3)
    ls = [synth.bits_layer(l) for l in synth.stack_layers(cfg)]
    rng = np.random.default_rng(3)
    idx = []
    for _ in range(3):
        a = np.full((1, 64, 8), -1, dtype=np.int32)
        for t in range(64):
            n = min(t + 1, 8)
            a[0, t, :n] = np.sort(rng.choice(t + 1, size=n, replace=False))
        idx.append(a)
    sc = synth.sm_scale(cfg)
    S = oracle.similarity_matrix(ls, idx, cfg["d_v"], cfg["v_off"], sc)
    for i in range(3):
        own, _ = oracle.sparse_attn(ls[i]["Q"], ls[i]["KV"], idx[i], cfg["d_v"], cfg["v_off"], sc)
        for j in range(i):
            re, _ = oracle.sparse_attn(ls[i]["Q"], ls[i]["KV"], idx[j], cfg["d_v"], cfg["v_off"], sc)
            mean, _ = oracle.cosine_rows(_bf16(own.reshape(64, -1)), _bf16(re.reshape(64, -1)))
            assert S[i, j] == pytest.approx(mean, abs=2e-3)
            assert 0.0 < S[i, j] < 1.0


def test_pattern_loss_forward_on_orthogonal_values_is_set_overlap(oracle):
    # indexer: one head, one-hot q, w = 1, so the score of key s is its coordinate v_l[s] and the top-k
    # of token t are the k largest of v_l[0..t] (sorted here with Python, lower position first on ties)
    Lk = Tq = 9
    k, d = 3, 64
    vals = [
        [5, 1, 4, 2, 8, 7, 3, 6, 0],
        [5, 1, 4, 2, 8, 0, 3, 6, 7],
        [0, 1, 2, 3, 4, 5, 6, 7, 8],
        [5, 1, 4, 2, 8, 7, 3, 6, 0],
    ]
    layers = []
    for v in vals:
        L = _onehot_layer(Lk, Tq, d)
        q = np.zeros((1, Tq, 1, d), dtype=np.float32); q[..., 3] = 1.0
        kk = np.zeros((1, Lk, d), dtype=np.float32); kk[0, :, 3] = np.array(v, dtype=np.float32) + 1.0
        L.update({"q": _bf16(q), "k": _bf16(kk), "w": np.ones((1, Tq, 1), dtype=np.float32)})
        layers.append(L)

    def topk(v, t):
        return set(sorted(range(t + 1), key=lambda s: (-v[s], s))[:k])

    args = (k, 0, d, d, 1.0)
    ref, used, _ = oracle.forward_stack(layers, [True] * 4, *args)
    for l in range(4):                                             # the driver's sets are the hand-sorted ones
        for t in range(Tq):
            assert set(int(s) for s in used[l][0, t] if s >= 0) == topk(vals[l], t)
    for mask in ([True, False, False, False], [True, False, True, False], [True, True, False, True], [True] * 4):
        want, src = 0.0, 0
        for l in range(4):
            if mask[l]:
                src = l
            want += 1.0 - np.mean([_set_cos(topk(vals[src], t), topk(vals[l], t)) for t in range(Tq)])
        got = oracle.pattern_loss_forward(layers, mask, *args, ref)
        assert got == pytest.approx(want / 4.0, abs=1e-12)
    # one value by hand: FSSS.  Layer 3 has layer 0's keys (loss 0).  Layer 1 agrees with layer 0 up to
    # token 4 and shares two of three positions afterwards (token 5, 6: {0,4,5} | {0,2,4}; token 7:
    # {4,5,7} | {0,4,7}; token 8: {4,5,7} | {4,7,8}), so its similarity is (5 + 4 * 2/3) / 9.
    got = oracle.pattern_loss_forward(layers, [True, False, False, False], *args, ref)
    l1 = 1.0 - np.mean([1, 1, 1, 1, 1, 2 / 3, 2 / 3, 2 / 3, 2 / 3])
    l2 = 1.0 - np.mean([_set_cos(topk(vals[0], t), topk(vals[2], t)) for t in range(Tq)])
    assert got == pytest.approx((0.0 + l1 + l2 + 0.0) / 4.0, abs=1e-12)
