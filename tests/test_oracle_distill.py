"""Pins for the oracle's multi-layer distillation loss (paper Sec. 3.3: Eq. 1, Eq. 2, Prop. 1)."""
import math

import numpy as np
import pytest
import torch

import synth


def _bits(x):
    return synth.bits(torch.from_numpy(np.asarray(x, dtype=np.float32)).to(torch.bfloat16))


def _softmax(x):
    e = np.exp(x - x.max(-1, keepdims=True))
    return e / e.sum(-1, keepdims=True)


def test_kl_closed_forms(oracle):
    n = 8
    u = np.full(n, 1.0 / n)
    d = np.zeros(n); d[3] = 1.0
    assert oracle.kl_rows(u, u) == 0.0
    assert oracle.kl_rows(d, u) == pytest.approx(math.log(n), abs=1e-15)
    assert oracle.kl_rows([0.5, 0.5], [0.25, 0.75]) == pytest.approx(0.5 * math.log(2) + 0.5 * math.log(2 / 3), abs=1e-15)
    assert np.isinf(oracle.kl_rows([0.5, 0.5], [1.0, 0.0]))
    rng = np.random.default_rng(0)
    p, q = _softmax(rng.standard_normal((20, 33))), _softmax(rng.standard_normal((20, 33)))
    assert np.all(oracle.kl_rows(p, q) > 0) and np.allclose(oracle.kl_rows(p, p), 0, atol=1e-15)   # Gibbs


def test_indexer_distribution_special_cases(oracle):
    sc = np.array([[0.0, 0.0, -np.inf, 0.0], [1.0, -np.inf, -np.inf, -np.inf], [-np.inf] * 4,
                   [math.log(1), math.log(2), math.log(3), math.log(4)]])
    q = oracle.indexer_distribution(sc)
    assert np.allclose(q[0], [1 / 3, 1 / 3, 0, 1 / 3]) and np.array_equal(q[1], [1, 0, 0, 0]) and np.all(q[2] == 0)
    assert np.allclose(q[3], [0.1, 0.2, 0.3, 0.4], atol=1e-15)
    big = oracle.indexer_distribution(np.array([1000.0, 999.0]))       # no overflow
    assert big[0] == pytest.approx(1 / (1 + math.exp(-1)))


def test_aggregated_attention_is_tied_to_the_attention_oracle(oracle):
    # MQA shares the value row across heads, so sum_s p_bar(s) V[s] = mean over heads of the
    # attention output; with no more selected rows than value features and random V that pins
    # every p_bar(s), and the attention output is pinned elsewhere (dense softmax, library routines)
    rng = np.random.default_rng(3)
    B, Tq, Lk, H, d_qk, d_v, row, ks = 2, 9, 40, 4, 64, 64, 128, 24
    Q, KV = _bits(rng.standard_normal((B, Tq, H, d_qk))), _bits(rng.standard_normal((B, Lk, row)))
    idx = np.full((B, Tq, ks), -1, dtype=np.int32)
    for b in range(B):
        for t in range(Tq):
            n = rng.integers(1, ks + 1)
            idx[b, t, :n] = np.sort(rng.choice(Lk, size=n, replace=False))
    idx[0, 0, :] = -1                                                    # an empty row
    P = oracle.attn_distribution_selected(Q, KV, idx, 0.125)
    O, _ = oracle.sparse_attn(Q, KV, idx, d_v, 64, 0.125)
    V = oracle._widen_bf16(KV)[:, :, 64:128]
    for b in range(B):
        for t in range(Tq):
            sel = idx[b, t] >= 0
            assert np.allclose(P[b, t, ~sel], 0) and (not sel.any() or abs(P[b, t].sum() - 1) < 1e-12)
            want = O[b, t].mean(axis=0)
            assert np.allclose(P[b, t, sel] @ V[b, idx[b, t, sel]], want, atol=1e-12)
            if sel.any():                                                # and the map p -> p V is injective here
                sol = np.linalg.lstsq(V[b, idx[b, t, sel]].T, want, rcond=None)[0]
                assert np.allclose(sol, P[b, t, sel], atol=1e-9)
    assert np.all(P[0, 0] == 0)


def test_dense_and_selected_forms_agree_when_everything_is_selected(oracle):
    rng = np.random.default_rng(4)
    B, Tq, Lk, H, d = 1, 12, 12, 3, 64
    Q, KV = _bits(rng.standard_normal((B, Tq, H, d))), _bits(rng.standard_normal((B, Lk, 128)))
    dense = oracle.attn_distribution_dense(Q, KV, 0.2, 0)
    idx = np.full((B, Tq, Lk), -1, dtype=np.int32)
    for t in range(Tq):
        idx[0, t, :t + 1] = np.arange(t + 1)
    assert np.allclose(oracle.attn_distribution_selected(Q, KV, idx, 0.2), dense, atol=1e-15)
    assert np.allclose(dense.sum(-1), 1) and np.all(np.triu(dense[0], 1) == 0)
    # zero queries: every visible key gets the same probability
    Z = oracle.attn_distribution_dense(_bits(np.zeros((B, Tq, H, d))), KV, 0.2, 0)
    for t in range(Tq):
        assert np.allclose(Z[0, t, :t + 1], 1.0 / (t + 1))


def test_proposition_1(oracle):
    rng = np.random.default_rng(5)
    T, n, m = 7, 19, 3
    ps = [_softmax(2 * rng.standard_normal((T, n))) for _ in range(m + 1)]
    logits = rng.standard_normal((T, n))
    q = oracle.indexer_distribution(logits)
    lm, la = oracle.distill_loss_multi(ps, q), oracle.distill_loss_avg(ps, q)
    # Eq. 1 - Eq. 2 = H(p_bar) - mean_j H(p_j): no q in it (that is the proof), and >= 0 (Jensen)
    H = lambda p: -(p * np.log(p)).sum()
    gap = H(sum(ps) / (m + 1)) - sum(H(p) for p in ps) / (m + 1)
    assert lm - la == pytest.approx(gap, abs=1e-12) and gap > 0
    q2 = oracle.indexer_distribution(rng.standard_normal((T, n)))
    assert oracle.distill_loss_multi(ps, q2) - oracle.distill_loss_avg(ps, q2) == pytest.approx(gap, abs=1e-12)
    # the gradients with respect to the logits: finite differences of both losses against q - p_bar
    g = oracle.distill_grad_logits(ps, q)
    assert np.allclose(g, q - sum(ps) / (m + 1), atol=1e-15)
    eps = 1e-6
    for (t, s) in [(0, 0), (3, 7), (6, 18)]:
        lp, lmn = logits.copy(), logits.copy()
        lp[t, s] += eps; lmn[t, s] -= eps
        qp, qm = oracle.indexer_distribution(lp), oracle.indexer_distribution(lmn)
        fd_multi = (oracle.distill_loss_multi(ps, qp) - oracle.distill_loss_multi(ps, qm)) / (2 * eps)
        fd_avg = (oracle.distill_loss_avg(ps, qp) - oracle.distill_loss_avg(ps, qm)) / (2 * eps)
        assert fd_multi == pytest.approx(g[t, s], abs=1e-8) and fd_avg == pytest.approx(g[t, s], abs=1e-8)
    # m = 0 is the single-layer DSA loss; identical targets make the two losses equal
    assert oracle.distill_loss_multi(ps[:1], q) == pytest.approx(kl := oracle.kl_rows(ps[0], q).sum())
    assert oracle.distill_loss_avg(ps[:1], q) == pytest.approx(kl)
    assert oracle.distill_loss_multi([ps[0]] * 3, q) == pytest.approx(oracle.distill_loss_avg([ps[0]] * 3, q), abs=1e-12)
