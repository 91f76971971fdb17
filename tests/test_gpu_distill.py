"""Forward of the indexer's distillation loss (paper Sec. 3.3) on the GPU against the oracle."""
import math
import sys

import numpy as np
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu


def say(msg):
    print("[gpu-test] " + msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def ic():
    import paper_2603_12201_amd as m
    m.lib()
    return m


def _rand_idx(seed, B, Tq, Lk, ks, p0, holes):
    rng = np.random.default_rng(seed)
    idx = np.full((B, Tq, ks), -1, dtype=np.int32)
    for b in range(B):
        for i in range(Tq):
            nv = max(0, min(Lk, p0 + i + 1))
            n = min(nv, ks)
            idx[b, i, :n] = np.sort(rng.choice(nv, size=n, replace=False))
            if holes and n > 3:
                idx[b, i, rng.choice(n, size=n // 3, replace=False)] = -1
    return idx


PROB_CASES = [
    # B, Tq, Lk, Hq, d_qk, row, k_sel, q_pos0, holes
    (1, 40, 300, 32, 576, 576, 128, 260, False),     # MLA rows, two tiles
    (2, 9, 200, 20, 576, 640, 100, 150, True),       # ragged heads, padded rows, ragged last tile, holes
    (1, 50, 50, 4, 64, 128, 16, 0, False),           # tiny-config shape, short causal rows
    (1, 6, 500, 32, 576, 576, 300, 494, True),
    (1, 4, 5000, 32, 576, 576, 2048, 4996, True),   # the workload's k: 32 steps per wave
]


@pytest.mark.parametrize("case", PROB_CASES)
def test_attn_probs_matches_oracle(ic, oracle, case):
    B, Tq, Lk, Hq, d_qk, row, ks, p0, holes = case
    say("attention probabilities B=%d Tq=%d Lk=%d Hq=%d dqk=%d row=%d k=%d p0=%d holes=%s" % case)
    g = torch.Generator().manual_seed(40 + Tq + ks)
    Q = torch.randn((B, Tq, Hq, d_qk), generator=g).to(torch.bfloat16)
    KV = torch.randn((B, Lk, row), generator=g).to(torch.bfloat16)
    idx = _rand_idx(7 + Tq, B, Tq, Lk, ks, p0, holes)
    idx[0, 0, :] = -1                                  # an empty row
    scale = 1.0 / math.sqrt(d_qk)
    d_v, v_off = (512, 0) if d_qk == 576 else (64, 64)
    idx_d = torch.from_numpy(idx).cuda()
    _, lse = ic.sparse_attn(Q.cuda(), KV.cuda(), idx_d, d_v, v_off, scale, want_lse=True)
    P = ic.attn_probs(Q.cuda(), KV.cuda(), idx_d, scale, lse)
    torch.cuda.synchronize()
    want = oracle.attn_distribution_selected(synth.bits(Q), synth.bits(KV), idx, scale)
    got = P.cpu().numpy()
    # bf16 inputs, fp32 accumulation over 576 features, probabilities <= 1
    assert np.abs(got - want).max() <= 2e-3 * max(want.max(), 1e-3) + 1e-6
    assert np.all(got[idx < 0] == 0) and np.all(got[0, 0] == 0)
    sums = got.sum(-1)
    assert np.allclose(sums[(idx >= 0).any(-1)], 1.0, atol=2e-3)


def test_distill_loss_and_proposition_1(ic, oracle):
    """One Full layer serving itself and two Shared layers: Eq. 1, Eq. 2 and the shared gradient."""
    cfg = synth.config("c0", Tq=160, Lk=160, k_sel=32)
    say("distillation loss, 3 served layers, L=160 k=32")
    ix = synth.indexer_layer(cfg, 0, device="cuda")
    idx, sel = ic.indexer_topk(ix["q"], ix["k"], ix["w"], cfg["k_sel"], 0, want_scores=True)
    scale = synth.sm_scale(cfg)
    probs, at_host = [], []
    for l in range(3):
        at = synth.attn_layer(cfg, l, device="cuda")
        _, lse = ic.sparse_attn(at["Q"], at["KV"], idx, cfg["d_v"], cfg["v_off"], scale, want_lse=True)
        probs.append(ic.attn_probs(at["Q"], at["KV"], idx, scale, lse))
        at_host.append((synth.bits(at["Q"].cpu()), synth.bits(at["KV"].cpu())))
    lm, la, grad = ic.distill_loss(probs, sel, want_grad=True)
    torch.cuda.synchronize()
    idx_h = idx.cpu().numpy()
    # the oracle on the GPU's own index sets: its scores at those positions, its distributions
    sc = oracle.indexer_scores(synth.bits(ix["q"].cpu()), synth.bits(ix["k"].cpu()), synth.bits(ix["w"].cpu()), 0)
    sel_o = np.where(idx_h >= 0, np.take_along_axis(sc, np.maximum(idx_h, 0), axis=-1), -np.inf)
    q = oracle.indexer_distribution(sel_o)
    ps = [oracle.attn_distribution_selected(Q, KV, idx_h, scale) for Q, KV in at_host]
    want_m, want_a = oracle.distill_loss_multi(ps, q), oracle.distill_loss_avg(ps, q)
    say("Eq.1 gpu %.6f oracle %.6f | Eq.2 gpu %.6f oracle %.6f" % (float(lm), want_m, float(la), want_a))
    assert float(lm) == pytest.approx(want_m, rel=1e-2) and float(la) == pytest.approx(want_a, rel=1e-2)
    g = grad.cpu().numpy()
    assert np.abs(g - oracle.distill_grad_logits(ps, q)).max() <= 3e-3
    # Prop. 1 on the GPU's own numbers: the gap between the two losses is the entropy gap of the targets
    P = [p.double().cpu().numpy() for p in probs]
    H = lambda p: -np.where(p > 0, p * np.log(np.where(p > 0, p, 1.0)), 0.0).sum()
    gap = H(sum(P) / 3) - sum(H(p) for p in P) / 3
    assert float(lm) - float(la) == pytest.approx(gap, rel=1e-4, abs=1e-6) and gap > 0
    # the gap does not move when the indexer changes: another layer's scores on the same sets
    ix2 = synth.indexer_layer(cfg, 1, device="cuda")
    sc2 = ic.debug_indexer_scores(ix2["q"], ix2["k"], ix2["w"], 0, 0, cfg["Tq"])
    sel2 = torch.where(idx >= 0, torch.gather(sc2, 2, idx.clamp(min=0).long()), torch.full_like(sel, float("-inf")))
    lm2, la2 = ic.distill_loss(probs, sel2.contiguous())
    assert float(lm2) - float(la2) == pytest.approx(gap, rel=1e-4, abs=1e-6)
    # one served layer: Eq. 1 = Eq. 2 = the single-layer DSA loss
    l1, a1 = ic.distill_loss(probs[:1], sel)
    assert float(l1) == pytest.approx(float(a1), rel=1e-6) and float(l1) == pytest.approx(oracle.kl_rows(ps[0], q).sum(), rel=1e-2)


@pytest.mark.parametrize("k_sel", [700, 2048, 3000])
def test_distill_loss_row_lengths(ic, oracle, k_sel):
    """ic_distill_loss on given distributions: the register-resident row kernel (k <= 2048, ragged and
    full) and the re-reading one (longer rows), with empty slots and one empty row."""
    say("distillation loss on synthetic distributions, k=%d" % k_sel)
    nq, m1 = 37, 3
    rng = np.random.default_rng(k_sel)
    logits = rng.normal(size=(1, nq, k_sel)).astype(np.float32) * 2.0
    empty = rng.random((1, nq, k_sel)) < 0.1
    empty[0, 5] = True                                       # a row with nothing selected
    logits[empty] = -np.inf
    ps = []
    for j in range(m1):
        e = rng.random((1, nq, k_sel)) ** 4
        e[empty] = 0.0
        s = e.sum(-1, keepdims=True)
        ps.append(np.where(s > 0, e / np.where(s > 0, s, 1.0), 0.0).astype(np.float32))
    lm, la, grad = ic.distill_loss([torch.from_numpy(p).cuda() for p in ps], torch.from_numpy(logits).cuda(), want_grad=True)
    torch.cuda.synchronize()
    q = oracle.indexer_distribution(logits.astype(np.float64))
    p64 = [p.astype(np.float64) for p in ps]
    want_m, want_a = oracle.distill_loss_multi(p64, q), oracle.distill_loss_avg(p64, q)
    assert float(lm) == pytest.approx(want_m, rel=1e-5) and float(la) == pytest.approx(want_a, rel=1e-5)
    g = grad.cpu().numpy()
    assert np.abs(g - oracle.distill_grad_logits(p64, q)).max() <= 1e-5
    assert np.all(g[0, 5] == 0)
