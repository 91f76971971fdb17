"""Similarity-based pattern search (paper App. C) on the GPU against the oracle."""
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


@pytest.mark.parametrize("shape", [(37, 16384), (5, 200), (3, 7), (300, 64)])
def test_cosine_rows_matches_oracle(ic, oracle, shape):
    say("cosine rows %s" % (shape,))
    g = torch.Generator().manual_seed(shape[0] * 131 + shape[1])
    A = torch.randn(shape, generator=g).to(torch.bfloat16)
    B = (0.6 * A.float() + 0.8 * torch.randn(shape, generator=g)).to(torch.bfloat16)
    A[1] = 0                                                     # a zero row against a non-zero one
    if shape[0] > 2:
        A[2] = 0
        B[2] = 0                                                 # two zero rows
    mean, rows = ic.cosine_rows(A.cuda(), B.cuda(), want_rows=True)
    torch.cuda.synchronize()
    want_mean, want_rows = oracle.cosine_rows(synth.bits(A), synth.bits(B))
    assert np.allclose(rows.cpu().numpy(), want_rows, rtol=0, atol=2e-6)   # fp32 partial sums of exact products
    assert abs(float(mean) - want_mean) <= 2e-6
    assert rows[1] == 0.0 and (shape[0] <= 2 or rows[2] == 1.0)


def test_similarity_matrix_and_search_on_a_small_stack(ic, oracle):
    """4 drifting layers, L = 256: S against the oracle's fp64 attention outputs (the GPU rounds its
    outputs to bf16 first, hence the tolerance), then the dynamic program on the GPU's S against the
    exhaustive search."""
    cfg = synth.config("c0", Tq=256, Lk=256, k_sel=32)
    say("similarity matrix, 4 layers L=256 k=32")
    n = 4
    ix = list(synth.chain_indexer_layers(cfg, n, device="cuda"))
    idxs = [ic.indexer_topk(l["q"], l["k"], l["w"], cfg["k_sel"], 0) for l in ix]
    at = [synth.attn_layer(cfg, l, device="cuda") for l in range(n)]
    outs = [torch.empty((cfg["B"], cfg["Tq"], cfg["H_q"], cfg["d_v"]), dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    arr = ic.make_layers(at, cfg["k_sel"], 0, cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg), outs)
    S = ic.similarity_matrix(arr, idxs)
    torch.cuda.synchronize()
    S = S.cpu().numpy()
    want = oracle.similarity_matrix([{"Q": synth.bits(a["Q"]), "KV": synth.bits(a["KV"])} for a in at],
                                    [i.cpu().numpy() for i in idxs], cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg))
    say("S (gpu) lower triangle: " + " ".join("%.4f" % S[i, j] for i in range(n) for j in range(i)))
    assert np.allclose(S, want, rtol=0, atol=3e-3)
    assert np.all(np.diag(S) == 1.0) and np.all(np.triu(S, 1) == 0.0)
    # layers[i].O holds the output under the layer's own indices
    own, _ = oracle.sparse_attn(synth.bits(at[2]["Q"]), synth.bits(at[2]["KV"]), idxs[2].cpu().numpy(),
                                cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg))
    assert np.abs(outs[2].float().cpu().numpy() - own).max() <= 2e-2
    # reusing a nearer layer's indices distorts less than reusing a farther layer's
    assert S[3, 2] > S[3, 0]
    for m in (1, 2, 3):
        mask, total = ic.pattern_search_dp(S, m)
        best, arg = oracle.pattern_search_exhaustive(S, m)
        assert abs(total - best) <= 1e-12 and mask in arg
