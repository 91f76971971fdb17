"""Pins for the oracle's sparse attention (O4) and its dense reference (O6)."""
import math

import numpy as np
import torch

import synth


def _bits(x):
    return synth.bits(torch.as_tensor(x, dtype=torch.float32).to(torch.bfloat16))


def _val(x):
    return torch.as_tensor(x, dtype=torch.float32).to(torch.bfloat16).to(torch.float64)


def test_dense_reference_vs_torch_sdpa(oracle):
    # the dense causal reference against the library routine (fp64, causal mask)
    rng = np.random.default_rng(1)
    B, L, Hq, dqk, dv = 2, 11, 3, 16, 8
    Q = rng.standard_normal((B, L, Hq, dqk))
    K = rng.standard_normal((B, L, dqk))
    V = rng.standard_normal((B, L, dv))
    KV = np.concatenate([K, V], axis=-1)                       # row = [K | V], v_off = d_qk
    scale = 1.0 / math.sqrt(dqk)
    got = oracle.dense_causal_attn(_bits(Q), _bits(KV), dv, dqk, scale, 0)
    q = _val(Q).permute(0, 2, 1, 3)                            # [B,Hq,L,d]
    k = _val(K)[:, None].expand(B, Hq, L, dqk)
    v = _val(V)[:, None].expand(B, Hq, L, dv)
    want = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True, scale=scale)
    want = want.permute(0, 2, 1, 3).numpy()
    assert np.allclose(got, want, rtol=1e-10, atol=1e-12)


def test_sparse_equals_dense_when_everything_is_selected(oracle):
    # n <= k: the index set is every causal position, so sparse == dense causal attention
    rng = np.random.default_rng(2)
    B, L, Hq, dqk, dv, k = 1, 14, 4, 16, 16, 16
    Q = rng.standard_normal((B, L, Hq, dqk))
    KV = rng.standard_normal((B, L, dqk + dv))
    idx = np.full((B, L, k), -1, dtype=np.int32)
    for t in range(L):
        perm = rng.permutation(t + 1)                          # any order
        idx[0, t, : t + 1] = perm
    scale = 0.25
    got, lse = oracle.sparse_attn(_bits(Q), _bits(KV), idx, dv, dqk, scale)
    want = oracle.dense_causal_attn(_bits(Q), _bits(KV), dv, dqk, scale, 0)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-13)


def test_sparse_mla_layout_shares_latent_between_k_and_v(oracle):
    # MLA row: logits over the whole row, V = the first d_v elements (v_off = 0)
    rng = np.random.default_rng(3)
    B, L, Hq, row, dv, k = 1, 9, 2, 24, 16, 4
    Q = rng.standard_normal((B, L, Hq, row))
    KV = rng.standard_normal((B, L, row))
    idx = np.stack([np.sort(rng.choice(L, size=k, replace=False)) for _ in range(L)])[None].astype(np.int32)
    got, lse = oracle.sparse_attn(_bits(Q), _bits(KV), idx, dv, 0, 0.2)
    q, kv = _val(Q).numpy(), _val(KV).numpy()
    for t in range(L):
        rows = kv[0, idx[0, t]]                                 # [k,row]
        z = 0.2 * q[0, t] @ rows.T                              # [Hq,k]
        p = np.exp(z - z.max(-1, keepdims=True))
        p /= p.sum(-1, keepdims=True)
        assert np.allclose(got[0, t], p @ rows[:, :dv], rtol=1e-12, atol=1e-13)
        assert np.allclose(lse[0, t], np.log(np.exp(z).sum(-1)), rtol=1e-12)


def test_sparse_special_cases(oracle):
    rng = np.random.default_rng(4)
    B, L, Hq, dqk, dv = 1, 10, 3, 8, 8
    Q = rng.standard_normal((B, L, Hq, dqk))
    KV = rng.standard_normal((B, L, dqk + dv))
    kvv = _val(KV).numpy()
    # k = 1: the output is the selected V row itself
    idx1 = rng.integers(0, L, size=(B, L, 1)).astype(np.int32)
    O1, _ = oracle.sparse_attn(_bits(Q), _bits(KV), idx1, dv, dqk, 0.3)
    for t in range(L):
        for h in range(Hq):
            assert np.array_equal(O1[0, t, h], kvv[0, idx1[0, t, 0], dqk:])
    # Q = 0: uniform weights, the output is the mean of the selected V rows; -1 entries skipped
    idx = np.array([[0, 3, -1, 7, 5, -1]] * L, dtype=np.int32)[None]
    O0, lse0 = oracle.sparse_attn(_bits(np.zeros_like(Q)), _bits(KV), idx, dv, dqk, 0.3)
    mean = kvv[0, [0, 3, 7, 5], dqk:].mean(0)
    assert np.allclose(O0[0, 2, 1], mean, rtol=1e-13)
    assert np.allclose(lse0, math.log(4.0))
    # permuting the index list does not change the result
    a, _ = oracle.sparse_attn(_bits(Q), _bits(KV), idx, dv, dqk, 0.3)
    b, _ = oracle.sparse_attn(_bits(Q), _bits(KV), np.ascontiguousarray(idx[:, :, ::-1]), dv, dqk, 0.3)
    assert np.allclose(a, b, rtol=1e-12, atol=1e-14)
    # an empty row gives zeros and lse = -inf
    e = np.full((B, L, 3), -1, dtype=np.int32)
    Oe, lsee = oracle.sparse_attn(_bits(Q), _bits(KV), e, dv, dqk, 0.3)
    assert np.all(Oe == 0) and np.all(np.isneginf(lsee))
    # row subset addressing
    rows = [1, 8]
    Os, _ = oracle.sparse_attn(_bits(Q), _bits(KV), idx, dv, dqk, 0.3, rows=rows)
    assert np.array_equal(Os[0], a[0, rows])
    Oss, _ = oracle.sparse_attn(_bits(Q), _bits(KV), np.ascontiguousarray(idx[:, rows]), dv, dqk, 0.3,
                                rows=rows, idx_is_subset=True)
    assert np.array_equal(Oss, Os)


def test_topk_attention_approaches_dense_as_k_grows(oracle):
    # brute force on a tiny stack: with k >= L sparse(indexer top-k) == dense; with smaller k the
    # selected softmax mass is a subset, so the output differs but stays a convex combination.
    cfg = synth.config("c0", Tq=48, Lk=48, k_sel=64)
    layer = synth.bits_layer(synth.stack_layers(cfg, n_layers=1)[0])
    r = oracle.indexer_topk(layer["q"], layer["k"], layer["w"], 0, cfg["k_sel"])
    O, _ = oracle.sparse_attn(layer["Q"], layer["KV"], r["idx"], cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg))
    D = oracle.dense_causal_attn(layer["Q"], layer["KV"], cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg), 0)
    assert np.allclose(O, D, rtol=1e-12, atol=1e-13)
    r8 = oracle.indexer_topk(layer["q"], layer["k"], layer["w"], 0, 8)
    O8, _ = oracle.sparse_attn(layer["Q"], layer["KV"], r8["idx"], cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg))
    assert np.allclose(O8[0, :8], D[0, :8], rtol=1e-12, atol=1e-13)      # rows with <= 8 keys
    assert not np.allclose(O8[0, 40:], D[0, 40:], atol=1e-3)
    V = torch.from_numpy(layer["KV"].view(np.int16)).view(torch.bfloat16).double().numpy()[0, :, cfg["v_off"]:]
    assert O8.max() <= V.max() + 1e-12 and O8.min() >= V.min() - 1e-12
