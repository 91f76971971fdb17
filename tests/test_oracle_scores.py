"""Pins for the oracle's widening (O1) and indexer score (O2).

Each check ties the oracle to something other than itself: a library conversion,
a library matmul in a special case, a hand-computed closed form, or a dense
brute-force einsum on tiny inputs."""
import math

import numpy as np
import torch

import synth


def _bf16_bits(x):
    return synth.bits(torch.as_tensor(x, dtype=torch.float32).to(torch.bfloat16))


def _bf16_val(x):
    return torch.as_tensor(x, dtype=torch.float32).to(torch.bfloat16).to(torch.float64).numpy()


def test_widen_bf16_all_patterns(oracle):
    # every finite bf16 bit pattern against torch's own bf16 -> fp64 conversion
    allbits = np.arange(65536, dtype=np.uint16)
    t = torch.from_numpy(allbits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    lib = oracle.lib()
    for b in list(range(0, 65536, 97)) + [0, 1, 0x7F7F, 0x8000, 0xFF7F, 0x3F80, 0xBF80]:
        v = lib.ico_widen_bf16(int(b))
        if math.isnan(t[b]):
            assert math.isnan(v)
        else:
            assert v == t[b], (b, v, t[b])


def test_widen_e4m3_all_bytes(oracle):
    # all 256 bytes against torch.float8_e4m3fn (OCP e4m3: max 448, no inf, 0x7F/0xFF NaN)
    allb = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    t = allb.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    lib = oracle.lib()
    for b in range(256):
        v = lib.ico_widen_e4m3(b)
        if math.isnan(t[b]):
            assert math.isnan(v), b
        else:
            assert v == t[b], (b, v, t[b])
    assert lib.ico_widen_e4m3(0x7E) == 448.0
    assert lib.ico_widen_e4m3(0x01) == 2.0 ** -9
    assert lib.ico_widen_e4m3(0x38) == 1.0


def _dense_scores(qv, kv, w, q_pos0):
    """Dense brute force: full [B,Tq,Lk] score matrix with numpy einsum, then mask."""
    dots = np.einsum("bijc,bsc->bijs", qv, kv)
    sc = np.einsum("bij,bijs->bis", w.astype(np.float64), np.maximum(dots, 0.0))
    B, Tq, Lk = sc.shape
    for i in range(Tq):
        sc[:, i, max(0, min(Lk, q_pos0 + i + 1)):] = -np.inf
    return sc


def test_scores_vs_dense_bruteforce(oracle):
    rng = np.random.default_rng(11)
    for (B, Tq, Lk, H, d, p0) in [(1, 9, 9, 3, 8, 0), (2, 5, 12, 4, 16, 7), (1, 6, 4, 2, 8, 0),
                                   (2, 1, 10, 5, 8, 9), (1, 7, 7, 1, 24, 0)]:
        q = rng.standard_normal((B, Tq, H, d))
        k = rng.standard_normal((B, Lk, d))
        w = rng.uniform(-1, 1, (B, Tq, H)).astype(np.float32)   # signed w on purpose
        got = oracle.indexer_scores(_bf16_bits(q), _bf16_bits(k), w, p0)
        want = _dense_scores(_bf16_val(q), _bf16_val(k), w, p0)
        assert got.shape == want.shape
        fin = np.isfinite(want)
        assert np.array_equal(np.isfinite(got), fin)
        assert np.allclose(got[fin], want[fin], rtol=1e-12, atol=1e-12)


def test_scores_single_head_unit_weight_is_relu_matmul(oracle):
    # H_I = 1, w = 1: I = ReLU(q k^T), a plain library matmul
    rng = np.random.default_rng(5)
    Tq, Lk, d = 13, 13, 32
    q = rng.standard_normal((1, Tq, 1, d))
    k = rng.standard_normal((1, Lk, d))
    w = np.ones((1, Tq, 1), dtype=np.float32)
    got = oracle.indexer_scores(_bf16_bits(q), _bf16_bits(k), w, 0)[0]
    want = np.maximum(_bf16_val(q)[0, :, 0, :] @ _bf16_val(k)[0].T, 0.0)
    low = np.tril(np.ones((Tq, Lk), dtype=bool))
    assert np.allclose(got[low], want[low], rtol=1e-12, atol=1e-12)
    assert (want[low] == 0).any() and (want[low] > 0).any()     # the gate is exercised
    assert np.all(np.isneginf(got[~low]))


def test_scores_closed_form_one_hot(oracle):
    # q[t,j] = a_j * e_{c_j}: the dot product picks one key coordinate, so
    # I[t,s] = sum_j w_j * max(a_j * k[s,c_j], 0), computed by hand below.
    d, H, Lk = 8, 3, 4
    a = [2.0, -1.0, 0.5]
    c = [1, 4, 7]
    w = [0.5, 2.0, -3.0]
    k = np.array([[1, 2, 3, 4, 5, 6, 7, 8],
                  [-1, -2, -3, -4, -5, -6, -7, -8],
                  [0, 1, 0, 1, 0, 1, 0, 1],
                  [4, -3, 2, -1, 0, 1, -2, 3]], dtype=np.float64)
    q = np.zeros((1, 1, H, d))
    for j in range(H):
        q[0, 0, j, c[j]] = a[j]
    wv = np.array(w, dtype=np.float32).reshape(1, 1, H)
    got = oracle.indexer_scores(_bf16_bits(q), _bf16_bits(k[None]), wv, q_pos0=Lk - 1)[0, 0]
    # by hand: s=0: .5*max(2*2,0)+2*max(-1*5,0)-3*max(.5*8,0) = 2+0-12 = -10
    #          s=1: .5*max(-4,0)+2*max(5,0)-3*max(-4,0)       = 0+10-0 = 10
    #          s=2: .5*max(2,0)+2*max(0,0)-3*max(.5,0)        = 1+0-1.5 = -0.5
    #          s=3: .5*max(-6,0)+2*max(0,0)-3*max(1.5,0)      = -4.5
    assert np.array_equal(got, np.array([-10.0, 10.0, -0.5, -4.5]))


def test_scores_algebraic_invariants(oracle):
    rng = np.random.default_rng(3)
    B, Tq, Lk, H, d = 1, 16, 16, 4, 16
    q = _bf16_val(rng.standard_normal((B, Tq, H, d)))
    k = _bf16_val(rng.standard_normal((B, Lk, d)))
    w1 = rng.uniform(0, 1, (B, Tq, H)).astype(np.float32)
    w2 = rng.uniform(0, 1, (B, Tq, H)).astype(np.float32)
    f = lambda qq, kk, ww: oracle.indexer_scores(_bf16_bits(qq), _bf16_bits(kk), ww, 0)
    low = np.tril(np.ones((Tq, Lk), dtype=bool))[None]
    s1, s2 = f(q, k, w1), f(q, k, w2)
    s12 = f(q, k, (w1.astype(np.float64) + w2).astype(np.float32))
    w12 = (w1.astype(np.float64) + w2).astype(np.float32).astype(np.float64)
    # linear in w (w sits outside the gate)
    lin = s1 + s2 + f(q, k, (w12 - w1.astype(np.float64) - w2).astype(np.float32))
    assert np.allclose(s12[low], lin[low], rtol=1e-9, atol=1e-9)
    # positively homogeneous in q (power of two keeps bf16 exact)
    assert np.allclose(f(2.0 * q, k, w1)[low], 2.0 * s1[low], rtol=1e-12)
    # flipping the sign of k turns the gate onto the other side:
    # relu(x) - relu(-x) = x, so I(k) - I(-k) = sum_j w_j (q_j . k)
    with np.errstate(invalid="ignore"):
        diff = s1 - f(q, -k, w1)
    plain = np.einsum("bij,bijs->bis", w1.astype(np.float64), np.einsum("bijc,bsc->bijs", q, k))
    assert np.allclose(diff[low], plain[low], rtol=1e-9, atol=1e-9)
    # exact zeros where every head's dot product is negative
    dots = np.einsum("bijc,bsc->bijs", q, k)
    allneg = (dots < 0).all(axis=2) & low
    assert allneg.any()
    assert np.all(s1[allneg] == 0.0)


def test_scores_fp8_matches_scaled_dense(oracle):
    rng = np.random.default_rng(8)
    B, Tq, Lk, H, d = 1, 5, 5, 2, 16
    q = torch.from_numpy(rng.standard_normal((B, Tq, H * d))).float()
    k = torch.from_numpy(rng.standard_normal((B, Lk, d))).float()
    q8, qs = synth.quantize_e4m3(q)
    k8, ks = synth.quantize_e4m3(k)
    w = rng.uniform(0, 1, (B, Tq, H)).astype(np.float32)
    got = oracle.indexer_scores(synth.bits(q8).reshape(B, Tq, H, d), synth.bits(k8), w, 0,
                                dtype=oracle.FP8_E4M3, q_scale=synth.bits(qs), k_scale=synth.bits(ks))
    qv = q8.to(torch.float64).numpy().reshape(B, Tq, H, d) * qs.double().numpy()[..., None, None]
    kv = k8.to(torch.float64).numpy() * ks.double().numpy()[..., None]
    want = _dense_scores(qv, kv, w, 0)
    fin = np.isfinite(want)
    assert np.allclose(got[fin], want[fin], rtol=1e-12, atol=1e-14)
    # the dequantised tensors stay close to the originals (quantiser sanity, 3 mantissa bits)
    assert np.abs(kv - k.double().numpy()).max() <= 0.0625 * np.abs(k.numpy()).max() + 1e-6
