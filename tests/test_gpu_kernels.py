"""GPU parity: each HIP kernel against the CPU oracle on small seeded cases that still span
several tiles and ragged tails.  Everything goes through the C ABI (ctypes binding)."""
import math
import sys

import numpy as np
import pytest
import torch

import synth
from tests import parity

pytestmark = pytest.mark.gpu


def say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def ic():
    import paper_2603_12201_amd as m
    m.lib()
    assert torch.cuda.is_available()
    return m


def _mk_indexer(seed, B, Tq, Lk, H, d, signed_w=False):
    g = torch.Generator().manual_seed(seed)
    q = (torch.randn((B, Tq, H, d), generator=g) / math.sqrt(d)).to(torch.bfloat16)
    k = torch.randn((B, Lk, d), generator=g).to(torch.bfloat16)
    w = torch.rand((B, Tq, H), generator=g)
    if signed_w:
        w = w * 2 - 1
    return q, k, w.float()


SCORE_CASES = [
    # B, Tq, Lk, H, d, q_pos0, signed
    (1, 40, 40, 4, 64, 0, False),        # tiny config shape, ragged tail of a 16-token block
    (2, 37, 150, 32, 128, 113, False),   # chunked prefill: queries in the middle of the context
    (1, 130, 130, 32, 128, 0, True),     # signed head weights, several key tiles
    (2, 1, 300, 32, 128, 299, False),    # decode: one query row per sequence
    (1, 20, 90, 64, 128, 70, False),     # 64 heads (two head tiles)
    (1, 24, 24, 7, 64, 0, False),        # head count that is not a multiple of anything
    (1, 9, 50, 32, 128, 10, False),      # Lk caps the visible range (q_pos0 + i >= Lk)
    # long rows: the key loop runs its steady state (unmasked tiles, pipelined across tiles) before
    # the diagonal; ragged and whole last tiles, every kernel shape
    (1, 30, 1000, 32, 128, 970, True),
    (1, 30, 1024, 32, 128, 994, False),
    (2, 26, 900, 64, 128, 874, True),
    (1, 30, 777, 32, 64, 747, False),
    (1, 26, 840, 64, 64, 814, True),
    (1, 200, 200, 32, 128, 0, False),    # causal square: every wave has a different number of unmasked tiles
]


@pytest.mark.parametrize("case", SCORE_CASES)
def test_indexer_scores(ic, oracle, case):
    B, Tq, Lk, H, d, p0, signed = case
    say("scores B=%d Tq=%d Lk=%d H=%d d=%d q_pos0=%d signed=%s" % case)
    q, k, w = _mk_indexer(100 + Tq + H, B, Tq, Lk, H, d, signed)
    got = ic.debug_indexer_scores(q.cuda(), k.cuda(), w.cuda(), p0, 0, Tq)
    torch.cuda.synchronize()
    want = oracle.indexer_scores(synth.bits(q), synth.bits(k), synth.bits(w), p0)
    parity.check_scores(got.cpu().numpy(), want)


# Few query rows per sequence (decode): the ring form of the score kernel -- several slots per wave, more tokens
# than are in flight at once, two head tiles, a head count that leaves part of a head tile empty, rows that see
# only part of the cache, caches shorter than one slot.
FEW_ROW_CASES = [
    # B, Tq, Lk, H, d, q_pos0, signed
    (3, 1, 5000, 32, 128, 4999, True),
    (2, 4, 3000, 64, 128, 2996, True),
    (11, 2, 700, 17, 128, 698, False),
    (1, 3, 100, 32, 128, 50, False),
    (9, 1, 40000, 32, 128, 39999, True),
    (20, 1, 31, 32, 128, 30, False),
    (5, 2, 2049, 40, 128, 2047, True),
]


@pytest.mark.parametrize("case", FEW_ROW_CASES)
def test_indexer_scores_few_rows(ic, oracle, case):
    B, Tq, Lk, H, d, p0, signed = case
    say("scores few rows B=%d Tq=%d Lk=%d H=%d d=%d q_pos0=%d signed=%s" % case)
    q, k, w = _mk_indexer(300 + B + Lk, B, Tq, Lk, H, d, signed)
    got = ic.debug_indexer_scores(q.cuda(), k.cuda(), w.cuda(), p0, 0, Tq)
    torch.cuda.synchronize()
    want = oracle.indexer_scores(synth.bits(q), synth.bits(k), synth.bits(w), p0)
    parity.check_scores(got.cpu().numpy(), want)


def _sweep_cases(n, seed):
    """Seeded random shapes around the tile (64 keys) and block (8 / 12 tokens) boundaries of the score kernel."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        H, d = [(32, 128), (64, 128), (32, 64), (64, 64), (17, 128), (40, 64)][int(rng.integers(0, 6))]
        B = int(rng.integers(1, 3))
        Tq = int(rng.integers(1, 60))
        extra = int(rng.choice([0, 1, 63, 64, 65, 127, 128, 200, 513, 1000]))
        Lk = Tq + extra
        p0 = int(rng.choice([Lk - Tq, max(0, Lk - Tq - 7), Lk]))     # aligned to the end, short of it, past it
        out.append((B, Tq, Lk, H, d, p0, bool(rng.integers(0, 2))))
    return out


@pytest.mark.parametrize("case", _sweep_cases(24, 20260312))
def test_indexer_scores_shape_sweep(ic, oracle, case):
    B, Tq, Lk, H, d, p0, signed = case
    say("scores sweep B=%d Tq=%d Lk=%d H=%d d=%d q_pos0=%d signed=%s" % case)
    q, k, w = _mk_indexer(900 + Tq + Lk, B, Tq, Lk, H, d, signed)
    got = ic.debug_indexer_scores(q.cuda(), k.cuda(), w.cuda(), p0, 0, Tq)
    torch.cuda.synchronize()
    want = oracle.indexer_scores(synth.bits(q), synth.bits(k), synth.bits(w), p0)
    parity.check_scores(got.cpu().numpy(), want)


FP8_CASES = [
    # B, Tq, Lk, H, q_pos0
    (1, 70, 70, 64, 0),        # configs[4] head count: two head tiles
    (2, 30, 200, 32, 170),
    (2, 1, 300, 64, 299),      # decode form
    (1, 40, 40, 20, 0),        # ragged head count
    (1, 30, 1000, 32, 970),    # long rows: steady-state key loop, ragged last tile
    (2, 26, 905, 64, 879),
    (1, 150, 150, 64, 0),
]


def _mk_fp8(seed, B, Tq, Lk, H, d=128):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn((B, Tq, H * d), generator=g) / math.sqrt(d)
    k = torch.randn((B, Lk, d), generator=g)
    w = torch.rand((B, Tq, H), generator=g)
    q8, qs = synth.quantize_e4m3(q)
    k8, ks = synth.quantize_e4m3(k)
    return q8.reshape(B, Tq, H, d).contiguous(), k8.contiguous(), w.float(), qs.contiguous(), ks.contiguous()


@pytest.mark.parametrize("case", FP8_CASES)
def test_indexer_scores_fp8(ic, oracle, case):
    B, Tq, Lk, H, p0 = case
    say("fp8 scores B=%d Tq=%d Lk=%d H=%d q_pos0=%d" % case)
    q8, k8, w, qs, ks = _mk_fp8(500 + Tq + H, B, Tq, Lk, H)
    got = ic.debug_indexer_scores(q8.cuda(), k8.cuda(), w.cuda(), p0, 0, Tq, q_scale=qs.cuda(), k_scale=ks.cuda())
    torch.cuda.synchronize()
    want = oracle.indexer_scores(synth.bits(q8), synth.bits(k8), synth.bits(w), p0, dtype=oracle.FP8_E4M3,
                                 q_scale=synth.bits(qs), k_scale=synth.bits(ks))
    parity.check_scores(got.cpu().numpy(), want)


def test_indexer_topk_fp8(ic, oracle):
    B, Tq, Lk, H, p0, ksel = 1, 48, 600, 64, 552, 128
    say("fp8 topk")
    q8, k8, w, qs, ks = _mk_fp8(77, B, Tq, Lk, H)
    idx = ic.indexer_topk(q8.cuda(), k8.cuda(), w.cuda(), ksel, p0, q_scale=qs.cuda(), k_scale=ks.cuda())
    torch.cuda.synchronize()
    sc = oracle.indexer_scores(synth.bits(q8), synth.bits(k8), synth.bits(w), p0, dtype=oracle.FP8_E4M3,
                               q_scale=synth.bits(qs), k_scale=synth.bits(ks))
    g = idx.cpu().numpy()
    for i in range(Tq):
        parity.check_idx_row(g[0, i], sc[0, i], min(Lk, p0 + i + 1), ksel, oracle)


def test_fp8_exact_on_power_of_two_inputs(ic, oracle):
    # every e4m3 value and product is exact in fp32; with power-of-two inputs and scales the sums
    # are exact too, so GPU and oracle must agree to the last bit
    say("fp8 exact")
    B, Tq, Lk, H, d = 1, 33, 33, 32, 128
    g = torch.Generator().manual_seed(3)
    q = torch.randint(-2, 3, (B, Tq, H, d), generator=g).float()
    k = torch.randint(-2, 3, (B, Lk, d), generator=g).float()
    w = torch.randint(0, 4, (B, Tq, H), generator=g).float() * 0.25
    qs = torch.full((B, Tq), 0.5)
    ks = torch.full((B, Lk), 2.0)
    q8, k8 = q.to(torch.float8_e4m3fn), k.to(torch.float8_e4m3fn)
    got = ic.debug_indexer_scores(q8.cuda(), k8.cuda(), w.cuda(), 0, 0, Tq, q_scale=qs.cuda(), k_scale=ks.cuda())
    want = oracle.indexer_scores(synth.bits(q8), synth.bits(k8), synth.bits(w), 0, dtype=oracle.FP8_E4M3,
                                 q_scale=synth.bits(qs), k_scale=synth.bits(ks))
    got = got.cpu().numpy().astype(np.float64)
    vis = np.isfinite(want)
    assert np.array_equal(got[vis], want[vis])


def test_indexer_scores_row_window(ic, oracle):
    say("scores row window")
    B, Tq, Lk, H, d, p0 = 1, 100, 100, 32, 128, 0
    q, k, w = _mk_indexer(7, B, Tq, Lk, H, d)
    got = ic.debug_indexer_scores(q.cuda(), k.cuda(), w.cuda(), p0, 33, 21)
    torch.cuda.synchronize()
    want = oracle.indexer_scores(synth.bits(q), synth.bits(k), synth.bits(w), p0, rows=list(range(33, 54)))
    parity.check_scores(got.cpu().numpy(), want)


TOPK_CASES = [
    # B, Tq, Lk, H, d, q_pos0, k_sel
    (1, 200, 200, 4, 64, 0, 64),         # tiny-config shape: zero-score ties at the boundary
    (2, 50, 400, 32, 128, 350, 128),
    (1, 70, 70, 32, 128, 0, 128),        # every row shorter than k: all positions selected
    (2, 1, 1000, 32, 128, 999, 256),     # decode
    (1, 33, 9000, 32, 128, 8967, 2048),  # long rows: 1024-thread select, LDS-cached row
    (1, 40, 300, 64, 128, 260, 1),       # k = 1: argmax
    (2, 2, 40000, 32, 128, 39998, 512),  # rows of 16385 keys and more: sampled threshold + candidate list
    (1, 3, 100000, 32, 128, 99997, 2048),  # rows past 65536 keys: sampled threshold + candidate list, one read of the row
    (1, 3, 16400, 32, 128, 16397, 2048),   # just past the candidate form's lower limit
    (1, 40, 16420, 32, 128, 16380, 512),   # a candidate-form launch whose first rows are too short for it (generic form inside)
    (1, 1, 140000, 32, 128, 139999, 2048), # beyond the candidate form's bitmap: the radix select streaming the row
    (1, 4, 25000, 32, 128, 24996, 2048),   # the candidate form's half-size instance (rows of 16385 to 32768 keys)
    (1, 3, 32769, 32, 128, 32766, 2048),   # its last two rows, and the first one past it in a launch of the full-size instance
    (1, 2, 32768, 32, 128, 32766, 1024),   # a launch that ends exactly at its limit
]


@pytest.mark.parametrize("case", TOPK_CASES)
def test_indexer_topk(ic, oracle, case):
    B, Tq, Lk, H, d, p0, ks = case
    say("topk B=%d Tq=%d Lk=%d H=%d d=%d q_pos0=%d k=%d" % case)
    q, k, w = _mk_indexer(200 + Tq + ks, B, Tq, Lk, H, d)
    idx, sel = ic.indexer_topk(q.cuda(), k.cuda(), w.cuda(), ks, p0, want_scores=True)
    torch.cuda.synchronize()
    idx, sel = idx.cpu().numpy(), sel.cpu().numpy()
    sc = oracle.indexer_scores(synth.bits(q), synth.bits(k), synth.bits(w), p0)
    kinds = {}
    for b in range(B):
        for i in range(Tq):
            nv = max(0, min(Lk, p0 + i + 1))
            kind = parity.check_idx_row(idx[b, i], sc[b, i], nv, ks, oracle)
            kinds[kind] = kinds.get(kind, 0) + 1
            n = min(nv, ks)
            want_sel = sc[b, i][idx[b, i, :n]]
            parity.check_scores(sel[b, i, :n][None], want_sel[None])
            assert np.all(np.isneginf(sel[b, i, n:]))
    say("row kinds: %s" % kinds)


def test_topk_tie_break_on_equal_scores(ic, oracle):
    # w = 0 makes every score exactly 0: the k lowest positions must win, on every row
    say("topk all-equal rows")
    B, Tq, Lk, H, d, ks = 1, 300, 300, 32, 128, 64
    q, k, w = _mk_indexer(5, B, Tq, Lk, H, d)
    w.zero_()
    idx = ic.indexer_topk(q.cuda(), k.cuda(), w.cuda(), ks, 0).cpu().numpy()
    for i in range(Tq):
        n = min(i + 1, ks)
        assert np.array_equal(idx[0, i, :n], np.arange(n))
        assert np.all(idx[0, i, n:] == -1)


@pytest.mark.parametrize("Lk", [3000, 9000, 25000, 40000, 70000])
def test_topk_ties_cut_at_the_boundary_on_long_rows(ic, oracle, Lk):
    # one head, one-hot q, keys from a handful of small integers: scores are exact on both sides
    # and fall into a few large tie classes, so the k-th score has far more ties than fit and the
    # lowest positions among them must win; every select variant (by row length) is covered
    say("topk tie classes, Lk=%d" % Lk)
    B, Tq, H, d, ks = 1, 3, 1, 64, 256
    g = torch.Generator().manual_seed(Lk)
    q = torch.zeros((B, Tq, H, d)); q[..., 3] = 1.0
    k = torch.zeros((B, Lk, d)); k[0, :, 3] = torch.randint(0, 8, (Lk,), generator=g).float()
    w = torch.ones((B, Tq, H))
    p0 = Lk - Tq
    idx = ic.indexer_topk(q.bfloat16().cuda(), k.bfloat16().cuda(), w.cuda(), ks, p0).cpu().numpy()
    sc = oracle.indexer_scores(synth.bits(q.bfloat16()), synth.bits(k.bfloat16()), synth.bits(w), p0)
    vals = k[0, :, 3].numpy()
    for i in range(Tq):
        nv = p0 + i + 1
        assert parity.check_idx_row(idx[0, i], sc[0, i], nv, ks, oracle) == "tie"
        # by hand: all 7s come first in position order; there are more of them than k
        want = np.nonzero(vals[:nv] == 7)[0][:ks]
        assert want.size == ks and np.array_equal(idx[0, i], want)


@pytest.mark.parametrize("Lk", [100000, 30000])
def test_topk_candidate_form_with_ties_at_the_boundary(ic, oracle, Lk):
    # candidate form (both of its instances, by row length): two one-hot heads with weights 1 and 1/256 and integer
    # key coordinates below 256 give 65536 exactly representable score levels, so small tie classes sit everywhere,
    # the boundary included: the exact ranking of the boundary bin decides
    say("topk candidate form, ties at the boundary, Lk=%d" % Lk)
    B, Tq, H, d, ks = 1, 4, 2, 64, 2048
    g = torch.Generator().manual_seed(99)
    q = torch.zeros((B, Tq, H, d)); q[:, :, 0, 3] = 1.0; q[:, :, 1, 5] = 1.0
    k = torch.zeros((B, Lk, d))
    k[0, :, 3] = torch.randint(0, 256, (Lk,), generator=g).float()
    k[0, :, 5] = torch.randint(0, 256, (Lk,), generator=g).float()
    w = torch.zeros((B, Tq, H)); w[..., 0] = 1.0; w[..., 1] = 1.0 / 256.0
    p0 = Lk - Tq
    idx, sel = ic.indexer_topk(q.bfloat16().cuda(), k.bfloat16().cuda(), w.cuda(), ks, p0, want_scores=True)
    idx, sel = idx.cpu().numpy(), sel.cpu().numpy()
    sc = oracle.indexer_scores(synth.bits(q.bfloat16()), synth.bits(k.bfloat16()), synth.bits(w), p0)
    kinds = {}
    for i in range(Tq):
        kind = parity.check_idx_row(idx[0, i], sc[0, i], p0 + i + 1, ks, oracle)
        kinds[kind] = kinds.get(kind, 0) + 1
        assert np.array_equal(sel[0, i].astype(np.float64), sc[0, i][idx[0, i]])       # exact scores on both sides
        r = oracle.topk_row(sc[0, i], p0 + i + 1, ks)
        assert np.array_equal(idx[0, i], np.sort(r["idx"]))                            # the oracle's set, ties and all
    say("row kinds: %s" % kinds)


@pytest.mark.parametrize("Lk", [70000, 140000])
def test_topk_tie_class_beyond_65535_entries(ic, oracle, Lk):
    # rows longer than 65536 keys take the select form that streams the row: there the tie class of the
    # k-th score can hold more than 65535 entries.  (a) every score equal (w = 0): the k lowest positions
    # win; (b) 100 larger scores spread over the row, everything else one tie class: the 100 plus the
    # first k - 100 positions of the class, in position order
    say("topk tie class beyond 65535 entries, Lk=%d" % Lk)
    B, Tq, H, d, ks = 1, 2, 1, 64, 256
    p0 = Lk - Tq
    q = torch.zeros((B, Tq, H, d)); q[..., 3] = 1.0
    g = torch.Generator().manual_seed(Lk + 7)
    vals = torch.full((Lk,), 7.0)
    big = torch.randperm(p0, generator=g)[:100]
    vals[big] = 9.0
    k = torch.zeros((B, Lk, d)); k[0, :, 3] = vals
    w = torch.ones((B, Tq, H))
    zero_w = torch.zeros((B, Tq, H))
    idx0 = ic.indexer_topk(q.bfloat16().cuda(), k.bfloat16().cuda(), zero_w.cuda(), ks, p0).cpu().numpy()
    for i in range(Tq):
        assert np.array_equal(idx0[0, i], np.arange(ks)), "all-equal row: the k lowest positions must win"
    idx = ic.indexer_topk(q.bfloat16().cuda(), k.bfloat16().cuda(), w.cuda(), ks, p0).cpu().numpy()
    sc = oracle.indexer_scores(synth.bits(q.bfloat16()), synth.bits(k.bfloat16()), synth.bits(w), p0)
    v = vals.numpy()
    for i in range(Tq):
        nv = p0 + i + 1
        assert parity.check_idx_row(idx[0, i], sc[0, i], nv, ks, oracle) == "tie"
        sevens = np.nonzero(v[:nv] == 7.0)[0][:ks - 100]
        want = np.sort(np.concatenate([np.sort(big.numpy()), sevens]))
        assert np.array_equal(idx[0, i], want)


@pytest.mark.parametrize("Lk", [3000, 9000, 25000, 40000, 70000])
def test_topk_boundary_bin_fully_selected(ic, oracle, Lk):
    # exactly k winners, all inside one bin of the first radix digit ([64, 72): sixteen bf16 values),
    # everything else far below: the digit sweeps may stop after the first one, and "selected" becomes
    # key >= the bin's lower edge, in every select variant (by row length)
    say("topk winners fill the boundary bin, Lk=%d" % Lk)
    B, Tq, H, d, ks = 1, 3, 1, 64, 256
    g = torch.Generator().manual_seed(Lk + 1)
    p0 = Lk - Tq
    vals = torch.randint(0, 32, (Lk,), generator=g).float() / 4.0            # losers: [0, 8)
    win = torch.randperm(p0, generator=g)[:ks]                                # winners visible to every row
    vals[win] = 64.0 + torch.randint(0, 16, (ks,), generator=g).float() / 2.0
    q = torch.zeros((B, Tq, H, d)); q[..., 3] = 1.0
    k = torch.zeros((B, Lk, d)); k[0, :, 3] = vals
    w = torch.ones((B, Tq, H))
    idx = ic.indexer_topk(q.bfloat16().cuda(), k.bfloat16().cuda(), w.cuda(), ks, p0).cpu().numpy()
    want = np.sort(win.numpy())
    for i in range(Tq):
        assert np.array_equal(idx[0, i], want)


def test_topk_monotone_scores(ic, oracle):
    # one head, one-hot q, keys increasing along that coordinate: scores increase with position,
    # so the last k visible positions win (the adversarial order for a streaming filter)
    say("topk monotone rows")
    B, Tq, Lk, H, d, ks = 1, 500, 500, 1, 64, 32
    q = torch.zeros((B, Tq, H, d)); q[..., 3] = 1.0
    k = torch.zeros((B, Lk, d)); k[0, :, 3] = torch.arange(Lk, dtype=torch.float32) / 4.0
    w = torch.ones((B, Tq, H))
    idx = ic.indexer_topk(q.bfloat16().cuda(), k.bfloat16().cuda(), w.cuda(), ks, 0).cpu().numpy()
    kb = k.bfloat16().float()[0, :, 3].numpy()
    assert np.all(np.diff(kb) >= 0)
    sc = oracle.indexer_scores(synth.bits(q.bfloat16()), synth.bits(k.bfloat16()), synth.bits(w), 0)
    for i in range(Tq):
        parity.check_idx_row(idx[0, i], sc[0, i], i + 1, ks, oracle)


def _mk_attn(seed, B, Tq, Lk, Hq, d_qk, row):
    g = torch.Generator().manual_seed(seed)
    Q = torch.randn((B, Tq, Hq, d_qk), generator=g).to(torch.bfloat16)
    KV = torch.randn((B, Lk, row), generator=g).to(torch.bfloat16)
    return Q, KV


def _rand_idx(seed, B, Tq, Lk, ks, p0, holes=False):
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


ATTN_CASES = [
    # B, Tq, Lk, Hq, d_qk, d_v, v_off, row, k_sel, q_pos0, holes
    (1, 300, 300, 4, 64, 64, 64, 128, 64, 0, False),     # tiny-config layout [K | V]
    (1, 260, 260, 32, 576, 512, 0, 576, 128, 0, False),  # MLA row, one workgroup per query
    (2, 3, 500, 32, 576, 512, 0, 576, 256, 497, False),  # few queries: split path + merge kernel
    (1, 20, 400, 20, 576, 512, 0, 576, 200, 380, True),  # ragged heads, ragged k_sel, holes in idx
    (2, 5, 90, 16, 64, 64, 64, 128, 70, 85, True),
    # 512 or more queries: one workgroup per query over 64-row tiles (the prefill form)
    (1, 600, 700, 32, 576, 512, 0, 576, 200, 100, True),  # ragged last tile, holes in idx
    (2, 300, 400, 20, 576, 512, 0, 576, 130, 150, True),  # ragged heads
    (1, 520, 520, 32, 576, 512, 0, 640, 64, 0, False),    # padded KV rows, one tile, short causal rows
    (1, 512, 300, 32, 576, 512, 0, 576, 2, 40, False),    # two slots only
    # whole selections of three or more tiles out of a dense MLA cache (the chained row-slab form)
    (1, 300, 3000, 32, 576, 512, 0, 576, 2048, 2700, False),  # 32 tiles; 44 workgroups walk two queries
    (2, 200, 500, 32, 576, 512, 0, 576, 192, 300, True),      # exactly three tiles, two sequences, holes
    (1, 700, 900, 32, 576, 512, 0, 576, 129, 200, False),     # one slot in the third tile; chains of three queries
    (1, 290, 400, 7, 576, 512, 0, 608, 333, 110, True),       # ragged heads, padded KV rows, ragged last tile
]


@pytest.mark.parametrize("case", ATTN_CASES)
def test_sparse_attn(ic, oracle, case):
    B, Tq, Lk, Hq, d_qk, d_v, v_off, row, ks, p0, holes = case
    say("attn B=%d Tq=%d Lk=%d Hq=%d dqk=%d dv=%d voff=%d row=%d k=%d p0=%d holes=%s" % case)
    Q, KV = _mk_attn(300 + Tq + ks, B, Tq, Lk, Hq, d_qk, row)
    idx = _rand_idx(400 + Tq, B, Tq, Lk, ks, p0, holes)
    scale = 1.0 / math.sqrt(d_qk)
    O, lse = ic.sparse_attn(Q.cuda(), KV.cuda(), torch.from_numpy(idx).cuda(), d_v, v_off, scale, want_lse=True)
    torch.cuda.synchronize()
    want, want_lse = oracle.sparse_attn(synth.bits(Q), synth.bits(KV), idx, d_v, v_off, scale)
    err = parity.check_attn(O.float().cpu().numpy(), want)
    say("max abs err %.4g" % err)
    assert np.allclose(lse.cpu().numpy(), want_lse, rtol=0, atol=2e-2)


@pytest.mark.parametrize("Tq", [4, 512])
def test_sparse_attn_empty_rows_and_out_of_range(ic, oracle, Tq):
    say("attn empty rows / out-of-range entries, Tq=%d" % Tq)
    B, Lk, Hq, d_qk, d_v, row, ks = 1, 50, 32, 576, 512, 576, 64
    Q, KV = _mk_attn(9, B, Tq, Lk, Hq, d_qk, row)
    idx = np.full((B, Tq, ks), -1, dtype=np.int32)
    idx[0, 1, :5] = [3, 7, 9, 11, 49]
    idx[0, 2, 10] = 20
    idx[0, 3, :3] = [1, 1000, 2]           # 1000 >= Lk must be skipped, not read
    scale = 1.0 / 24.0
    O, lse = ic.sparse_attn(Q.cuda(), KV.cuda(), torch.from_numpy(idx).cuda(), d_v, 0, scale, want_lse=True)
    torch.cuda.synchronize()
    idx_o = idx.copy(); idx_o[idx_o >= Lk] = -1
    want, want_lse = oracle.sparse_attn(synth.bits(Q), synth.bits(KV), idx_o, d_v, 0, scale)
    parity.check_attn(O.float().cpu().numpy(), want)
    assert np.all(O[0, 0].float().cpu().numpy() == 0)
    assert np.all(np.isneginf(lse[0, 0].cpu().numpy()))
    assert np.allclose(lse[0, 1:].cpu().numpy(), want_lse[0, 1:], atol=2e-2)


def test_calibration_kernels_run_on_small_inputs(ic):
    # measurement aids, no numerical result: every kind launches, stays inside its buffers (out-of-table and negative row
    # numbers are clamped) and leaves the stream usable
    say("calibration kernels")
    src = torch.arange(1 << 20, dtype=torch.int32, device="cuda").view(torch.uint8)
    dst = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    ic.calibrate(ic.CALIB_READ, src, dst, n=src.numel(), wgs=64)
    ic.calibrate(ic.CALIB_COPY, src, dst, n=dst.numel(), wgs=64)
    torch.cuda.synchronize()
    assert torch.equal(dst, src[:dst.numel()])
    table = torch.zeros((300, 1152), dtype=torch.uint8, device="cuda")
    rows = torch.randint(-5, 400, (64 * 9,), generator=torch.Generator().manual_seed(3)).to(torch.int32).cuda()
    scratch = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    for kind in (ic.CALIB_GATHER, ic.CALIB_TILE_GATHER, ic.CALIB_TILE_STORE, ic.CALIB_TILE_READ, ic.CALIB_TILE_READ2,
                 ic.CALIB_TILE_8WAVES, ic.CALIB_TILE_INTERLEAVED):
        ic.calibrate(kind, table, scratch, idx=rows, n=rows.numel(), table_rows=table.shape[0], row_bytes=1152, wgs=4)
    for kind in (ic.CALIB_MFMA_BF16, ic.CALIB_MFMA_FP8, ic.CALIB_LDS_READ16_PADDED, ic.CALIB_LDS_READ16_SWIZZLED,
                 ic.CALIB_LDS_TR8_ROWS2, ic.CALIB_LDS_TR8_ROWS1):
        ic.calibrate(kind, None, scratch, n=10, wgs=4)
    torch.cuda.synchronize()
    assert int(scratch.sum().item()) == 0          # the "rarely written" outputs were not written

