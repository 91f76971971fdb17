"""Greedy layer selection (paper Alg. 1) with the surrogate loss, on the GPU against the oracle."""
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


def _stack(ic, cfg, n):
    """n layers whose indexer inputs drift from layer to layer (so that reuse costs grow with the
    layer distance) with independent attention inputs; returns device dicts and the host array."""
    ix = list(synth.chain_indexer_layers(cfg, n, device="cuda"))
    layers = []
    for l in range(n):
        d = dict(ix[l])
        d.update(synth.attn_layer(cfg, l, device="cuda"))
        layers.append(d)
    outs = [torch.empty((cfg["B"], cfg["Tq"], cfg["H_q"], cfg["d_v"]), dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    arr = ic.make_layers(layers, cfg["k_sel"], 0, cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg), outs)
    return layers, outs, arr


def _all_full_reference(ic, cfg, arr, outs, n):
    ws = torch.empty(max(ic.forward_stack_workspace(arr), 256), dtype=torch.uint8, device="cuda")
    cache = torch.empty((cfg["B"], cfg["Tq"], cfg["k_sel"]), dtype=torch.int32, device="cuda")
    ic.forward_stack(arr, [True] * n, cache, ws)
    torch.cuda.synchronize()
    return [o.clone() for o in outs], cache


def test_pattern_loss_matches_the_oracle(ic, oracle):
    cfg = synth.config("c0", Tq=192, Lk=192, k_sel=24)
    n = 5
    say("pattern loss, %d layers L=192 k=24" % n)
    layers, outs, arr = _stack(ic, cfg, n)
    ref, cache = _all_full_reference(ic, cfg, arr, outs, n)
    lb = [synth.bits_layer({k: v.cpu() for k, v in l.items()}) for l in layers]
    args = (cfg["k_sel"], 0, cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg))
    o_ref, _, _ = oracle.forward_stack(lb, [True] * n, *args)
    for mask in ([True] * n, [True, False, False, False, False], [True, False, True, False, False], [True, True, True, False, True]):
        got = float(ic.pattern_loss(arr, mask, ref, cache))
        want = oracle.pattern_loss_forward(lb, mask, *args, o_ref)
        say("mask %s: loss gpu %.6f oracle %.6f" % ("".join("FS"[not m] for m in mask), got, want))
        # bf16 outputs on the GPU side against fp64 ones: a few 1e-3 on a per-layer similarity
        assert abs(got - want) <= 3e-3
        if all(mask):
            assert abs(got) <= 1e-12                       # the same kernels, the same bits
    # the loss grows when a layer has to reach further back for its indices
    l1 = float(ic.pattern_loss(arr, [True, True, True, True, False], ref, cache))
    l3 = float(ic.pattern_loss(arr, [True, True, False, False, False], ref, cache))
    assert 0 < l1 < l3


@pytest.mark.parametrize("blocks", [1, 2])
def test_greedy_search_by_forward_passes(ic, oracle, blocks):
    """The search driven by real forward passes of the stack finds what the host search finds on the
    similarity matrix of the same stack (the layers' inputs are independent of earlier outputs), and
    what the oracle's Alg. 1 finds on the oracle's similarity matrix wherever the choice is clear."""
    cfg = synth.config("c0", Tq=128, Lk=128, k_sel=16)
    n, K = 6, 3
    say("greedy by forward passes, %d layers, %d blocks" % (n, blocks))
    layers, outs, arr = _stack(ic, cfg, n)
    ref, cache = _all_full_reference(ic, cfg, arr, outs, n)
    n0 = ic.debug_indexer_launch_count()
    mask, order, curve = ic.greedy_search_forward(arr, K, ref, cache, n_blocks=blocks)
    n_idx = ic.debug_indexer_launch_count() - n0
    say("forward search: order %s curve %s (%d indexer runs)" % (order, ["%.5f" % c for c in curve], n_idx))
    assert mask[0] and sum(not m for m in mask) == K and sorted(order) == [l for l in range(n) if not mask[l]]
    # the similarity matrix of the same stack, on the GPU, and the host search on it
    idxs = [ic.indexer_topk(l["q"], l["k"], l["w"], cfg["k_sel"], 0) for l in layers]
    S = ic.similarity_matrix(arr, idxs).cpu().numpy()
    m2, o2, c2 = ic.pattern_search_greedy(S, K, blocks)
    assert np.allclose(curve, c2, rtol=0, atol=1e-6)
    # every commit was the best candidate by a margin, or the two searches may differ in a near-tie
    f = lambda m: oracle.pattern_loss_from_similarity(S, m)
    clear = True
    m = [True] * n
    size = -(-n // blocks)
    for l in o2:
        blk = l // size
        cands = [c for c in range(size * blk + 1, min(size * (blk + 1), n)) if m[c]]
        vals = sorted(f([x and (i != c) for i, x in enumerate(m)]) for c in cands)
        clear &= len(vals) < 2 or vals[1] - vals[0] > 1e-5
        m[l] = False
    if clear:
        assert order == o2 and mask == m2
    # against the oracle end to end (fp64 attention): same pattern when the oracle's margins are clear
    lb = [synth.bits_layer({k: v.cpu() for k, v in l.items()}) for l in layers]
    So = oracle.similarity_matrix(lb, [i.cpu().numpy() for i in idxs], cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg))
    mo, oo, co = oracle.greedy_search(lambda mm: oracle.pattern_loss_from_similarity(So, mm), n, K, blocks)
    assert np.allclose(curve, co, rtol=0, atol=3e-3)
    say("oracle search: order %s curve %s" % (oo, ["%.5f" % c for c in co]))
