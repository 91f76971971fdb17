"""GPU parity on the workload configurations: the whole tiny stack element by element, and the
full-size configurations (launched exactly as bench.py launches them) on sampled query rows the
oracle can compute one by one."""
import os
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


def _cuda(layer):
    return {k: v.cuda() for k, v in layer.items()}


def _run_stack(ic, cfg, layers_gpu, mask):
    B, Tq, ks = cfg["B"], cfg["Tq"], cfg["k_sel"]
    outs = [torch.empty((B, Tq, cfg["H_q"], cfg["d_v"]), dtype=torch.bfloat16, device="cuda") for _ in layers_gpu]
    arr = ic.make_layers(layers_gpu, ks, cfg["q_pos0"], cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg), outs)
    ws = torch.empty(max(ic.forward_stack_workspace(arr), 256), dtype=torch.uint8, device="cuda")
    idx_cache = torch.full((B, Tq, ks), -7, dtype=torch.int32, device="cuda")
    n0 = ic.debug_indexer_launch_count()
    ic.forward_stack(arr, mask, idx_cache, ws)
    torch.cuda.synchronize()
    return outs, idx_cache, ic.debug_indexer_launch_count() - n0


def test_tiny_stack_full_parity(ic, oracle):
    """configs[0]: L=512, 4 layers FSFS, every index row and every output element."""
    cfg = synth.config("c0")
    say("tiny stack %s" % cfg["pattern"])
    layers = synth.stack_layers(cfg)
    lg = [_cuda(l) for l in layers]
    mask = ic.pattern_from_string(cfg["pattern"])
    outs, idx_cache, n_idx = _run_stack(ic, cfg, lg, mask)
    assert n_idx == sum(mask)                                   # the indexer ran on Full layers only
    lb = [synth.bits_layer(l) for l in layers]
    o_outs, o_used, o_n = oracle.forward_stack(lb, mask, cfg["k_sel"], 0, cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg))
    assert o_n == n_idx
    # indices of each Full layer, through the same entry point the stack uses
    gpu_idx = {}
    for l in range(cfg["n_layers"]):
        if mask[l]:
            gpu_idx[l] = ic.indexer_topk(lg[l]["q"], lg[l]["k"], lg[l]["w"], cfg["k_sel"], 0)
    torch.cuda.synchronize()
    assert torch.equal(idx_cache, gpu_idx[2])                   # cache holds the LAST Full layer's indices
    kinds = {}
    for l, gi in gpu_idx.items():
        sc = oracle.indexer_scores(lb[l]["q"], lb[l]["k"], lb[l]["w"], 0)
        g = gi.cpu().numpy()
        for t in range(cfg["Tq"]):
            kind = parity.check_idx_row(g[0, t], sc[0, t], t + 1, cfg["k_sel"], oracle)
            kinds[kind] = kinds.get(kind, 0) + 1
    say("row kinds %s" % kinds)
    assert kinds.get("tie", 0) + kinds.get("exact", 0) > 0
    worst = 0.0
    for l in range(cfg["n_layers"]):
        f = oracle.source_layer(mask, l)
        # a Shared layer's output is bit-identical to attention run with its Full layer's indices
        again = ic.sparse_attn(lg[l]["Q"], lg[l]["KV"], gpu_idx[f], cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg))
        torch.cuda.synchronize()
        assert torch.equal(again, outs[l])
        # attention parity proper: oracle attention over the indices the GPU selected ...
        want, _ = oracle.sparse_attn(lb[l]["Q"], lb[l]["KV"], gpu_idx[f].cpu().numpy(), cfg["d_v"], cfg["v_off"],
                                     synth.sm_scale(cfg))
        worst = max(worst, parity.check_attn(outs[l].float().cpu().numpy(), want))
        # ... and end to end against the oracle's own stack wherever both chose the same set
        same = np.all(np.sort(o_used[l], axis=-1) == np.sort(gpu_idx[f].cpu().numpy(), axis=-1), axis=-1)[0]
        assert same.mean() > 0.9
        parity.check_attn(outs[l].float().cpu().numpy()[0, same], o_outs[l][0, same])
    say("worst attention error %.4g" % worst)


def test_all_full_mask_and_irregular_patterns(ic, oracle):
    """All-ones mask = standard DSA; the paper's searched 47-layer patterns drive the loop."""
    cfg = synth.config("c0", Tq=96, Lk=96, k_sel=16, n_layers=47)
    base = [_cuda(l) for l in synth.stack_layers(cfg, n_layers=3)]
    lg = [base[l % 3] for l in range(47)]
    pats = []
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "searched_patterns.txt")):
        if line.startswith("dsa30b"):
            pats.append(line.split()[2])
    pats.append("F" * 47)
    for pat in pats:
        say("pattern %s" % pat)
        mask = ic.pattern_from_string(pat)
        outs, idx_cache, n_idx = _run_stack(ic, cfg, lg, mask)
        assert n_idx == pat.count("F")
        last_f = max(l for l in range(47) if mask[l])
        want_idx = ic.indexer_topk(lg[last_f]["q"], lg[last_f]["k"], lg[last_f]["w"], cfg["k_sel"], 0)
        torch.cuda.synchronize()
        assert torch.equal(idx_cache, want_idx)
        for l in (1, 8, 30, 46):
            f = oracle.source_layer(mask, l)
            fi = ic.indexer_topk(lg[f]["q"], lg[f]["k"], lg[f]["w"], cfg["k_sel"], 0)
            again = ic.sparse_attn(lg[l]["Q"], lg[l]["KV"], fi, cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg))
            torch.cuda.synchronize()
            assert torch.equal(again, outs[l])


def _sample_rows(Tq, k_sel, n, seed):
    """n query rows: an even stride over the whole range plus the rows where something changes (the first
    rows, the rows around k_sel where the select starts to cut, the first and last query each workgroup
    of the chained attention kernel walks (rounds of 256 queries), the last rows) and a few random ones."""
    rng = np.random.default_rng(seed)
    fixed = [0, 1, k_sel - 2, k_sel - 1, k_sel, k_sel + 1, 255, 256, 257, Tq // 2, Tq - 257, Tq - 256, Tq - 255,
             Tq - 2, Tq - 1]
    rows = set(r for r in fixed if 0 <= r < Tq)
    stride = max(1, Tq // max(1, n - len(rows) - 8))
    rows.update(range(stride // 2, Tq, stride))
    while len(rows) < n:
        rows.add(int(rng.integers(0, Tq)))
    return sorted(rows)


def _check_indexer_rows(ic, oracle, cfg, layer_gpu, idx_gpu, sel_gpu, rows, b=0):
    lb = {k: synth.bits(v[b:b + 1]) for k, v in layer_gpu.items() if k in ("q", "k", "w", "q_scale", "k_scale")}
    if cfg["dtype"] == "fp8":
        sc = oracle.indexer_scores(lb["q"], lb["k"], lb["w"], cfg["q_pos0"], dtype=oracle.FP8_E4M3,
                                   q_scale=lb["q_scale"], k_scale=lb["k_scale"], rows=rows)
    else:
        sc = oracle.indexer_scores(lb["q"], lb["k"], lb["w"], cfg["q_pos0"], rows=rows)
    g = idx_gpu[b].cpu().numpy()
    kinds = {}
    for j, t in enumerate(rows):
        nv = max(0, min(cfg["Lk"], cfg["q_pos0"] + t + 1))
        kind = parity.check_idx_row(g[t], sc[0, j], nv, cfg["k_sel"], oracle)
        kinds[kind] = kinds.get(kind, 0) + 1
        if sel_gpu is not None:
            n = min(nv, cfg["k_sel"])
            parity.check_scores(sel_gpu[b, t, :n].cpu().numpy()[None], sc[0, j][g[t, :n]][None])
    return kinds


def test_indexer_topk_prefill_16k_sampled(ic, oracle):
    """configs[1]: L=16384, H_I=32, d_I=128, k=2048, launched at full size."""
    cfg = synth.config("c1")
    say("c1 full-size indexer+topk")
    lay = synth.indexer_layer(cfg, 0, device="cuda")
    idx, sel = ic.indexer_topk(lay["q"], lay["k"], lay["w"], cfg["k_sel"], 0, want_scores=True)
    torch.cuda.synchronize()
    # properties that hold on every row
    valid = idx >= 0
    n_valid = valid.sum(-1)[0].cpu().numpy()
    assert np.array_equal(n_valid, np.minimum(np.arange(cfg["Tq"]) + 1, cfg["k_sel"]))
    pos = torch.arange(cfg["Tq"], device="cuda")[None, :, None]
    assert bool(((idx <= pos) | ~valid).all())
    d = idx[..., 1:] - idx[..., :-1]
    assert bool(((d > 0) | ~valid[..., 1:]).all())
    rows = _sample_rows(cfg["Tq"], cfg["k_sel"], 256, 1)
    kinds = _check_indexer_rows(ic, oracle, cfg, lay, idx, sel, rows)
    say("%d rows, kinds %s" % (len(rows), kinds))


def test_decode_step_sampled(ic, oracle):
    """configs[2]: batch 32, context 65536, one new token, 4 layers FSSS, launched at full size."""
    cfg = synth.config("c2")
    say("c2 decode step")
    layers = synth.stack_layers(cfg, device="cuda")
    mask = ic.pattern_from_string(cfg["pattern"])
    outs, idx_cache, n_idx = _run_stack(ic, cfg, layers, mask)
    assert n_idx == 1
    idx0, sel0 = ic.indexer_topk(layers[0]["q"], layers[0]["k"], layers[0]["w"], cfg["k_sel"], cfg["q_pos0"],
                                 want_scores=True)
    torch.cuda.synchronize()
    assert torch.equal(idx0, idx_cache)
    for b in (0, 13, 31):
        kinds = _check_indexer_rows(ic, oracle, cfg, layers[0], idx0, sel0, [0], b=b)
        say("seq %d kinds %s" % (b, kinds))
        for l in (0, 3):
            Qb, KVb = synth.bits(layers[l]["Q"][b:b + 1]), synth.bits(layers[l]["KV"][b:b + 1])
            want, _ = oracle.sparse_attn(Qb, KVb, idx0[b:b + 1].cpu().numpy(), cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg))
            err = parity.check_attn(outs[l][b:b + 1].float().cpu().numpy(), want)
            say("seq %d layer %d attention err %.4g" % (b, l, err))


def test_prefill_32k_layer_sampled(ic, oracle):
    """configs[3], one Full layer at full size (L=32768): sampled rows of idx and of O."""
    cfg = synth.config("c3")
    say("c3 one layer at L=32768")
    lay = synth.stack_layers(cfg, device="cuda", n_layers=1)[0]
    mask = [True]
    outs, idx_cache, n_idx = _run_stack(ic, cfg, [lay], mask)
    rows = _sample_rows(cfg["Tq"], cfg["k_sel"], 256, 3)
    # the selected scores come from the indexer entry point called on its own; its indices must be the
    # ones the stack cached
    idx1, sel1 = ic.indexer_topk(lay["q"], lay["k"], lay["w"], cfg["k_sel"], 0, want_scores=True)
    torch.cuda.synchronize()
    assert torch.equal(idx1, idx_cache)
    kinds = _check_indexer_rows(ic, oracle, cfg, lay, idx_cache, sel1, rows)
    del idx1, sel1
    say("%d rows, kinds %s" % (len(rows), kinds))
    Qb, KVb = synth.bits(lay["Q"]), synth.bits(lay["KV"])
    idx_rows = np.ascontiguousarray(idx_cache[:, rows].cpu().numpy())
    want, _ = oracle.sparse_attn(Qb, KVb, idx_rows, cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg), rows=rows,
                                 idx_is_subset=True)
    err = parity.check_attn(outs[0][:, rows].float().cpu().numpy(), want)
    say("attention err %.4g" % err)


@pytest.mark.parametrize("half", [0, 1])
def test_fp8_long_context_layer_sampled(ic, oracle, half):
    """configs[4], one Full layer at full size (L=131072, 64 fp8 heads): sampled rows of idx and O.  The 256 sampled
    rows are checked in two halves (every other row each): the oracle needs about half a second per row here."""
    cfg = synth.config("c4")
    say("c4 one fp8 layer at L=131072, rows %d of every 2" % half)
    lay = synth.stack_layers(cfg, device="cuda", n_layers=1)[0]
    torch.cuda.synchronize()
    outs, idx_cache, n_idx = _run_stack(ic, cfg, [lay], [True])
    assert n_idx == 1
    rows = _sample_rows(cfg["Tq"], cfg["k_sel"], 256, 5)[half::2]
    kinds = _check_indexer_rows(ic, oracle, cfg, lay, idx_cache, None, rows)
    say("%d rows, kinds %s" % (len(rows), kinds))
    Qb, KVb = synth.bits(lay["Q"][:, rows]), synth.bits(lay["KV"])
    idx_rows = np.ascontiguousarray(idx_cache[:, rows].cpu().numpy())
    # Q rows were gathered: address them as rows 0..n-1 of a compact Q
    want, _ = oracle.sparse_attn(Qb, KVb, idx_rows, cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg))
    err = parity.check_attn(outs[0][:, rows].float().cpu().numpy(), want)
    say("attention err %.4g" % err)


def test_prefill_stack_rows_with_fewer_than_k_entries(ic, oracle):
    """A prefill from position 0 through the stack: the first k_sel - 1 rows hold fewer than k_sel entries, and the
    chained attention kernel leaves the tiles behind their last entry out.  Every row of the first layer and of a
    Shared layer against the oracle, and against the stand-alone launch that knows nothing of the rows' lengths."""
    cfg = synth.config("c3", Tq=1024, Lk=1024, k_sel=512, n_layers=2)
    say("prefill stack L=1024 k=512: short rows")
    layers = synth.stack_layers(cfg, device="cuda")
    mask = ic.pattern_from_string("FS")
    outs, idx_cache, n_idx = _run_stack(ic, cfg, layers, mask)
    assert n_idx == 1
    g = idx_cache.cpu().numpy()
    assert np.all(g[0, 10, 11:] == -1) and np.all(g[0, 10, :11] == np.arange(11))
    for l in range(2):
        want, _ = oracle.sparse_attn(synth.bits(layers[l]["Q"]), synth.bits(layers[l]["KV"]), g, cfg["d_v"], cfg["v_off"],
                                     synth.sm_scale(cfg))
        err = parity.check_attn(outs[l].float().cpu().numpy(), want)
        alone = ic.sparse_attn(layers[l]["Q"], layers[l]["KV"], idx_cache, cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg))
        torch.cuda.synchronize()
        diff = (alone.float() - outs[l].float()).abs().max().item()
        say("layer %d: err vs oracle %.4g, vs the stand-alone launch %.4g" % (l, err, diff))
        assert diff <= 2e-2
