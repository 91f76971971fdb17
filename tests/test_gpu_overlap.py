"""Cross-layer top-k overlap (paper App. A) on the GPU against the oracle: integer counts exact."""
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


def _random_layers(seed, n, shape, k, Lk, holes):
    rng = np.random.default_rng(seed)
    nq = int(np.prod(shape))
    out = []
    for l in range(n):
        idx = np.full((nq, k), -1, dtype=np.int32)
        for t in range(nq):
            m = int(rng.integers(0, k + 1)) if holes else k
            idx[t, :m] = rng.choice(Lk, size=m, replace=False)          # unsorted on purpose
        out.append(idx.reshape(*shape, k))
    return out


@pytest.mark.parametrize("case", [
    # n_layers, shape of the query axes, k_sel, Lk, rows with fewer members
    (5, (2, 19), 24, 300, True),       # ragged query block (38 rows, blocks of 16), tiny Lk
    (3, (1, 64), 2048, 40000, False),  # full-size rows, bitmap of several KB
    (1, (1, 5), 7, 33, True),          # single layer: only the diagonal
    (9, (1, 33), 100, 1 << 20, True),  # largest supported position range (128 KB bitmap): the membership form
    # the bitmap form beyond one chunk, one tile or one pass
    (48, (1, 20), 256, 40000, True),   # 12 x 12 tiles of layers, three chunks of the position range
    (128, (1, 6), 64, 9000, True),     # the most layers: short chunks, 32 x 32 tiles
    (7, (1, 9), 5000, 20000, False),   # rows longer than one pass of the workgroup; layers not a multiple of four
    (6, (3, 5), 30, 5000, True),       # k_sel not a multiple of four: scalar reads
    (2, (1, 300), 16, 64, False),      # more query rows than workgroups walk in one round; tiny bitmaps
])
def test_overlap_matches_oracle(ic, oracle, case):
    n, shape, k, Lk, holes = case
    say("overlap n_layers=%d shape=%s k=%d Lk=%d holes=%s" % (n, shape, k, Lk, holes))
    layers = _random_layers(1000 + n + k, n, shape, k, Lk, holes)
    layers[-1][..., 0] = Lk + 5                                           # out of range: not a member
    ov, inter, sizes = ic.topk_overlap([torch.from_numpy(a).cuda() for a in layers], Lk)
    torch.cuda.synchronize()
    want_ov, want_inter, want_sizes = oracle.topk_overlap(layers, Lk)
    assert np.array_equal(inter.cpu().numpy().astype(np.uint64), want_inter)
    assert np.array_equal(sizes.cpu().numpy().astype(np.uint64), want_sizes)
    got = ov.cpu().numpy()
    ok = want_sizes > 0
    assert np.array_equal(got[ok], want_ov[ok])                           # same two integers divided in fp64
    assert np.all(got[~ok] == 0.0)


def test_overlap_of_a_shared_stack(ic, oracle):
    """Indices out of ic_forward_stack: layers of one sharing block overlap fully, correlated Full
    layers overlap more than chance (the keys of the synthetic stack are correlated across layers)."""
    cfg = synth.config("c0")
    say("overlap on the c0 stack, pattern %s" % cfg["pattern"])
    layers = synth.stack_layers(cfg, device="cuda")
    mask = ic.pattern_from_string(cfg["pattern"])
    used = []
    for l, lay in enumerate(layers):
        if mask[l]:
            cur = ic.indexer_topk(lay["q"], lay["k"], lay["w"], cfg["k_sel"], 0)
        used.append(cur)
    ov, inter, sizes = ic.topk_overlap(used, cfg["Lk"])
    torch.cuda.synchronize()
    want_ov, want_inter, want_sizes = oracle.topk_overlap([u.cpu().numpy() for u in used], cfg["Lk"])
    assert np.array_equal(inter.cpu().numpy().astype(np.uint64), want_inter)
    got = ov.cpu().numpy()
    src = [oracle.source_layer(mask, l) for l in range(len(mask))]
    for i in range(len(mask)):
        for j in range(len(mask)):
            if src[i] == src[j]:
                assert got[i, j] == 1.0
            else:
                assert cfg["k_sel"] / cfg["Lk"] < got[i, j] < 1.0        # above the chance level of independent sets


def test_overlap_decays_with_layer_distance_on_a_drifting_stack(ic):
    """Qualitative shape of the appendix's heat map: with q and k drifting from layer to layer the
    overlap is highest next to the diagonal and falls with the distance between the layers."""
    cfg = synth.config("c1", Tq=1024, Lk=1024, k_sel=128)
    say("overlap band structure, 8 drifting layers, L=1024, k=128")
    idxs = [ic.indexer_topk(lay["q"], lay["k"], lay["w"], cfg["k_sel"], 0)
            for lay in synth.chain_indexer_layers(cfg, 8, device="cuda")]
    ov = ic.topk_overlap(idxs, cfg["Lk"])[0].cpu()
    by_dist = [float(torch.diagonal(ov, d).mean()) for d in range(8)]
    say("mean overlap by distance: " + " ".join("%.3f" % v for v in by_dist))
    assert by_dist[0] == 1.0
    assert all(by_dist[d] > by_dist[d + 1] for d in range(0, 5))
    assert torch.allclose(ov, ov.T)                                       # every row holds the same number of members
