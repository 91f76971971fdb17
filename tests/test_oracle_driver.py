"""Pins for the oracle's Full/Shared layer loop (O5; Fig. 2 and Sec. 3 Overview)."""
import os

import numpy as np
import pytest

import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "searched_patterns.txt")


def _patterns():
    out = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        model, ratio, s = line.split()
        num, den = ratio.split("/")
        out.append((model, int(num) / int(den), s))
    return out


def test_paper_pattern_strings_parse(oracle):
    pats = _patterns()
    assert len(pats) == 5
    for model, ratio, s in pats:
        mask = oracle.pattern_from_string(s)
        assert len(mask) == (47 if model == "dsa30b" else 78)     # 47 layers: Sec. 4 setup
        assert mask[0]                                             # first layer always F
        assert abs(sum(mask) / len(mask) - ratio) < 0.04           # "keep 1/2, 1/4, 1/8"
        for l in range(len(mask)):
            f = oracle.source_layer(mask, l)
            if mask[l]:
                assert f == l
            else:
                assert f < l and mask[f] and not any(mask[f + 1: l + 1])


def test_pattern_errors(oracle):
    with pytest.raises(ValueError):
        oracle.pattern_from_string("SFFS")
    with pytest.raises(ValueError):
        oracle.pattern_from_string("FSX")
    with pytest.raises(ValueError):
        oracle.pattern_from_string("")
    assert oracle.pattern_uniform(9, 4) == [True, False, False, False, True, False, False, False, True]
    assert "".join("F" if m else "S" for m in oracle.pattern_uniform(8, 4)) == "FSSSFSSS"   # Sec. 3.1


@pytest.fixture(scope="module")
def tiny_stack():
    cfg = synth.config("c0", Tq=96, Lk=96, k_sel=16)
    layers = [synth.bits_layer(l) for l in synth.stack_layers(cfg)]
    return cfg, layers


def _run(oracle, cfg, layers, mask):
    return oracle.forward_stack(layers, mask, cfg["k_sel"], 0, cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg))


def test_shared_layers_reuse_nearest_preceding_full(oracle, tiny_stack):
    cfg, layers = tiny_stack
    for pat in ["FSFS", "FSSS", "FFSF"]:
        mask = oracle.pattern_from_string(pat)
        outs, used, n_idx = _run(oracle, cfg, layers, mask)
        assert n_idx == sum(mask)                                 # indexer runs only on F layers
        for l in range(len(mask)):
            f = oracle.source_layer(mask, l)
            assert np.array_equal(used[l], used[f])               # bit-identical indices
            own = oracle.indexer_topk(layers[f]["q"], layers[f]["k"], layers[f]["w"], 0, cfg["k_sel"])["idx"]
            assert np.array_equal(used[l], own)
            # an S layer attends over its OWN Q/KV with the inherited indices
            O, _ = oracle.sparse_attn(layers[l]["Q"], layers[l]["KV"], own, cfg["d_v"], cfg["v_off"],
                                      synth.sm_scale(cfg))
            assert np.array_equal(outs[l], O)


def test_all_full_mask_is_standard_dsa(oracle, tiny_stack):
    cfg, layers = tiny_stack
    outs, used, n_idx = _run(oracle, cfg, layers, [True] * 4)
    assert n_idx == 4
    for l in range(4):
        own = oracle.indexer_topk(layers[l]["q"], layers[l]["k"], layers[l]["w"], 0, cfg["k_sel"])["idx"]
        assert np.array_equal(used[l], own)
    # correlated keys but independent queries: layers pick different sets
    assert not np.array_equal(used[0], used[1])


def test_first_layer_must_be_full(oracle, tiny_stack):
    cfg, layers = tiny_stack
    with pytest.raises(ValueError):
        _run(oracle, cfg, layers, [False, True, True, True])


def test_tiny_config_has_exact_zero_scores(oracle):
    # with H_I = 4 about 1/16 of all causal scores are exactly 0 (all four heads gated off)
    cfg = synth.config("c0", Tq=128, Lk=128)
    layer = synth.bits_layer(synth.indexer_layer(cfg, 0))
    sc = oracle.indexer_scores(layer["q"], layer["k"], layer["w"], 0)[0]
    low = np.tril(np.ones((128, 128), dtype=bool))
    frac = (sc[low] == 0).mean()
    assert 0.04 < frac < 0.09
