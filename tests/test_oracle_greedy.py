"""Pins for the oracle's greedy layer selection (paper Alg. 1) and its surrogate loss."""
import itertools

import numpy as np
import pytest


def _loss(oracle, S):
    return lambda mask: oracle.pattern_loss_from_similarity(S, mask)


def test_loss_is_tied_to_the_similarity_objective(oracle):
    # loss(c) = (#Shared - sum_l S[l, src(l)]) / N: the App. C objective (pinned elsewhere by the
    # exhaustive search) seen from the other side
    rng = np.random.default_rng(1)
    N = 9
    S = np.tril(rng.random((N, N)), -1) + np.eye(N)
    for bits in itertools.product([False, True], repeat=N - 1):
        mask = [True] + list(bits)
        want = ((N - sum(mask)) - oracle.pattern_total(S, mask)) / N
        assert oracle.pattern_loss_from_similarity(S, mask) == pytest.approx(want, abs=1e-14)
    assert oracle.pattern_loss_from_similarity(S, [True] * N) == 0.0


def test_first_flip_is_the_best_single_flip_and_counts_hold(oracle):
    rng = np.random.default_rng(2)
    N = 10
    S = np.tril(rng.random((N, N)), -1) + np.eye(N)
    f = _loss(oracle, S)
    mask, order, curve = oracle.greedy_search(f, N, 1)
    # one step of Alg. 1 is an exhaustive search over single flips: 1 - S[l, l-1] minimal
    want = min(range(1, N), key=lambda l: (1.0 - S[l, l - 1], l))
    assert order == [want] and curve[0] == pytest.approx((1.0 - S[want, want - 1]) / N)
    for K in range(N):
        mask, order, curve = oracle.greedy_search(f, N, K)
        assert mask[0] and sum(not m for m in mask) == K and len(set(order)) == K and 0 not in order
        assert sorted(order) == [l for l in range(N) if not mask[l]]
        # the recorded curve is the loss of the pattern after each flip, recomputed from scratch
        m = [True] * N
        for l, v in zip(order, curve):
            m[l] = False
            assert v == pytest.approx(f(m), abs=1e-15)
    with pytest.raises(ValueError):
        oracle.greedy_search(f, N, N)


def test_worked_example_where_greedy_differs_from_the_optimum(oracle):
    # 4 layers.  Layer 2 reads layer 1 almost for free, so greedy flips it first; after that layer 1
    # can only be flipped at the price of sending layer 2 to layer 0 as well.
    S = np.eye(4)
    S[1, 0], S[2, 1], S[2, 0], S[3, 2], S[3, 1], S[3, 0] = 0.90, 0.99, 0.20, 0.50, 0.40, 0.30
    f = _loss(oracle, S)
    mask, order, curve = oracle.greedy_search(f, 4, 2)
    # step 1: candidates 1, 2, 3 cost 0.10, 0.01, 0.50 -> layer 2
    # step 2: {1,2} costs 0.10 + 0.80 = 0.90; {2,3} costs 0.01 + (1 - S[3,1]) = 0.61 -> layer 3
    assert order == [2, 3] and mask == [True, True, False, False]
    assert curve == pytest.approx([0.01 / 4, 0.61 / 4])
    # the best pattern with two Shared layers is {1, 3}: 0.10 + 0.50 = 0.60 < 0.61
    best = min((f([True] + [l not in c for l in range(1, 4)]), c) for c in itertools.combinations(range(1, 4), 2))
    assert best[1] == (1, 3) and best[0] == pytest.approx(0.60 / 4)
    assert curve[-1] > best[0]


def test_ties_go_to_the_lowest_layer_and_decay_matrix_order(oracle):
    N = 6
    S = np.eye(N) + np.tril(np.full((N, N), 0.5), -1)       # every reuse costs the same
    mask, order, _ = oracle.greedy_search(_loss(oracle, S), N, 3)
    assert order == [1, 2, 3]
    # similarity decays with the layer distance: a flip is cheapest where the source stays adjacent,
    # so greedy never creates a run of two Shared layers while an isolated candidate is left
    S = np.eye(N)
    for l in range(N):
        for j in range(l):
            S[l, j] = 0.9 ** (l - j)
    mask, order, _ = oracle.greedy_search(_loss(oracle, S), N, 2)
    assert order == [1, 3] and mask == [True, False, True, False, True, True]


def test_block_variant(oracle):
    rng = np.random.default_rng(5)
    N = 12
    S = np.tril(rng.random((N, N)), -1) + np.eye(N)
    f = _loss(oracle, S)
    # one block is plain Alg. 1
    assert oracle.greedy_search(f, N, 5, 1) == oracle.greedy_search(f, N, 5)
    # three blocks of four: layers 0, 4, 8 stay Full, one flip per block and step, blocks in order
    mask, order, curve = oracle.greedy_search(f, N, 6, 3)
    assert mask[0] and mask[4] and mask[8] and sum(not m for m in mask) == 6
    assert [l // 4 for l in order] == [0, 1, 2, 0, 1, 2]
    # each commit is the best candidate of its block given everything committed before it
    m = [True] * N
    for l, v in zip(order, curve):
        blk = l // 4
        cands = [c for c in range(4 * blk + 1, 4 * blk + 4) if m[c]]
        vals = {}
        for c in cands:
            t = list(m); t[c] = False
            vals[c] = f(t)
        assert l == min(cands, key=lambda c: (vals[c], c)) and v == pytest.approx(vals[l], abs=1e-15)
        m[l] = False
    with pytest.raises(ValueError):
        oracle.greedy_search(f, N, 10, 3)                    # only 9 candidates exist


def test_forward_loss_equals_the_similarity_form_on_an_attention_only_stack(oracle):
    import synth
    cfg = synth.config("c0", Tq=96, Lk=96, k_sel=16, n_layers=5)
    layers = [synth.bits_layer(l) for l in synth.stack_layers(cfg)]
    args = (cfg["k_sel"], 0, cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg))
    ref, used, _ = oracle.forward_stack(layers, [True] * 5, *args)
    S = oracle.similarity_matrix(layers, used, cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg))
    for mask in ([True, False, False, True, False], [True, True, False, False, False], [True] * 5):
        a = oracle.pattern_loss_forward(layers, mask, *args, ref)
        b = oracle.pattern_loss_from_similarity(S, mask)
        assert a == pytest.approx(b, abs=1e-12)
