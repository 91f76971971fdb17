"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and turns bad arguments into status codes before anything is launched."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "indexcache.h")


@pytest.fixture(scope="module")
def ic():
    import paper_2603_12201_amd as m
    if not os.path.exists(m.lib_path()):
        from paper_2603_12201_amd import build
        build.build()
    m.lib()
    return m


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ic_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(ic):
    names = _declared()
    assert {"ic_indexer_topk", "ic_sparse_attn", "ic_forward_stack"} <= set(names)
    L = ic.lib()
    for n in names:
        assert hasattr(L, n), "libindexcache.so does not export %s" % n


def test_struct_sizes_match_header_layout(ic):
    # field order/size as declared: 6*int32 + int64 + int32 + uint32 + 2 pointers
    assert C.sizeof(ic.IndexerDesc) == 56
    assert C.sizeof(ic.AttnDesc) == 40
    assert C.sizeof(ic.Layer) == 56 + 24 + 40 + 24


def test_pattern_helpers(ic):
    assert ic.pattern_uniform(8, 4) == [True, False, False, False, True, False, False, False]
    assert ic.pattern_uniform(3, 1) == [True, True, True]
    assert ic.pattern_from_string("FSSF") == [True, False, False, True]
    for bad, st in [("SFF", ic.Status.ERR_PATTERN), ("FXS", ic.Status.ERR_PATTERN)]:
        with pytest.raises(ic.IcError) as e:
            ic.pattern_from_string(bad)
        assert e.value.status == st
    with pytest.raises(ic.IcError) as e:
        ic.pattern_uniform(4, 0)
    assert e.value.status == ic.Status.ERR_SHAPE
    L = ic.lib()
    buf = C.create_string_buffer(4)
    assert L.ic_pattern_from_string(b"FS", buf, 3) == ic.Status.ERR_SHAPE      # length mismatch
    assert L.ic_pattern_from_string(None, buf, 3) == ic.Status.ERR_NULL
    assert b"pattern" in L.ic_last_error() or b"NULL" in L.ic_last_error()


def test_paper_patterns_through_the_library(ic):
    for line in open(os.path.join(ROOT, "tests", "golden", "searched_patterns.txt")):
        if line.startswith("#") or not line.strip():
            continue
        _, _, s = line.split()
        mask = ic.pattern_from_string(s)
        assert [c == "F" for c in s] == mask


def _ixd(ic, **kw):
    d = dict(B=1, Tq=128, Lk=128, H_I=32, d_I=128, k_sel=64, q_pos0=0, dtype=0, flags=0,
             q_scale=None, k_scale=None)
    d.update(kw)
    return ic.IndexerDesc(**d)


def _atd(ic, **kw):
    d = dict(B=1, Tq=128, Lk=128, H_q=32, d_qk=576, d_v=512, v_off=0, row_elems=576, k_sel=64, sm_scale=0.04)
    d.update(kw)
    return ic.AttnDesc(**d)


def test_indexer_argument_errors(ic):
    L = ic.lib()
    S = ic.Status
    one = C.c_void_p(4096)   # never dereferenced: validation fails first
    good = _ixd(ic)
    ws = L.ic_indexer_topk_workspace(C.byref(good))
    assert ws >= 16 * 128 * 4 and ws % 256 == 0
    assert L.ic_indexer_topk(None, one, one, one, one, None, one, ws, None) == S.ERR_NULL
    assert L.ic_indexer_topk(C.byref(good), None, one, one, one, None, one, ws, None) == S.ERR_NULL
    assert L.ic_indexer_topk(C.byref(good), one, one, one, None, None, one, ws, None) == S.ERR_NULL
    assert L.ic_indexer_topk(C.byref(good), one, one, one, one, None, None, ws, None) == S.ERR_WORKSPACE
    assert L.ic_indexer_topk(C.byref(good), one, one, one, one, None, C.c_void_p(4096 + 8), ws, None) == S.ERR_WORKSPACE
    assert L.ic_indexer_topk(C.byref(good), one, one, one, one, None, one, 1024, None) == S.ERR_WORKSPACE
    for kw, st in [(dict(k_sel=4096), S.ERR_UNSUPPORTED), (dict(k_sel=0), S.ERR_SHAPE), (dict(B=0), S.ERR_SHAPE),
                   (dict(Lk=-3), S.ERR_SHAPE), (dict(d_I=96), S.ERR_UNSUPPORTED), (dict(H_I=65), S.ERR_UNSUPPORTED),
                   (dict(dtype=7), S.ERR_UNSUPPORTED), (dict(flags=1), S.ERR_UNSUPPORTED)]:
        bad = _ixd(ic, **kw)
        assert L.ic_indexer_topk_workspace(C.byref(bad)) == 0
        assert L.ic_indexer_topk(C.byref(bad), one, one, one, one, None, one, ws, None) == st, kw
        assert len(L.ic_last_error()) > 0


def test_attention_argument_errors(ic):
    L = ic.lib()
    S = ic.Status
    one = C.c_void_p(4096)
    good = _atd(ic, k_sel=256)
    assert L.ic_sparse_attn_workspace(C.byref(good)) > 0          # 128 queries < 256: split path
    assert L.ic_sparse_attn_workspace(C.byref(_atd(ic, Tq=4096, Lk=4096))) == 0
    assert L.ic_sparse_attn(C.byref(good), None, one, one, one, None, one, 1 << 30, None) == S.ERR_NULL
    assert L.ic_sparse_attn(C.byref(good), one, one, one, one, None, None, 0, None) == S.ERR_WORKSPACE
    for kw, st in [(dict(H_q=33), S.ERR_UNSUPPORTED), (dict(d_qk=128), S.ERR_UNSUPPORTED),
                   (dict(v_off=4), S.ERR_SHAPE), (dict(v_off=128), S.ERR_UNSUPPORTED),
                   (dict(row_elems=512), S.ERR_UNSUPPORTED), (dict(sm_scale=0.0), S.ERR_SHAPE),
                   (dict(k_sel=0), S.ERR_SHAPE)]:
        bad = _atd(ic, **kw)
        assert L.ic_sparse_attn(C.byref(bad), one, one, one, one, None, one, 1 << 30, None) == st, kw


def test_forward_stack_argument_errors(ic):
    L = ic.lib()
    S = ic.Status
    one = 4096
    arr = (ic.Layer * 2)()
    for l in range(2):
        arr[l].ix = _ixd(ic, Tq=4096, Lk=4096)
        arr[l].at = _atd(ic, Tq=4096, Lk=4096)
        arr[l].q = arr[l].k = arr[l].w = arr[l].Q = arr[l].KV = arr[l].O = one
    ws = L.ic_forward_stack_workspace(arr, 2)
    assert ws > 0
    p = C.c_void_p(one)
    # the first layer must be Full (there is nothing to reuse yet)
    assert L.ic_forward_stack(arr, 2, bytes([0, 1]), p, p, ws, None) == S.ERR_PATTERN
    assert L.ic_forward_stack(arr, 2, None, p, p, ws, None) == S.ERR_NULL
    assert L.ic_forward_stack(arr, 2, bytes([1, 0]), None, p, ws, None) == S.ERR_NULL
    assert L.ic_forward_stack(arr, 0, bytes([1]), p, p, ws, None) == S.ERR_SHAPE
    assert L.ic_forward_stack(arr, 2, bytes([1, 0]), p, p, 16, None) == S.ERR_WORKSPACE
    arr[1].at.k_sel = 32                                             # one index buffer: k_sel must agree
    assert L.ic_forward_stack(arr, 2, bytes([1, 0]), p, p, ws, None) == S.ERR_SHAPE
    arr[1].at.k_sel = 64
    arr[0].ix.Lk = 8192                                              # indexer scores keys the KV cache does not hold
    assert L.ic_forward_stack(arr, 2, bytes([1, 0]), p, p, ws, None) == S.ERR_SHAPE
    assert b"KV cache" in L.ic_last_error()
    arr[0].ix.Lk = 4096
    arr[1].at.Lk = 2048                                              # a Shared layer's cache is shorter than the inherited indices
    assert L.ic_forward_stack(arr, 2, bytes([1, 0]), p, p, ws, None) == S.ERR_SHAPE
    assert b"Shared layer 1" in L.ic_last_error()
    arr[1].at.Lk = 8192                                              # a longer one is fine: it gets past the shape checks
    assert L.ic_forward_stack(arr, 2, bytes([1, 0]), p, p, 16, None) == S.ERR_WORKSPACE
    arr[1].at.Lk = 4096
    arr[1].q = None                                                  # a Shared layer may omit q,k,w ...
    arr[0].q = None                                                  # ... a Full layer may not
    assert L.ic_forward_stack(arr, 2, bytes([1, 0]), p, p, ws, None) == S.ERR_NULL
    # workspace need does not grow with the number of Shared layers (one index buffer, one strip)
    assert L.ic_forward_stack_workspace(arr, 1) <= ws


def test_prof_api_without_gpu(ic):
    ic.prof_reset()
    assert ic.prof_get(0) == (0, 0.0)
    with pytest.raises(ic.IcError):
        ic.prof_get(9)


def test_overlap_argument_errors_need_no_gpu():
    import paper_2603_12201_amd as ic
    L, S = ic.lib(), ic.Status
    one = C.c_void_p(4096)
    ptrs = (C.c_void_p * 3)(4096, 8192, 12288)
    ws = L.ic_topk_overlap_workspace(3)
    assert ws >= (9 + 3) * 8
    assert L.ic_topk_overlap_workspace(0) == 0 and L.ic_topk_overlap_workspace(129) == 0
    assert L.ic_topk_overlap(None, 3, 10, 8, 100, one, None, None, one, ws, None) == S.ERR_NULL
    assert L.ic_topk_overlap(ptrs, 3, 10, 8, 100, None, None, None, one, ws, None) == S.ERR_NULL      # no output
    assert L.ic_topk_overlap(ptrs, 0, 10, 8, 100, one, None, None, one, ws, None) == S.ERR_SHAPE
    assert L.ic_topk_overlap(ptrs, 3, 10, 0, 100, one, None, None, one, ws, None) == S.ERR_SHAPE
    assert L.ic_topk_overlap(ptrs, 3, -1, 8, 100, one, None, None, one, ws, None) == S.ERR_SHAPE
    assert L.ic_topk_overlap(ptrs, 3, 10, 8, (1 << 20) + 1, one, None, None, one, ws, None) == S.ERR_UNSUPPORTED
    assert L.ic_topk_overlap(ptrs, 129, 10, 8, 100, one, None, None, one, ws, None) == S.ERR_UNSUPPORTED
    assert L.ic_topk_overlap(ptrs, 3, 10, 8, 100, one, None, None, None, ws, None) == S.ERR_WORKSPACE
    assert L.ic_topk_overlap(ptrs, 3, 10, 8, 100, one, None, None, one, 8, None) == S.ERR_WORKSPACE
    bad = (C.c_void_p * 3)(4096, None, 12288)
    assert L.ic_topk_overlap(bad, 3, 10, 8, 100, one, None, None, one, ws, None) == S.ERR_NULL
    assert b"idx_layers[1]" in L.ic_last_error()


def test_pattern_search_dp_matches_exhaustive_search(oracle):
    """Host-only: the dynamic program against the definition (every pattern enumerated)."""
    import numpy as np
    import paper_2603_12201_amd as ic
    rng = np.random.default_rng(8)
    for n in (1, 2, 5, 9, 12):
        S = np.tril(rng.random((n, n)), -1)
        for m in sorted({1, 2, (n + 1) // 2, n}):
            if m > n:
                continue
            mask, total = ic.pattern_search_dp(S, m)
            best, arg = oracle.pattern_search_exhaustive(S, m)
            assert mask[0] and sum(mask) == m
            assert abs(total - best) <= 1e-12 and abs(oracle.pattern_total(S, mask) - best) <= 1e-12
            if len(arg) == 1:
                assert mask == arg[0]
    # block-structured similarities: the optimum puts the Full layers on the block heads
    blocks = [0, 0, 0, 3, 3, 5, 5, 5, 5, 9]
    S = np.array([[1.0 if blocks[l] == blocks[j] else 0.2 for j in range(10)] for l in range(10)])
    mask, total = ic.pattern_search_dp(S, 4)
    assert [l for l in range(10) if mask[l]] == [0, 3, 5, 9] and abs(total - 6.0) < 1e-12
    # paper-sized problem (47 layers, a quarter kept) runs at once and is at least as good as uniform
    S = np.tril(rng.random((47, 47)), -1)
    mask, total = ic.pattern_search_dp(S, 12)
    assert mask[0] and sum(mask) == 12
    uni = ic.pattern_uniform(47, 4)
    assert sum(uni) == 12 and total >= oracle.pattern_total(S, uni) - 1e-12


def test_similarity_argument_errors_need_no_gpu():
    import paper_2603_12201_amd as ic
    L, S = ic.lib(), ic.Status
    one = C.c_void_p(4096)
    assert L.ic_cosine_rows(None, one, 4, 8, one, None, one, 256, None) == S.ERR_NULL
    assert L.ic_cosine_rows(one, one, 0, 8, one, None, one, 256, None) == S.ERR_SHAPE
    assert L.ic_cosine_rows(one, one, 4, 8, one, None, None, 256, None) == S.ERR_WORKSPACE
    assert L.ic_cosine_rows(one, one, 4, 8, one, None, one, 8, None) == S.ERR_WORKSPACE
    flat = (C.c_double * 4)(0, 0, 0.5, 0)
    buf = C.create_string_buffer(2)
    assert L.ic_pattern_search_dp(flat, 2, 3, buf, None) == S.ERR_SHAPE
    assert L.ic_pattern_search_dp(flat, 2, 0, buf, None) == S.ERR_SHAPE
    assert L.ic_pattern_search_dp(None, 2, 1, buf, None) == S.ERR_NULL
    assert L.ic_pattern_search_dp(flat, 2, 1, buf, None) == S.OK and buf.raw[:2] == bytes([1, 0])


def test_paged_cache_argument_errors(ic):
    L, S = ic.lib(), ic.Status
    one = C.c_void_p(4096)
    ixd = _ixd(ic)
    atd = _atd(ic, k_sel=256)
    ws = max(L.ic_indexer_topk_workspace(C.byref(ixd)), L.ic_sparse_attn_workspace(C.byref(atd)))
    Lk = ixd.Lk
    pages = -(-Lk // 64)

    def pc(page_size=64, max_pages=pages, table=4096, lens=4096):
        return ic.PagedCache(page_size, max_pages, table, lens)

    def ix(p, d=ixd):
        return L.ic_indexer_topk_paged(C.byref(d), C.byref(p) if p is not None else None, one, one, one, one, None, one, ws, None)

    def at(p):
        return L.ic_sparse_attn_paged(C.byref(atd), C.byref(p) if p is not None else None, one, one, one, one, None, one, ws, None)

    for call in (ix, at):
        assert call(None) == S.ERR_NULL
        assert call(pc(table=None, lens=None)) == S.ERR_NULL             # neither ragged nor paged
        assert call(pc(page_size=48)) == S.ERR_SHAPE                     # not a power of two
        assert call(pc(page_size=32, max_pages=4 * pages)) == S.ERR_SHAPE   # below one key tile
        assert call(pc(max_pages=pages - 1)) == S.ERR_SHAPE              # table rows do not cover Lk
        assert call(pc(max_pages=0)) == S.ERR_SHAPE
        assert len(L.ic_last_error()) > 0
    # the page geometry is ignored when only the lengths are given
    assert L.ic_indexer_topk_paged(C.byref(ixd), C.byref(pc(page_size=0, max_pages=0, table=None)), None, one, one, one,
                                   None, one, ws, None) == S.ERR_NULL    # got past the cache check: q is NULL
    fp8 = _ixd(ic, dtype=1)
    fp8.q_scale = fp8.k_scale = 4096
    assert ix(pc(), fp8) == S.ERR_UNSUPPORTED                            # paged fp8 index keys
    assert L.ic_indexer_topk_paged(C.byref(ixd), C.byref(pc()), one, one, one, one, None, one, 16, None) == S.ERR_WORKSPACE
    # the stack entry point applies the same checks to every layer
    arr = (ic.Layer * 2)()
    for l in range(2):
        arr[l].ix, arr[l].at = _ixd(ic), _atd(ic, k_sel=64)
        arr[l].q = arr[l].k = arr[l].w = arr[l].Q = arr[l].KV = arr[l].O = 4096
    wss = L.ic_forward_stack_workspace(arr, 2)
    assert L.ic_forward_stack_paged(arr, 2, bytes([1, 0]), None, one, one, wss, None) == S.ERR_NULL
    assert L.ic_forward_stack_paged(arr, 2, bytes([1, 0]), C.byref(pc(max_pages=1)), one, one, wss, None) == S.ERR_SHAPE
    assert L.ic_forward_stack_paged(arr, 2, bytes([0, 1]), C.byref(pc()), one, one, wss, None) == S.ERR_PATTERN


def test_greedy_search_on_a_similarity_matrix_matches_the_oracle(oracle):
    """Host-only: Alg. 1 in the library against the oracle's, plain and blocked, random matrices."""
    import numpy as np
    import paper_2603_12201_amd as ic
    rng = np.random.default_rng(11)
    for n in (2, 5, 9, 16):
        S = np.tril(rng.random((n, n)), -1) + np.eye(n)
        f = lambda m: oracle.pattern_loss_from_similarity(S, m)
        for blocks in (1, 2, 3):
            if blocks > n:
                continue
            size = -(-n // blocks)
            n_cand = sum(min(size, n - b0) - 1 for b0 in range(0, n, size))
            for K in sorted({0, min(1, n_cand), n_cand // 2, n_cand}):
                mask, order, curve = ic.pattern_search_greedy(S, K, blocks)
                want_mask, want_order, want_curve = oracle.greedy_search(f, n, K, blocks)
                assert mask == want_mask and order == want_order
                assert np.allclose(curve, want_curve, rtol=0, atol=1e-13)
    # the worked example: greedy takes {2, 3}, the optimum is {1, 3}
    S = np.eye(4)
    S[1, 0], S[2, 1], S[2, 0], S[3, 2], S[3, 1], S[3, 0] = 0.90, 0.99, 0.20, 0.50, 0.40, 0.30
    mask, order, curve = ic.pattern_search_greedy(S, 2)
    assert order == [2, 3] and mask == [True, True, False, False] and curve == pytest.approx([0.0025, 0.1525])


def test_greedy_argument_errors_need_no_gpu(ic):
    L, S = ic.lib(), ic.Status
    flat = (C.c_double * 16)(*([1.0] * 16))
    buf = C.create_string_buffer(4)
    assert L.ic_pattern_search_greedy(None, 4, 1, 1, buf, None, None) == S.ERR_NULL
    assert L.ic_pattern_search_greedy(flat, 4, 1, 1, None, None, None) == S.ERR_NULL
    assert L.ic_pattern_search_greedy(flat, 4, 4, 1, buf, None, None) == S.ERR_SHAPE      # layer 0 stays Full
    assert L.ic_pattern_search_greedy(flat, 4, -1, 1, buf, None, None) == S.ERR_SHAPE
    assert L.ic_pattern_search_greedy(flat, 4, 1, 0, buf, None, None) == S.ERR_SHAPE
    assert L.ic_pattern_search_greedy(flat, 4, 1, 5, buf, None, None) == S.ERR_SHAPE
    assert L.ic_pattern_search_greedy(flat, 4, 3, 2, buf, None, None) == S.ERR_SHAPE      # two blocks: two candidates
    assert L.ic_pattern_search_greedy(flat, 4, 2, 2, buf, None, None) == S.OK and buf.raw == b"\x01\x00\x01\x00"
    arr = (ic.Layer * 2)()
    for l in range(2):
        arr[l].ix, arr[l].at = _ixd(ic), _atd(ic, k_sel=64)
        arr[l].q = arr[l].k = arr[l].w = arr[l].Q = arr[l].KV = arr[l].O = 4096
    ws = L.ic_pattern_loss_workspace(arr, 2)
    assert ws > 0 and L.ic_greedy_search_forward_workspace(arr, 2) > ws
    one = C.c_void_p(8192)
    refs = (C.c_void_p * 2)(8192, 12288)
    assert L.ic_pattern_loss(arr, 2, bytes([1, 0]), None, one, one, one, ws, None) == S.ERR_NULL
    assert L.ic_pattern_loss(arr, 2, bytes([1, 0]), refs, one, None, one, ws, None) == S.ERR_NULL
    assert L.ic_pattern_loss(arr, 2, bytes([1, 0]), refs, one, one, one, 64, None) == S.ERR_WORKSPACE
    own = (C.c_void_p * 2)(8192, 4096)                                                     # a layer's own O
    assert L.ic_pattern_loss(arr, 2, bytes([1, 0]), own, one, one, one, ws, None) == S.ERR_SHAPE
    assert L.ic_greedy_search_forward(arr, 2, 1, 1, refs, one, None, None, None, one, 1 << 30, None) == S.ERR_NULL
    assert L.ic_greedy_search_forward(arr, 2, 1, 1, refs, one, buf, None, None, one, 64, None) == S.ERR_WORKSPACE


def test_distill_argument_errors_need_no_gpu(ic):
    L, S = ic.lib(), ic.Status
    one = C.c_void_p(4096)
    atd = _atd(ic)
    assert L.ic_attn_probs(None, one, one, one, one, one, None) == S.ERR_NULL
    assert L.ic_attn_probs(C.byref(atd), one, one, one, None, one, None) == S.ERR_NULL         # the normalisers are required
    assert L.ic_attn_probs(C.byref(_atd(ic, d_qk=128)), one, one, one, one, one, None) == S.ERR_UNSUPPORTED
    ws = L.ic_distill_loss_workspace(1000)
    assert ws >= 2 * 8000 and L.ic_distill_loss_workspace(0) > 0
    ptrs = (C.c_void_p * 2)(4096, 8192)
    assert L.ic_distill_loss(None, 2, one, 1000, 64, one, one, None, one, ws, None) == S.ERR_NULL
    assert L.ic_distill_loss(ptrs, 2, None, 1000, 64, one, one, None, one, ws, None) == S.ERR_NULL
    assert L.ic_distill_loss(ptrs, 0, one, 1000, 64, one, one, None, one, ws, None) == S.ERR_SHAPE
    assert L.ic_distill_loss(ptrs, 17, one, 1000, 64, one, one, None, one, ws, None) == S.ERR_SHAPE
    assert L.ic_distill_loss(ptrs, 2, one, 1000, 0, one, one, None, one, ws, None) == S.ERR_SHAPE
    assert L.ic_distill_loss(ptrs, 2, one, 1000, 64, None, None, None, one, ws, None) == S.ERR_NULL   # no output
    assert L.ic_distill_loss(ptrs, 2, one, 1000, 64, one, one, None, one, 64, None) == S.ERR_WORKSPACE
    bad = (C.c_void_p * 2)(4096, None)
    assert L.ic_distill_loss(bad, 2, one, 1000, 64, one, one, None, one, ws, None) == S.ERR_NULL


def test_calibrate_argument_errors_need_no_gpu(ic):
    L, S = ic.lib(), ic.Status
    one = C.c_void_p(4096)
    assert L.ic_calibrate(99, one, one, None, 16, 0, 0, 1, None) == S.ERR_SHAPE               # unknown kind
    assert L.ic_calibrate(ic.CALIB_READ, one, None, None, 16, 0, 0, 1, None) == S.ERR_NULL       # no dst
    assert L.ic_calibrate(ic.CALIB_READ, None, one, None, 16, 0, 0, 1, None) == S.ERR_NULL       # no src
    assert L.ic_calibrate(ic.CALIB_READ, one, one, None, 24, 0, 0, 1, None) == S.ERR_SHAPE       # not a multiple of 16
    assert L.ic_calibrate(ic.CALIB_READ, one, one, None, 16, 0, 0, 0, None) == S.ERR_SHAPE       # no workgroups
    assert L.ic_calibrate(ic.CALIB_GATHER, one, one, None, 64, 10, 1152, 1, None) == S.ERR_NULL  # no idx
    assert L.ic_calibrate(ic.CALIB_GATHER, one, one, one, 64, 10, 512, 1, None) == S.ERR_UNSUPPORTED
    assert L.ic_calibrate(ic.CALIB_GATHER, one, one, one, 64, 0, 1152, 1, None) == S.ERR_SHAPE
    for kind in (ic.CALIB_TILE_GATHER, ic.CALIB_TILE_STORE, ic.CALIB_TILE_READ, ic.CALIB_TILE_READ2, ic.CALIB_TILE_8WAVES,
                 ic.CALIB_TILE_INTERLEAVED):
        assert L.ic_calibrate(kind, one, one, None, 64, 10, 1152, 1, None) == S.ERR_NULL
        assert L.ic_calibrate(kind, one, one, one, 100, 10, 1152, 1, None) == S.ERR_SHAPE        # whole tiles of 64 rows
        assert L.ic_calibrate(kind, one, one, one, 64, 10, 256, 1, None) == S.ERR_UNSUPPORTED
    assert L.ic_calibrate(ic.CALIB_MFMA_BF16, None, one, None, 1 << 40, 0, 0, 1, None) == S.ERR_SHAPE
    assert L.ic_calibrate(ic.CALIB_LDS_TR8_ROWS1, None, one, None, 1 << 40, 0, 0, 1, None) == S.ERR_SHAPE
    assert L.ic_calibrate(ic.CALIB_LDS_TR8_ROWS1 + 1, None, one, None, 1, 0, 0, 1, None) == S.ERR_SHAPE   # unknown kind


def test_bench_refuses_more_than_one_gpu():
    """The build is for one GPU: the bench says so and exits instead of pretending to scale."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
