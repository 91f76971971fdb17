"""ctypes binding of include/indexcache.h.  Same names as the C entry points, marshalling only."""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

BF16, FP8_E4M3 = 0, 1


class Status:
    OK, ERR_NULL, ERR_SHAPE, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_PATTERN, ERR_HIP = range(7)


class IcError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__("ic_status %d: %s" % (status, msg))
        self.status = status


class IndexerDesc(C.Structure):
    _fields_ = [("B", C.c_int32), ("Tq", C.c_int32), ("Lk", C.c_int32), ("H_I", C.c_int32),
                ("d_I", C.c_int32), ("k_sel", C.c_int32), ("q_pos0", C.c_int64),
                ("dtype", C.c_int32), ("flags", C.c_uint32),
                ("q_scale", C.c_void_p), ("k_scale", C.c_void_p)]


class AttnDesc(C.Structure):
    _fields_ = [("B", C.c_int32), ("Tq", C.c_int32), ("Lk", C.c_int32), ("H_q", C.c_int32),
                ("d_qk", C.c_int32), ("d_v", C.c_int32), ("v_off", C.c_int32),
                ("row_elems", C.c_int32), ("k_sel", C.c_int32), ("sm_scale", C.c_float)]


class PagedCache(C.Structure):
    _fields_ = [("page_size", C.c_int32), ("max_pages", C.c_int32), ("page_table", C.c_void_p), ("seq_lens", C.c_void_p)]


class Layer(C.Structure):
    _fields_ = [("ix", IndexerDesc), ("q", C.c_void_p), ("k", C.c_void_p), ("w", C.c_void_p),
                ("at", AttnDesc), ("Q", C.c_void_p), ("KV", C.c_void_p), ("O", C.c_void_p)]


def lib_path():
    return os.path.join(_HERE, "libindexcache.so")


def lib():
    """Load libindexcache.so.  No fallback: a missing library is an error."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise IcError(-1, "libindexcache.so is not built (run paper_2603_12201_amd/build.py "
                              "or __graft_entry__.build()); there is no fallback path")
        L = C.CDLL(path)
        vp, sz, i32 = C.c_void_p, C.c_size_t, C.c_int32
        L.ic_last_error.restype = C.c_char_p
        L.ic_indexer_topk_workspace.restype = sz
        L.ic_indexer_topk_workspace.argtypes = [C.POINTER(IndexerDesc)]
        L.ic_indexer_topk.restype = C.c_int
        L.ic_indexer_topk.argtypes = [C.POINTER(IndexerDesc), vp, vp, vp, vp, vp, vp, sz, vp]
        L.ic_sparse_attn_workspace.restype = sz
        L.ic_sparse_attn_workspace.argtypes = [C.POINTER(AttnDesc)]
        L.ic_sparse_attn.restype = C.c_int
        L.ic_sparse_attn.argtypes = [C.POINTER(AttnDesc), vp, vp, vp, vp, vp, vp, sz, vp]
        L.ic_calibrate.restype = C.c_int
        L.ic_calibrate.argtypes = [i32, vp, vp, vp, C.c_int64, C.c_int64, i32, i32, vp]
        L.ic_sparse_attn_static.restype = C.c_int
        L.ic_sparse_attn_static.argtypes = [C.POINTER(AttnDesc), vp, vp, vp, vp, vp, vp]
        L.ic_forward_stack_workspace.restype = sz
        L.ic_forward_stack_workspace.argtypes = [C.POINTER(Layer), i32]
        L.ic_forward_stack.restype = C.c_int
        L.ic_forward_stack.argtypes = [C.POINTER(Layer), i32, C.c_char_p, vp, vp, sz, vp]
        L.ic_pattern_from_string.restype = C.c_int
        L.ic_pattern_from_string.argtypes = [C.c_char_p, C.c_char_p, i32]
        L.ic_pattern_uniform.restype = C.c_int
        L.ic_pattern_uniform.argtypes = [i32, i32, C.c_char_p]
        L.ic_indexer_topk_paged.restype = C.c_int
        L.ic_indexer_topk_paged.argtypes = [C.POINTER(IndexerDesc), C.POINTER(PagedCache), vp, vp, vp, vp, vp, vp, sz, vp]
        L.ic_sparse_attn_paged.restype = C.c_int
        L.ic_sparse_attn_paged.argtypes = [C.POINTER(AttnDesc), C.POINTER(PagedCache), vp, vp, vp, vp, vp, vp, sz, vp]
        L.ic_forward_stack_paged.restype = C.c_int
        L.ic_forward_stack_paged.argtypes = [C.POINTER(Layer), i32, C.c_char_p, C.POINTER(PagedCache), vp, vp, sz, vp]
        L.ic_cosine_rows_workspace.restype = sz
        L.ic_cosine_rows.restype = C.c_int
        L.ic_cosine_rows.argtypes = [vp, vp, C.c_int64, C.c_int64, vp, vp, vp, sz, vp]
        L.ic_similarity_matrix_workspace.restype = sz
        L.ic_similarity_matrix_workspace.argtypes = [C.POINTER(Layer), i32]
        L.ic_similarity_matrix.restype = C.c_int
        L.ic_similarity_matrix.argtypes = [C.POINTER(Layer), i32, C.POINTER(vp), vp, vp, sz, vp]
        L.ic_pattern_search_greedy.restype = C.c_int
        L.ic_pattern_search_greedy.argtypes = [C.POINTER(C.c_double), i32, i32, i32, C.c_char_p, C.POINTER(i32), C.POINTER(C.c_double)]
        L.ic_pattern_loss_workspace.restype = sz
        L.ic_pattern_loss_workspace.argtypes = [C.POINTER(Layer), i32]
        L.ic_pattern_loss.restype = C.c_int
        L.ic_pattern_loss.argtypes = [C.POINTER(Layer), i32, C.c_char_p, C.POINTER(vp), vp, vp, vp, sz, vp]
        L.ic_greedy_search_forward_workspace.restype = sz
        L.ic_greedy_search_forward_workspace.argtypes = [C.POINTER(Layer), i32]
        L.ic_greedy_search_forward.restype = C.c_int
        L.ic_greedy_search_forward.argtypes = [C.POINTER(Layer), i32, i32, i32, C.POINTER(vp), vp, C.c_char_p, C.POINTER(i32),
                                               C.POINTER(C.c_double), vp, sz, vp]
        L.ic_attn_probs.restype = C.c_int
        L.ic_attn_probs.argtypes = [C.POINTER(AttnDesc), vp, vp, vp, vp, vp, vp]
        L.ic_distill_loss_workspace.restype = sz
        L.ic_distill_loss_workspace.argtypes = [C.c_int64]
        L.ic_distill_loss.restype = C.c_int
        L.ic_distill_loss.argtypes = [C.POINTER(vp), i32, vp, C.c_int64, i32, vp, vp, vp, vp, sz, vp]
        L.ic_pattern_search_dp.restype = C.c_int
        L.ic_pattern_search_dp.argtypes = [C.POINTER(C.c_double), i32, i32, C.c_char_p, C.POINTER(C.c_double)]
        L.ic_topk_overlap_workspace.restype = sz
        L.ic_topk_overlap_workspace.argtypes = [i32]
        L.ic_topk_overlap.restype = C.c_int
        L.ic_topk_overlap.argtypes = [C.POINTER(vp), i32, C.c_int64, i32, i32, vp, vp, vp, vp, sz, vp]
        L.ic_debug_indexer_scores.restype = C.c_int
        L.ic_debug_indexer_scores.argtypes = [C.POINTER(IndexerDesc), vp, vp, vp, i32, i32, vp, vp]
        L.ic_debug_indexer_launch_count.restype = C.c_uint64
        L.ic_prof_enable.restype = None
        L.ic_prof_enable.argtypes = [i32]
        L.ic_prof_collect.restype = C.c_int
        L.ic_prof_get.restype = C.c_int
        L.ic_prof_get.argtypes = [i32, C.POINTER(C.c_int64), C.POINTER(C.c_double)]
        L.ic_prof_reset.restype = None
        _LIB = L
    return _LIB


def last_error():
    return lib().ic_last_error().decode()


def _check(rc):
    if rc != 0:
        raise IcError(rc, last_error())


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _dtype_code(t):
    import torch
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float8_e4m3fn:
        return FP8_E4M3
    raise IcError(Status.ERR_UNSUPPORTED, "q/k dtype %s is not bf16 or float8_e4m3fn" % t.dtype)


def _need(t, name, dtype=None, ndim=None):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise IcError(Status.ERR_NULL, "%s must be a CUDA(HIP) tensor" % name)
    if not t.is_contiguous():
        raise IcError(Status.ERR_SHAPE, "%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise IcError(Status.ERR_SHAPE, "%s must have dtype %s, got %s" % (name, dtype, t.dtype))
    if ndim is not None and t.dim() != ndim:
        raise IcError(Status.ERR_SHAPE, "%s must have %d dims" % (name, ndim))


def indexer_desc(q, k, w, k_sel, q_pos0, q_scale=None, k_scale=None):
    import torch
    _need(q, "q", ndim=4)
    _need(k, "k", q.dtype, 3)
    _need(w, "w", torch.float32, 3)
    B, Tq, H, d = q.shape
    if k.shape[0] != B or k.shape[2] != d or tuple(w.shape) != (B, Tq, H):
        raise IcError(Status.ERR_SHAPE, "q %s, k %s, w %s disagree" % (tuple(q.shape), tuple(k.shape), tuple(w.shape)))
    code = _dtype_code(q)
    if code == FP8_E4M3:
        _need(q_scale, "q_scale", torch.float32, 2)
        _need(k_scale, "k_scale", torch.float32, 2)
    return IndexerDesc(B, Tq, k.shape[1], H, d, k_sel, q_pos0, code, 0,
                       q_scale.data_ptr() if q_scale is not None else None,
                       k_scale.data_ptr() if k_scale is not None else None)


def attn_desc(Q, KV, idx, d_v, v_off, sm_scale):
    import torch
    _need(Q, "Q", torch.bfloat16, 4)
    _need(KV, "KV", torch.bfloat16, 3)
    _need(idx, "idx", torch.int32, 3)
    B, Tq, Hq, d_qk = Q.shape
    if KV.shape[0] != B or idx.shape[0] != B or idx.shape[1] != Tq:
        raise IcError(Status.ERR_SHAPE, "Q %s, KV %s, idx %s disagree" % (tuple(Q.shape), tuple(KV.shape), tuple(idx.shape)))
    return AttnDesc(B, Tq, KV.shape[1], Hq, d_qk, d_v, v_off, KV.shape[2], idx.shape[2], sm_scale)


def _workspace(nbytes, like):
    import torch
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=like.device)


def indexer_topk_workspace(desc):
    return int(lib().ic_indexer_topk_workspace(C.byref(desc)))


def indexer_topk(q, k, w, k_sel, q_pos0=0, q_scale=None, k_scale=None, want_scores=False,
                 workspace=None, stream=None, idx=None):
    """ic_indexer_topk: returns idx [B,Tq,k_sel] int32 (ascending positions, -1 tail) and,
    if want_scores, sel_scores [B,Tq,k_sel] fp32."""
    import torch
    d = indexer_desc(q, k, w, k_sel, q_pos0, q_scale, k_scale)
    if workspace is None:
        need = indexer_topk_workspace(d)
        if need == 0:
            raise IcError(Status.ERR_UNSUPPORTED, last_error())
        workspace = _workspace(need, q)
    if idx is None:
        idx = torch.empty((d.B, d.Tq, k_sel), dtype=torch.int32, device=q.device)
    sel = torch.empty((d.B, d.Tq, k_sel), dtype=torch.float32, device=q.device) if want_scores else None
    _check(lib().ic_indexer_topk(C.byref(d), _ptr(q), _ptr(k), _ptr(w), _ptr(idx), _ptr(sel),
                                 _ptr(workspace), workspace.numel(), _stream(stream)))
    return (idx, sel) if want_scores else idx


def sparse_attn_workspace(desc):
    return int(lib().ic_sparse_attn_workspace(C.byref(desc)))


def sparse_attn(Q, KV, idx, d_v, v_off, sm_scale, want_lse=False, workspace=None, stream=None, out=None):
    """ic_sparse_attn: returns O [B,Tq,H_q,d_v] bf16 (and lse [B,Tq,H_q] fp32 if want_lse)."""
    import torch
    d = attn_desc(Q, KV, idx, d_v, v_off, sm_scale)
    if workspace is None:
        workspace = _workspace(sparse_attn_workspace(d), Q)
    O = out if out is not None else torch.empty((d.B, d.Tq, d.H_q, d_v), dtype=torch.bfloat16, device=Q.device)
    lse = torch.empty((d.B, d.Tq, d.H_q), dtype=torch.float32, device=Q.device) if want_lse else None
    _check(lib().ic_sparse_attn(C.byref(d), _ptr(Q), _ptr(KV), _ptr(idx), _ptr(O), _ptr(lse),
                                _ptr(workspace), workspace.numel(), _stream(stream)))
    return (O, lse) if want_lse else O


CALIB_READ, CALIB_COPY, CALIB_GATHER, CALIB_MFMA_BF16, CALIB_MFMA_FP8 = range(5)
CALIB_TILE_GATHER, CALIB_TILE_STORE, CALIB_TILE_READ, CALIB_TILE_READ2, CALIB_TILE_8WAVES, CALIB_TILE_INTERLEAVED = range(5, 11)
CALIB_LDS_READ16_PADDED, CALIB_LDS_READ16_SWIZZLED, CALIB_LDS_TR8_ROWS2, CALIB_LDS_TR8_ROWS1 = range(11, 15)


def calibrate(kind, src, dst, idx=None, n=0, table_rows=0, row_bytes=0, wgs=2048, stream=None):
    """ic_calibrate: one launch of a calibration kernel on the current stream (see indexcache.h)."""
    _check(lib().ic_calibrate(kind, _ptr(src), _ptr(dst), _ptr(idx), int(n), int(table_rows), int(row_bytes), int(wgs),
                              _stream(stream)))


STATIC_SCRATCH_BYTES = 16 << 20


def sparse_attn_static(Q, KV, idx, d_v, v_off, sm_scale, out, lse=None, stream=None):
    """ic_sparse_attn_static: ic_sparse_attn with the split partials in the library's own static scratch.
    Allocates nothing: the caller passes `out` [B,Tq,H_q,d_v] bf16 (and `lse` [B,Tq,H_q] fp32 if wanted)."""
    d = attn_desc(Q, KV, idx, d_v, v_off, sm_scale)
    _check(lib().ic_sparse_attn_static(C.byref(d), _ptr(Q), _ptr(KV), _ptr(idx), _ptr(out), _ptr(lse), _stream(stream)))
    return out


def paged_cache(seq_lens=None, page_table=None, page_size=0):
    """ic_paged_cache from device tensors: seq_lens [B] int32 and/or page_table [B, max_pages] int32.
    The returned struct keeps the tensors alive."""
    import torch
    if seq_lens is not None:
        _need(seq_lens, "seq_lens", torch.int32, 1)
    if page_table is not None:
        _need(page_table, "page_table", torch.int32, 2)
    pc = PagedCache(page_size, page_table.shape[1] if page_table is not None else 0,
                    page_table.data_ptr() if page_table is not None else None,
                    seq_lens.data_ptr() if seq_lens is not None else None)
    pc._keep = (seq_lens, page_table)
    return pc


def indexer_topk_paged(q, k_pool, w, k_sel, Lk, pc, want_scores=False, workspace=None, stream=None):
    """ic_indexer_topk_paged: q [B,Tq,H_I,d_I], k_pool [rows, d_I] (paged) or [B,Lk,d_I] (ragged only),
    Lk = bound on the sequence lengths.  Returns idx of LOGICAL positions (and the selected scores)."""
    import torch
    _need(q, "q", ndim=4)
    _need(w, "w", torch.float32, 3)
    B, Tq, H, d = q.shape
    desc = IndexerDesc(B, Tq, Lk, H, d, k_sel, 0, _dtype_code(q), 0, None, None)
    if workspace is None:
        workspace = _workspace(indexer_topk_workspace(desc), q)
    idx = torch.empty((B, Tq, k_sel), dtype=torch.int32, device=q.device)
    sel = torch.empty((B, Tq, k_sel), dtype=torch.float32, device=q.device) if want_scores else None
    _check(lib().ic_indexer_topk_paged(C.byref(desc), C.byref(pc), _ptr(q), _ptr(k_pool), _ptr(w), _ptr(idx), _ptr(sel),
                                       _ptr(workspace), workspace.numel(), _stream(stream)))
    return (idx, sel) if want_scores else idx


def sparse_attn_paged(Q, KV_pool, idx, Lk, d_v, v_off, sm_scale, pc, want_lse=False, workspace=None, stream=None):
    """ic_sparse_attn_paged: Q [B,Tq,H_q,d_qk], KV_pool [rows, row_elems] (paged) or [B,Lk,row_elems]."""
    import torch
    _need(Q, "Q", torch.bfloat16, 4)
    _need(KV_pool, "KV_pool", torch.bfloat16)
    _need(idx, "idx", torch.int32, 3)
    B, Tq, Hq, d_qk = Q.shape
    d = AttnDesc(B, Tq, Lk, Hq, d_qk, d_v, v_off, KV_pool.shape[-1], idx.shape[2], sm_scale)
    if workspace is None:
        workspace = _workspace(sparse_attn_workspace(d), Q)
    O = torch.empty((B, Tq, Hq, d_v), dtype=torch.bfloat16, device=Q.device)
    lse = torch.empty((B, Tq, Hq), dtype=torch.float32, device=Q.device) if want_lse else None
    _check(lib().ic_sparse_attn_paged(C.byref(d), C.byref(pc), _ptr(Q), _ptr(KV_pool), _ptr(idx), _ptr(O), _ptr(lse),
                                      _ptr(workspace), workspace.numel(), _stream(stream)))
    return (O, lse) if want_lse else O


def forward_stack_paged(layer_arr, full_mask, pc, idx_cache, workspace, stream=None):
    """ic_forward_stack_paged: as forward_stack, every layer's k / KV being a pool laid out by pc.
    Build layer_arr with make_layers(..., Lk=bound)."""
    mask = bytes(bytearray(int(bool(m)) for m in full_mask))
    if len(mask) != len(layer_arr):
        raise IcError(Status.ERR_SHAPE, "full_mask has %d entries for %d layers" % (len(mask), len(layer_arr)))
    _check(lib().ic_forward_stack_paged(layer_arr, len(layer_arr), mask, C.byref(pc), _ptr(idx_cache),
                                        _ptr(workspace), workspace.numel(), _stream(stream)))


def make_layers(layers, k_sel, q_pos0, d_v, v_off, sm_scale, outs, Lk=None):
    """Build the host array of ic_layer from per-layer tensor dicts (q,k,w may be absent on
    Shared layers) and output tensors.  The returned object keeps the tensors alive.
    Lk: bound on the sequence lengths when k / KV are page pools (forward_stack_paged);
    by default the length is the caches' second dimension."""
    arr = (Layer * len(layers))()
    keep = []
    for l, (t, O) in enumerate(zip(layers, outs)):
        Q, KV = t["Q"], t["KV"]
        B, Tq, Hq, d_qk = Q.shape
        arr[l].at = AttnDesc(B, Tq, KV.shape[1] if Lk is None else Lk, Hq, d_qk, d_v, v_off, KV.shape[-1], k_sel, sm_scale)
        arr[l].Q, arr[l].KV, arr[l].O = Q.data_ptr(), KV.data_ptr(), O.data_ptr()
        if t.get("q") is not None:
            if Lk is None:
                arr[l].ix = indexer_desc(t["q"], t["k"], t["w"], k_sel, q_pos0, t.get("q_scale"), t.get("k_scale"))
            else:
                arr[l].ix = IndexerDesc(B, Tq, Lk, t["q"].shape[2], t["q"].shape[3], k_sel, 0, _dtype_code(t["q"]), 0, None, None)
            arr[l].q, arr[l].k, arr[l].w = t["q"].data_ptr(), t["k"].data_ptr(), t["w"].data_ptr()
        keep.append((t, O))
    arr._keep = keep
    return arr


def forward_stack_workspace(layer_arr):
    return int(lib().ic_forward_stack_workspace(layer_arr, len(layer_arr)))


def forward_stack(layer_arr, full_mask, idx_cache, workspace, stream=None):
    """ic_forward_stack over a host array built by make_layers.  full_mask: bytes / list of 0/1."""
    mask = bytes(bytearray(int(bool(m)) for m in full_mask))
    if len(mask) != len(layer_arr):
        raise IcError(Status.ERR_SHAPE, "full_mask has %d entries for %d layers" % (len(mask), len(layer_arr)))
    _check(lib().ic_forward_stack(layer_arr, len(layer_arr), mask, _ptr(idx_cache),
                                  _ptr(workspace), workspace.numel(), _stream(stream)))


def pattern_from_string(fs):
    buf = C.create_string_buffer(max(len(fs), 1))
    _check(lib().ic_pattern_from_string(fs.encode(), buf, len(fs)))
    return [b != 0 for b in buf.raw[:len(fs)]]


def pattern_uniform(n, r):
    buf = C.create_string_buffer(max(n, 1))
    _check(lib().ic_pattern_uniform(n, r, buf))
    return [b != 0 for b in buf.raw[:n]]


def topk_overlap(idx_layers, Lk, workspace=None, stream=None):
    """ic_topk_overlap over a list of index tensors [..., k_sel] int32 of one shape.
    Returns (overlap [n,n] float64, inter [n,n] int64, sizes [n] int64), all on the device."""
    import torch
    n = len(idx_layers)
    if n == 0:
        raise IcError(Status.ERR_SHAPE, "no index tensors")
    first = idx_layers[0]
    for t in idx_layers:
        _need(t, "idx", torch.int32)
        if t.shape != first.shape:
            raise IcError(Status.ERR_SHAPE, "index tensors must share one shape")
    k_sel = first.shape[-1]
    nq = first.numel() // k_sel
    if workspace is None:
        workspace = _workspace(int(lib().ic_topk_overlap_workspace(n)), first)
    ov = torch.empty((n, n), dtype=torch.float64, device=first.device)
    inter = torch.empty((n, n), dtype=torch.int64, device=first.device)
    sizes = torch.empty((n,), dtype=torch.int64, device=first.device)
    ptrs = (C.c_void_p * n)(*[t.data_ptr() for t in idx_layers])
    _check(lib().ic_topk_overlap(ptrs, n, nq, k_sel, Lk, _ptr(ov), _ptr(inter), _ptr(sizes),
                                 _ptr(workspace), workspace.numel(), _stream(stream)))
    return ov, inter, sizes


def cosine_rows(A, B, want_rows=False, stream=None):
    """ic_cosine_rows: mean per-row cosine similarity of two bf16 tensors shaped [n_rows, row_len].
    Returns a 0-d float64 device tensor (and the per-row float32 values if want_rows)."""
    import torch
    _need(A, "A", torch.bfloat16, 2)
    _need(B, "B", torch.bfloat16, 2)
    if A.shape != B.shape:
        raise IcError(Status.ERR_SHAPE, "A %s and B %s differ in shape" % (tuple(A.shape), tuple(B.shape)))
    mean = torch.empty((), dtype=torch.float64, device=A.device)
    rows = torch.empty((A.shape[0],), dtype=torch.float32, device=A.device) if want_rows else None
    ws = _workspace(int(lib().ic_cosine_rows_workspace()), A)
    _check(lib().ic_cosine_rows(_ptr(A), _ptr(B), A.shape[0], A.shape[1], _ptr(mean), _ptr(rows),
                                _ptr(ws), ws.numel(), _stream(stream)))
    return (mean, rows) if want_rows else mean


def similarity_matrix(layer_arr, idx_layers, workspace=None, stream=None):
    """ic_similarity_matrix over a host array built by make_layers (attention part) and one index
    tensor per layer.  Returns S [n,n] float64 on the device (lower triangle; diagonal 1)."""
    import torch
    n = len(layer_arr)
    if len(idx_layers) != n:
        raise IcError(Status.ERR_SHAPE, "%d index tensors for %d layers" % (len(idx_layers), n))
    for t in idx_layers:
        _need(t, "idx", torch.int32, 3)
    if workspace is None:
        workspace = _workspace(int(lib().ic_similarity_matrix_workspace(layer_arr, n)), idx_layers[0])
    S = torch.empty((n, n), dtype=torch.float64, device=idx_layers[0].device)
    ptrs = (C.c_void_p * n)(*[t.data_ptr() for t in idx_layers])
    _check(lib().ic_similarity_matrix(layer_arr, n, ptrs, _ptr(S), _ptr(workspace), workspace.numel(), _stream(stream)))
    return S


def pattern_search_dp(S, n_full):
    """ic_pattern_search_dp (host): S is an [n,n] array-like of floats (lower triangle used).
    Returns (list of bools, True = Full; total similarity)."""
    rows = [list(map(float, r)) for r in S]
    n = len(rows)
    flat = (C.c_double * (n * n))(*[rows[i][j] for i in range(n) for j in range(n)])
    buf = C.create_string_buffer(max(n, 1))
    total = C.c_double(0.0)
    _check(lib().ic_pattern_search_dp(flat, n, n_full, buf, C.byref(total)))
    return [b != 0 for b in buf.raw[:n]], float(total.value)


def pattern_search_greedy(S, n_shared, n_blocks=1):
    """ic_pattern_search_greedy (host): Alg. 1 on a similarity matrix.  Returns (mask as list of
    bools, True = Full; flipped layers in commit order; loss after each commit)."""
    rows = [list(map(float, r)) for r in S]
    n = len(rows)
    flat = (C.c_double * (n * n))(*[rows[i][j] for i in range(n) for j in range(n)])
    buf = C.create_string_buffer(max(n, 1))
    order = (C.c_int32 * max(n_shared, 1))()
    curve = (C.c_double * max(n_shared, 1))()
    _check(lib().ic_pattern_search_greedy(flat, n, n_shared, n_blocks, buf, order, curve))
    return [b != 0 for b in buf.raw[:n]], list(order[:n_shared]), list(curve[:n_shared])


def pattern_loss(layer_arr, full_mask, O_ref, idx_cache, workspace=None, stream=None):
    """ic_pattern_loss: run the stack under full_mask and compare with the all-Full outputs O_ref
    (list of device tensors).  Returns the loss as a device float64 scalar tensor."""
    import torch
    n = len(layer_arr)
    mask = bytes(bytearray(int(bool(m)) for m in full_mask))
    if len(mask) != n or len(O_ref) != n:
        raise IcError(Status.ERR_SHAPE, "mask / O_ref length differs from the %d layers" % n)
    if workspace is None:
        workspace = _workspace(int(lib().ic_pattern_loss_workspace(layer_arr, n)), idx_cache)
    loss = torch.empty((), dtype=torch.float64, device=idx_cache.device)
    ptrs = (C.c_void_p * n)(*[t.data_ptr() for t in O_ref])
    _check(lib().ic_pattern_loss(layer_arr, n, mask, ptrs, _ptr(idx_cache), _ptr(loss), _ptr(workspace), workspace.numel(),
                                 _stream(stream)))
    return loss


def greedy_search_forward(layer_arr, n_shared, O_ref, idx_cache, n_blocks=1, workspace=None, stream=None):
    """ic_greedy_search_forward: Alg. 1 with one forward pass of the stack per candidate.
    Synchronises the stream once per search step.  Returns (mask, order, loss curve)."""
    n = len(layer_arr)
    if len(O_ref) != n:
        raise IcError(Status.ERR_SHAPE, "O_ref length differs from the %d layers" % n)
    if workspace is None:
        workspace = _workspace(int(lib().ic_greedy_search_forward_workspace(layer_arr, n)), idx_cache)
    ptrs = (C.c_void_p * n)(*[t.data_ptr() for t in O_ref])
    buf = C.create_string_buffer(max(n, 1))
    order = (C.c_int32 * max(n_shared, 1))()
    curve = (C.c_double * max(n_shared, 1))()
    _check(lib().ic_greedy_search_forward(layer_arr, n, n_shared, n_blocks, ptrs, _ptr(idx_cache), buf, order, curve,
                                          _ptr(workspace), workspace.numel(), _stream(stream)))
    return [b != 0 for b in buf.raw[:n]], list(order[:n_shared]), list(curve[:n_shared])


def attn_probs(Q, KV, idx, sm_scale, lse, stream=None):
    """ic_attn_probs: head-aggregated attention probabilities over the selected rows, [B,Tq,k_sel]
    fp32.  lse: what sparse_attn(..., want_lse=True) returned for the same Q, KV, idx."""
    import torch
    _need(lse, "lse", torch.float32, 3)
    d = attn_desc(Q, KV, idx, 512 if Q.shape[3] == 576 else Q.shape[3], 0, sm_scale)   # the value layout plays no role here
    probs = torch.empty(tuple(idx.shape), dtype=torch.float32, device=Q.device)
    _check(lib().ic_attn_probs(C.byref(d), _ptr(Q), _ptr(KV), _ptr(idx), _ptr(lse), _ptr(probs), _stream(stream)))
    return probs


def distill_loss(probs, sel_scores, want_grad=False, workspace=None, stream=None):
    """ic_distill_loss: probs = list of [B,Tq,k_sel] fp32 targets (the Full layer and the Shared layers
    it serves), sel_scores = the Full layer's selected indexer scores.  Returns device float64
    scalars (loss_multi, loss_avg) and, if asked, the gradient with respect to the logits."""
    import torch
    _need(sel_scores, "sel_scores", torch.float32, 3)
    for p in probs:
        _need(p, "probs", torch.float32, 3)
        if tuple(p.shape) != tuple(sel_scores.shape):
            raise IcError(Status.ERR_SHAPE, "probs %s vs sel_scores %s" % (tuple(p.shape), tuple(sel_scores.shape)))
    nq, k_sel = sel_scores.shape[0] * sel_scores.shape[1], sel_scores.shape[2]
    if workspace is None:
        workspace = _workspace(int(lib().ic_distill_loss_workspace(nq)), sel_scores)
    lm = torch.empty((), dtype=torch.float64, device=sel_scores.device)
    la = torch.empty((), dtype=torch.float64, device=sel_scores.device)
    grad = torch.empty_like(sel_scores) if want_grad else None
    ptrs = (C.c_void_p * len(probs))(*[p.data_ptr() for p in probs])
    _check(lib().ic_distill_loss(ptrs, len(probs), _ptr(sel_scores), nq, k_sel, _ptr(lm), _ptr(la), _ptr(grad),
                                 _ptr(workspace), workspace.numel(), _stream(stream)))
    return (lm, la, grad) if want_grad else (lm, la)


def debug_indexer_scores(q, k, w, q_pos0, row0, n_rows, q_scale=None, k_scale=None, stream=None):
    """ic_debug_indexer_scores: fp32 [B,n_rows,Lk], hidden keys -inf."""
    import torch
    d = indexer_desc(q, k, w, 1, q_pos0, q_scale, k_scale)
    out = torch.empty((d.B, n_rows, d.Lk), dtype=torch.float32, device=q.device)
    _check(lib().ic_debug_indexer_scores(C.byref(d), _ptr(q), _ptr(k), _ptr(w), row0, n_rows,
                                         _ptr(out), _stream(stream)))
    return out


def debug_indexer_launch_count():
    return int(lib().ic_debug_indexer_launch_count())


def prof_enable(on):
    lib().ic_prof_enable(1 if on else 0)


def prof_collect():
    _check(lib().ic_prof_collect())


def prof_get(which):
    n, ms = C.c_int64(), C.c_double()
    _check(lib().ic_prof_get(which, C.byref(n), C.byref(ms)))
    return n.value, ms.value


def prof_reset():
    lib().ic_prof_reset()
