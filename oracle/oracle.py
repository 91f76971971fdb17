"""Python face of the CPU oracle (ctypes over oracle/libic_oracle.so) + the layer loop.

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg; never by the product package.  It imports nothing
from the product package either.

Array conventions (numpy, C-contiguous):
  q   [B,Tq,H_I,d_I]  uint16 (bfloat16 bit patterns) or uint8 (e4m3 bytes)
  k   [B,Lk,d_I]      same element type as q
  w   [B,Tq,H_I]      float32
  q_scale [B,Tq], k_scale [B,Lk] float32 (fp8 only)
  Q   [B,Tq,H_q,d_qk] uint16 ; KV [B,Lk,row_elems] uint16
  idx [B,Tq,k_sel]    int32, -1 padded
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

BF16, FP8_E4M3 = 0, 1


def lib():
    global _LIB
    if _LIB is None:
        path = os.path.join(_HERE, "libic_oracle.so")
        if not os.path.exists(path):
            from . import build as _b
            _b.build(force=True)
        _LIB = C.CDLL(path)
        _LIB.ico_widen_bf16.restype = C.c_double
        _LIB.ico_widen_bf16.argtypes = [C.c_uint16]
        _LIB.ico_widen_e4m3.restype = C.c_double
        _LIB.ico_widen_e4m3.argtypes = [C.c_uint8]
        _LIB.ico_num_threads.restype = C.c_int
    return _LIB


def num_threads():
    return int(lib().ico_num_threads())


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _rows(rows):
    if rows is None:
        return None, 0
    r = np.ascontiguousarray(np.asarray(rows, dtype=np.int32))
    return r, int(r.size)


def _check_indexer(q, k, w, dtype, q_scale, k_scale):
    et = np.uint16 if dtype == BF16 else np.uint8
    assert q.dtype == et and k.dtype == et, (q.dtype, k.dtype)
    assert w.dtype == np.float32
    assert q.ndim == 4 and k.ndim == 3 and w.ndim == 3
    B, Tq, H, d = q.shape
    assert k.shape[0] == B and k.shape[2] == d and w.shape == (B, Tq, H)
    for a in (q, k, w):
        assert a.flags.c_contiguous
    if dtype == FP8_E4M3:
        assert q_scale.dtype == np.float32 and q_scale.shape == (B, Tq)
        assert k_scale.dtype == np.float32 and k_scale.shape == (B, k.shape[1])
    return B, Tq, k.shape[1], H, d


def indexer_scores(q, k, w, q_pos0, dtype=BF16, q_scale=None, k_scale=None, rows=None):
    """I[b, r, s] in fp64 for the chosen query rows; hidden keys are -inf."""
    B, Tq, Lk, H, d = _check_indexer(q, k, w, dtype, q_scale, k_scale)
    r, n = _rows(rows)
    n_rows = n if r is not None else Tq
    out = np.empty((B, n_rows, Lk), dtype=np.float64)
    rc = lib().ico_indexer_scores(C.c_int(dtype), _p(q), _p(k), _p(w), _p(q_scale), _p(k_scale),
                                  C.c_int(B), C.c_int(Tq), C.c_int(Lk), C.c_int(H), C.c_int(d),
                                  C.c_long(q_pos0), _p(r), C.c_int(n_rows), _p(out))
    assert rc == 0, rc
    return out


def topk_row(scores, nv, k_sel):
    """Top-k of one scored row (first nv entries visible)."""
    scores = np.ascontiguousarray(scores, dtype=np.float64)
    idx = np.empty(k_sel, dtype=np.int32)
    sel = np.empty(k_sel, dtype=np.float64)
    kth, nxt, ma = C.c_double(), C.c_double(), C.c_double()
    rc = lib().ico_topk_row(_p(scores), C.c_int(nv), C.c_int(k_sel), _p(idx), _p(sel),
                            C.byref(kth), C.byref(nxt), C.byref(ma))
    assert rc == 0, rc
    return dict(idx=idx, sel=sel, kth=kth.value, next=nxt.value, mean_abs=ma.value)


def indexer_topk(q, k, w, q_pos0, k_sel, dtype=BF16, q_scale=None, k_scale=None, rows=None):
    """Indexer + top-k.  Returns idx [B,n_rows,k_sel] (score-descending, ties lower
    position first, -1 tail), sel (their fp64 scores), and per row: kth (last selected
    score), next (best unselected score or -inf), mean_abs (mean |I| over visible keys)."""
    B, Tq, Lk, H, d = _check_indexer(q, k, w, dtype, q_scale, k_scale)
    r, n = _rows(rows)
    n_rows = n if r is not None else Tq
    idx = np.empty((B, n_rows, k_sel), dtype=np.int32)
    sel = np.empty((B, n_rows, k_sel), dtype=np.float64)
    kth = np.empty((B, n_rows), dtype=np.float64)
    nxt = np.empty((B, n_rows), dtype=np.float64)
    ma = np.empty((B, n_rows), dtype=np.float64)
    rc = lib().ico_indexer_topk(C.c_int(dtype), _p(q), _p(k), _p(w), _p(q_scale), _p(k_scale),
                                C.c_int(B), C.c_int(Tq), C.c_int(Lk), C.c_int(H), C.c_int(d),
                                C.c_long(q_pos0), C.c_int(k_sel), _p(r), C.c_int(n_rows),
                                _p(idx), _p(sel), _p(kth), _p(nxt), _p(ma))
    assert rc == 0, rc
    return dict(idx=idx, sel=sel, kth=kth, next=nxt, mean_abs=ma)


def _check_attn(Q, KV, idx):
    assert Q.dtype == np.uint16 and KV.dtype == np.uint16 and idx.dtype == np.int32
    assert Q.ndim == 4 and KV.ndim == 3 and idx.ndim == 3
    for a in (Q, KV, idx):
        assert a.flags.c_contiguous
    B, Tq, Hq, d_qk = Q.shape
    assert KV.shape[0] == B and idx.shape[0] == B
    return B, Tq, KV.shape[1], Hq, d_qk, KV.shape[2], idx.shape[2]


def sparse_attn(Q, KV, idx, d_v, v_off, sm_scale, rows=None, idx_is_subset=False):
    """Sparse MQA attention over the rows named by idx.  Returns (O fp64 [B,n,Hq,d_v], lse)."""
    B, Tq, Lk, Hq, d_qk, row, k_sel = _check_attn(Q, KV, idx)
    r, n = _rows(rows)
    n_rows = n if r is not None else Tq
    assert idx.shape[1] == (n_rows if idx_is_subset else Tq)
    O = np.empty((B, n_rows, Hq, d_v), dtype=np.float64)
    lse = np.empty((B, n_rows, Hq), dtype=np.float64)
    rc = lib().ico_sparse_attn(_p(Q), _p(KV), _p(idx), C.c_int(B), C.c_int(Tq), C.c_int(Lk),
                               C.c_int(Hq), C.c_int(d_qk), C.c_int(d_v), C.c_int(v_off),
                               C.c_int(row), C.c_int(k_sel), C.c_double(sm_scale), _p(r),
                               C.c_int(n_rows), C.c_int(1 if idx_is_subset else 0), _p(O), _p(lse))
    assert rc == 0, rc
    return O, lse


def dense_causal_attn(Q, KV, d_v, v_off, sm_scale, q_pos0):
    """Textbook causal softmax attention over every visible key (pin for sparse_attn)."""
    assert Q.dtype == np.uint16 and KV.dtype == np.uint16
    B, Tq, Hq, d_qk = Q.shape
    Lk, row = KV.shape[1], KV.shape[2]
    O = np.empty((B, Tq, Hq, d_v), dtype=np.float64)
    rc = lib().ico_dense_causal_attn(_p(Q), _p(KV), C.c_int(B), C.c_int(Tq), C.c_int(Lk),
                                     C.c_int(Hq), C.c_int(d_qk), C.c_int(d_v), C.c_int(v_off),
                                     C.c_int(row), C.c_double(sm_scale), C.c_long(q_pos0), _p(O))
    assert rc == 0, rc
    return O


def topk_overlap(idx_layers, Lk):
    """Cross-layer overlap of the index sets (App. A).  idx_layers: list of int32 arrays
    [..., k_sel] of one shape.  Returns (overlap [n,n] float64 = inter / sizes[:,None],
    inter [n,n] uint64, sizes [n] uint64); overlap(i,j) = sum_t |T_t(i) ^ T_t(j)| / sum_t |T_t(i)|."""
    n = len(idx_layers)
    arrs = [np.ascontiguousarray(a, dtype=np.int32) for a in idx_layers]
    k_sel = arrs[0].shape[-1]
    nq = arrs[0].size // k_sel
    assert all(a.shape == arrs[0].shape for a in arrs)
    ptrs = (C.c_void_p * n)(*[a.ctypes.data for a in arrs])
    inter = np.zeros((n, n), dtype=np.uint64)
    sizes = np.zeros((n,), dtype=np.uint64)
    rc = lib().ico_topk_overlap(ptrs, C.c_int(n), C.c_long(nq), C.c_int(k_sel), C.c_int(Lk), _p(inter), _p(sizes))
    assert rc == 0, rc
    with np.errstate(divide="ignore", invalid="ignore"):
        ov = inter.astype(np.float64) / sizes.astype(np.float64)[:, None]
    return ov, inter, sizes


def cosine_rows(A, B):
    """Mean over the rows of the cosine similarity of corresponding rows of two bf16 tensors
    (uint16 bit patterns, same shape [..., row_len] flattened to [n_rows, row_len] by the caller).
    Returns (mean, per_row float64)."""
    assert A.dtype == np.uint16 and B.dtype == np.uint16 and A.shape == B.shape and A.ndim == 2
    A = np.ascontiguousarray(A); B = np.ascontiguousarray(B)
    per = np.empty((A.shape[0],), dtype=np.float64)
    mean = C.c_double(0.0)
    rc = lib().ico_cosine_rows(_p(A), _p(B), C.c_long(A.shape[0]), C.c_long(A.shape[1]), _p(per), C.byref(mean))
    assert rc == 0, rc
    return float(mean.value), per


def similarity_matrix(layers, idx_layers, d_v, v_off, sm_scale):
    """S[i, j], j < i: mean per-token cosine similarity between layer i's sparse attention under its
    own indices and under layer j's (App. C), from the fp64 attention outputs; diagonal 1, upper 0."""
    n = len(layers)
    S = np.eye(n)
    for i in range(n):
        own, _ = sparse_attn(layers[i]["Q"], layers[i]["KV"], idx_layers[i], d_v, v_off, sm_scale)
        a = own.reshape(-1, own.shape[-2] * own.shape[-1])
        for j in range(i):
            reuse, _ = sparse_attn(layers[i]["Q"], layers[i]["KV"], idx_layers[j], d_v, v_off, sm_scale)
            b = reuse.reshape(a.shape)
            na, nb = np.linalg.norm(a, axis=1), np.linalg.norm(b, axis=1)
            with np.errstate(divide="ignore", invalid="ignore"):
                cs = (a * b).sum(1) / (na * nb)
            cs = np.where((na == 0) & (nb == 0), 1.0, np.where((na == 0) | (nb == 0), 0.0, cs))
            S[i, j] = cs.mean()
    return S


def pattern_total(S, mask):
    """Objective of the similarity-based search (App. C): sum over the Shared layers l of
    S[l, src(l)], src(l) the nearest preceding Full layer."""
    tot = 0.0
    for l in range(len(mask)):
        if not mask[l]:
            tot += float(S[l, source_layer(mask, l)])
    return tot


def pattern_search_exhaustive(S, n_full):
    """argmax over every pattern with exactly n_full Full layers (the first one Full) of
    pattern_total: the definition written out, for small N.  Returns (best total, list of all
    patterns that reach it)."""
    import itertools
    N = S.shape[0]
    assert 1 <= n_full <= N
    best, arg = -np.inf, []
    for rest in itertools.combinations(range(1, N), n_full - 1):
        mask = [False] * N
        mask[0] = True
        for l in rest:
            mask[l] = True
        t = pattern_total(S, mask)
        if t > best + 1e-12:
            best, arg = t, [mask]
        elif abs(t - best) <= 1e-12:
            arg.append(mask)
    return best, arg


# ---- greedy layer selection (Alg. 1, Sec. 3.2) with a surrogate loss -----------------------

def pattern_loss_from_similarity(S, mask):
    """Stand-in for EvalLoss(M, D, c) of Alg. 1 (the language-model loss needs the model): the
    attention-output error of pattern c against the all-Full stack,
        loss(c) = 1/N * sum_l (1 - sim_l(c)),   sim_l(c) = mean per-token cosine of layer l's
    output under c and under all-Full.  With layers whose inputs do not depend on earlier outputs
    (the attention-only stack of this build) sim_l(c) = S[l, src(l)], so a Full layer adds 0."""
    N = len(mask)
    return sum(1.0 - float(S[l, source_layer(mask, l)]) for l in range(N) if not mask[l]) / N


def pattern_loss_forward(layers, full_mask, k_sel, q_pos0, d_v, v_off, sm_scale, O_ref):
    """The same loss measured the way Alg. 1 measures it: run the whole stack under the pattern
    (forward_stack) and compare every layer's output with the all-Full run's O_ref (fp64 arrays)."""
    outs, _, _ = forward_stack(layers, full_mask, k_sel, q_pos0, d_v, v_off, sm_scale)
    tot = 0.0
    for O, R in zip(outs, O_ref):
        a = O.reshape(-1, O.shape[-2] * O.shape[-1])
        b = R.reshape(a.shape)
        na, nb = np.linalg.norm(a, axis=1), np.linalg.norm(b, axis=1)
        with np.errstate(divide="ignore", invalid="ignore"):
            cs = (a * b).sum(1) / (na * nb)
        cs = np.where((na == 0) & (nb == 0), 1.0, np.where((na == 0) | (nb == 0), 0.0, cs))
        tot += 1.0 - cs.mean()
    return tot / len(layers)


def greedy_search(eval_loss, n_layers, n_shared, n_blocks=1):
    """Alg. 1: start from all-Full; n_shared times, try every remaining candidate layer as Shared,
    evaluate the loss of the resulting pattern and commit the flip with the lowest loss (ties:
    the lowest layer).  Layer 0 is never a candidate.  n_blocks > 1 is the pipeline-parallel
    variant of Sec. 3.2 (Complexity): the layers are cut into n_blocks contiguous blocks of
    ceil(N / n_blocks), the first layer of a block stays Full, and within one step the blocks are
    searched one after the other, each committing its own best flip before the next is searched.
    eval_loss(mask) -> float.  Returns (mask, order of flipped layers, loss after each flip)."""
    N = n_layers
    if not (0 <= n_shared <= N - 1) or n_blocks < 1:
        raise ValueError("need 0 <= n_shared <= N-1 and n_blocks >= 1")
    size = -(-N // n_blocks)
    blocks = [list(range(b0, min(b0 + size, N))) for b0 in range(0, N, size)]
    mask = [True] * N
    cand = [set(b[1:]) for b in blocks]                 # a block's first layer is fixed Full
    if n_shared > sum(len(c) for c in cand):
        raise ValueError("more Shared layers asked for than candidates exist")
    order, curve = [], []
    while len(order) < n_shared:
        for c in cand:
            if len(order) == n_shared or not c:
                continue
            best, arg = None, None
            for l in sorted(c):
                trial = list(mask)
                trial[l] = False
                v = eval_loss(trial)
                if best is None or v < best:
                    best, arg = v, l
            mask[arg] = False
            c.remove(arg)
            order.append(arg)
            curve.append(best)
    return mask, order, curve


# ---- multi-layer distillation loss (Sec. 3.3, Eq. 1 and Prop. 1) -------------------------

def _widen_bf16(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def indexer_distribution(scores):
    """q_t = Softmax(I_t) over the finite entries of each row (hidden keys / empty slots hold -inf
    and get probability 0).  scores [..., n] float64."""
    sc = np.asarray(scores, dtype=np.float64)
    m = np.max(np.where(np.isfinite(sc), sc, -np.inf), axis=-1, keepdims=True)
    m = np.where(np.isfinite(m), m, 0.0)
    e = np.where(np.isfinite(sc), np.exp(sc - m), 0.0)
    z = e.sum(-1, keepdims=True)
    return np.where(z > 0, e / np.where(z > 0, z, 1.0), 0.0)


def attn_distribution_dense(Q, KV, sm_scale, q_pos0):
    """p_t: the attention distribution of a layer aggregated over its heads (Sec. 2.1: the
    indexer's training target), p_t(s) = 1/H sum_h softmax_s(sm_scale * Q[t,h] . K[s]) over the
    causally visible keys s <= q_pos0 + t; K[s] = the first d_qk features of KV row s.
    Returns [B,Tq,Lk] float64 (0 on hidden keys)."""
    Qf, KVf = _widen_bf16(Q), _widen_bf16(KV)
    B, Tq, H, d = Qf.shape
    Lk = KVf.shape[1]
    P = np.zeros((B, Tq, Lk))
    for b in range(B):
        K = KVf[b, :, :d]
        for t in range(Tq):
            nv = max(0, min(Lk, q_pos0 + t + 1))
            if nv == 0:
                continue
            z = sm_scale * (Qf[b, t] @ K[:nv].T)                  # [H, nv]
            z -= z.max(axis=1, keepdims=True)
            e = np.exp(z)
            P[b, t, :nv] = (e / e.sum(axis=1, keepdims=True)).mean(axis=0)
    return P


def attn_distribution_selected(Q, KV, idx, sm_scale):
    """The same aggregated distribution when the layer attends only to the rows named by idx (a
    Full layer's own T_t, or the T_t a Shared layer inherits): softmax over the selected rows,
    mean over the heads.  Returns [B,Tq,k_sel] float64 in slot order (0 on empty slots)."""
    Qf, KVf = _widen_bf16(Q), _widen_bf16(KV)
    B, Tq, H, d = Qf.shape
    Lk = KVf.shape[1]
    P = np.zeros(idx.shape)
    for b in range(B):
        for t in range(Tq):
            slots = np.nonzero((idx[b, t] >= 0) & (idx[b, t] < Lk))[0]
            if slots.size == 0:
                continue
            z = sm_scale * (Qf[b, t] @ KVf[b, idx[b, t, slots], :d].T)   # [H, n]
            z -= z.max(axis=1, keepdims=True)
            e = np.exp(z)
            P[b, t, slots] = (e / e.sum(axis=1, keepdims=True)).mean(axis=0)
    return P


def kl_rows(p, q):
    """D_KL(p || q) per row = sum_s p(s) log(p(s) / q(s)), with 0 log 0 = 0 (inf if q = 0 < p)."""
    p, q = np.asarray(p, dtype=np.float64), np.asarray(q, dtype=np.float64)
    with np.errstate(divide="ignore", invalid="ignore"):
        t = np.where(p > 0, p * (np.log(p) - np.log(q)), 0.0)
    return t.sum(-1)


def distill_loss_multi(p_list, q):
    """Eq. 1: sum_j 1/(m+1) sum_t D_KL(p_t^(l+j) || q_t^(l)) for the m+1 layers a Full layer serves
    (itself and its m Shared followers).  p_list: m+1 arrays [..., n]; q [..., n]."""
    return sum(kl_rows(p, q).sum() for p in p_list) / len(p_list)


def distill_loss_avg(p_list, q):
    """Eq. 2: the single-target loss against the averaged distribution p_bar = mean_j p^(l+j)."""
    return kl_rows(sum(np.asarray(p, dtype=np.float64) for p in p_list) / len(p_list), q).sum()


def distill_grad_logits(p_list, q):
    """d/dI of either loss with respect to the indexer's logits (q = Softmax(I)): q_t * (row mass of
    p_bar) - p_bar_t, i.e. q - p_bar for normalised targets.  What Prop. 1 says is that Eq. 1 and
    Eq. 2 share it."""
    pb = sum(np.asarray(p, dtype=np.float64) for p in p_list) / len(p_list)
    return np.asarray(q, dtype=np.float64) * pb.sum(-1, keepdims=True) - pb


# ---- pattern strings and the layer loop (Fig. 2, Sec. 3 Overview) -------------

def pattern_from_string(s):
    """'FSSF..' -> list of bools (True = Full).  The first layer must be F (Sec. 3 Overview)."""
    mask = []
    for ch in s:
        if ch not in "FS":
            raise ValueError("pattern characters must be F or S: %r" % ch)
        mask.append(ch == "F")
    if not mask or not mask[0]:
        raise ValueError("the first layer must be F")
    return mask


def pattern_uniform(n, r):
    """Uniform interleave: keep every r-th indexer, FSSSFSSS... for r = 4 (Sec. 3.1)."""
    if n <= 0 or r <= 0:
        raise ValueError("n and r must be positive")
    return [(l % r) == 0 for l in range(n)]


def source_layer(mask, l):
    """f(l) = max{ j < l : c_j = F } for an S layer; l itself for an F layer."""
    if mask[l]:
        return l
    for j in range(l - 1, -1, -1):
        if mask[j]:
            return j
    raise ValueError("S layer with no preceding F layer")


def forward_stack(layers, full_mask, k_sel, q_pos0, d_v, v_off, sm_scale, dtype=BF16):
    """IndexCache inference loop (Fig. 2b) over attention-only layers.

    layers: list of dicts with q,k,w (may be absent on S layers) and Q,KV.
    F layer: T_cache <- Top-k(Indexer); S layer: T_cache untouched; then sparse attention
    with the layer's own Q/KV and T_cache.  Returns (list of O, list of the idx each layer used,
    number of indexer invocations)."""
    if not full_mask or not full_mask[0]:
        raise ValueError("the first layer must be F")
    t_cache = None
    outs, used, n_indexer = [], [], 0
    for l, layer in enumerate(layers):
        if full_mask[l]:
            t_cache = indexer_topk(layer["q"], layer["k"], layer["w"], q_pos0, k_sel, dtype,
                                   layer.get("q_scale"), layer.get("k_scale"))["idx"]
            n_indexer += 1
        O, _ = sparse_attn(layer["Q"], layer["KV"], t_cache, d_v, v_off, sm_scale)
        outs.append(O)
        used.append(t_cache)
    return outs, used, n_indexer
