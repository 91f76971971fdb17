"""GPU parity for the ragged / paged cache entry points (decode with the KV cache filled,
Sec. 4.3): per-sequence logical tensors are scattered into page pools through a random page
permutation; the oracle is run per sequence on the logical tensors (it knows nothing of pages)."""
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


def _page_table(seed, seq_lens, page_size, max_pages, spare=3):
    """Random assignment of distinct physical pages to the logical pages in use; unused entries
    name a spare page, whose rows hold the pool's fill value (reading one would wreck a result)."""
    rng = np.random.default_rng(seed)
    need = [(-(-int(n) // page_size)) for n in seq_lens]
    n_phys = sum(need) + spare
    perm = rng.permutation(n_phys)
    pt = np.full((len(seq_lens), max_pages), perm[-1], dtype=np.int32)   # a spare page: rows of the fill value
    o = 0
    for b, n in enumerate(need):
        pt[b, :n] = perm[o:o + n]
        o += n
    return pt, n_phys


def _to_pool(logical, pt, page_size, n_phys, fill):
    """logical: list over sequences of [len_b, width] tensors -> pool [n_phys * page_size, width];
    rows no sequence owns are filled with `fill` (a large value that would wreck a result)."""
    width = logical[0].shape[1]
    pool = torch.full((n_phys * page_size, width), fill, dtype=logical[0].dtype)
    for b, t in enumerate(logical):
        for s0 in range(0, t.shape[0], page_size):
            n = min(page_size, t.shape[0] - s0)
            r0 = int(pt[b, s0 // page_size]) * page_size
            pool[r0:r0 + n] = t[s0:s0 + n]
    return pool


def _mk_seqs(seed, seq_lens, Tq, H, d):
    g = torch.Generator().manual_seed(seed)
    B = len(seq_lens)
    q = (torch.randn((B, Tq, H, d), generator=g) / math.sqrt(d)).to(torch.bfloat16)
    w = torch.rand((B, Tq, H), generator=g).float()
    ks = [torch.randn((int(n), d), generator=g).to(torch.bfloat16) for n in seq_lens]
    return q, w, ks


def _dense(logical, Lk, fill):
    out = torch.full((len(logical), Lk, logical[0].shape[1]), fill, dtype=logical[0].dtype)
    for b, t in enumerate(logical):
        out[b, :t.shape[0]] = t
    return out


def _oracle_idx_check(oracle, q, w, ks, seq_lens, Tq, k_sel, got):
    for b, n in enumerate(seq_lens):
        n = int(n)
        p0 = n - Tq
        if n == 0:                       # an empty sequence selects nothing
            assert np.all(got[b] == -1)
            continue
        sc = oracle.indexer_scores(synth.bits(q[b:b + 1]), synth.bits(ks[b][None]), synth.bits(w[b:b + 1]), p0)
        for i in range(Tq):
            parity.check_idx_row(got[b, i], sc[0, i], max(0, min(n, p0 + i + 1)), k_sel, oracle)


INDEXER_CASES = [
    # seq_lens, Tq, H, d, k_sel, page_size (0: ragged only), bound Lk
    ([300, 65, 1, 129, 256], 1, 32, 128, 64, 64, 320),       # decode: one row per sequence, partial last pages
    ([200, 450, 77], 1, 32, 128, 128, 128, 512),             # a sequence shorter than k_sel
    ([300, 200, 250], 5, 32, 128, 64, 64, 300),              # several new tokens per sequence (speculative / chunked)
    ([300, 65, 129, 256], 1, 32, 128, 64, 0, 300),           # ragged lengths in a dense [B, Lk, d] cache
    ([40, 33], 3, 4, 64, 16, 64, 64),                        # tiny-config head shape
    ([0, 130, 64], 1, 32, 128, 32, 64, 192),                 # an empty sequence (owns no page)
    ([9000, 5000, 8200], 1, 32, 128, 512, 256, 9000),        # rows longer than one select tile
    ([40000, 33000, 2100], 1, 32, 128, 2048, 64, 40000),     # candidate-form select range, k = 2048
]


@pytest.mark.parametrize("case", INDEXER_CASES)
def test_indexer_topk_paged(ic, oracle, case):
    seq_lens, Tq, H, d, k_sel, page, Lk = case
    say("paged indexer lens=%s Tq=%d H=%d d=%d k=%d page=%d Lk=%d" % (seq_lens, Tq, H, d, k_sel, page, Lk))
    q, w, ks = _mk_seqs(900 + len(seq_lens) + Tq + page, seq_lens, Tq, H, d)
    sl = torch.tensor(seq_lens, dtype=torch.int32).cuda()
    if page:
        max_pages = -(-Lk // page) + 1
        pt, n_phys = _page_table(5 + page, seq_lens, page, max_pages)
        pool = _to_pool(ks, pt, page, n_phys, 60.0).cuda()
        pc = ic.paged_cache(sl, torch.from_numpy(pt).cuda(), page)
    else:
        pool = _dense(ks, Lk, 60.0).cuda()
        pc = ic.paged_cache(sl)
    idx = ic.indexer_topk_paged(q.cuda(), pool, w.cuda(), k_sel, Lk, pc)
    torch.cuda.synchronize()
    _oracle_idx_check(oracle, q, w, ks, seq_lens, Tq, k_sel, idx.cpu().numpy())


def test_indexer_topk_paged_equal_lengths_follow_q_pos0(ic, oracle):
    # page table only: every sequence has Lk positions and q_pos0 places the query rows
    B, Tq, Lk, H, d, k_sel, page, p0 = 2, 7, 200, 32, 128, 32, 64, 150
    say("paged indexer without seq_lens")
    q, w, ks = _mk_seqs(31, [Lk] * B, Tq, H, d)
    pt, n_phys = _page_table(8, [Lk] * B, page, 4)
    pool = _to_pool(ks, pt, page, n_phys, 60.0).cuda()
    pc = ic.paged_cache(None, torch.from_numpy(pt).cuda(), page)
    import ctypes as C
    from paper_2603_12201_amd import binding as bd
    desc = bd.IndexerDesc(B, Tq, Lk, H, d, k_sel, p0, bd.BF16, 0, None, None)
    ws = torch.empty(bd.indexer_topk_workspace(desc), dtype=torch.uint8, device="cuda")
    idx = torch.empty((B, Tq, k_sel), dtype=torch.int32, device="cuda")
    qd, wd = q.cuda(), w.cuda()
    st = bd.lib().ic_indexer_topk_paged(C.byref(desc), C.byref(pc), qd.data_ptr(), pool.data_ptr(), wd.data_ptr(),
                                        idx.data_ptr(), None, ws.data_ptr(), ws.numel(), None)
    assert st == 0, bd.last_error()
    torch.cuda.synchronize()
    got = idx.cpu().numpy()
    for b in range(B):
        sc = oracle.indexer_scores(synth.bits(q[b:b + 1]), synth.bits(ks[b][None]), synth.bits(w[b:b + 1]), p0)
        for i in range(Tq):
            parity.check_idx_row(got[b, i], sc[0, i], min(Lk, p0 + i + 1), k_sel, oracle)


def _rand_idx_ragged(seed, seq_lens, Tq, k_sel, holes):
    rng = np.random.default_rng(seed)
    idx = np.full((len(seq_lens), Tq, k_sel), -1, dtype=np.int32)
    for b, n in enumerate(seq_lens):
        for i in range(Tq):
            nv = max(0, int(n) - Tq + i + 1)
            m = min(nv, k_sel)
            idx[b, i, :m] = np.sort(rng.choice(nv, size=m, replace=False))
            if holes and m > 3:
                idx[b, i, rng.choice(m, size=m // 3, replace=False)] = -1
    return idx


ATTN_CASES = [
    # seq_lens, Tq, Hq, d_qk, d_v, v_off, row, k_sel, page_size, Lk, holes
    ([300, 65, 1, 129], 1, 32, 576, 512, 0, 576, 64, 64, 320, False),     # decode form (split + merge)
    ([500, 210], 3, 32, 576, 512, 0, 576, 256, 128, 512, True),
    ([300, 65, 129], 1, 32, 576, 512, 0, 576, 64, 0, 300, False),         # ragged only
    ([90, 70], 5, 16, 64, 64, 64, 128, 70, 64, 128, True),                # [K | V] rows
    ([700, 650], 300, 32, 576, 512, 0, 576, 200, 64, 704, True),          # >= 512 queries: one workgroup per query
    ([0, 130], 1, 32, 576, 512, 0, 576, 64, 64, 192, False),              # an empty sequence: zero output
]


@pytest.mark.parametrize("case", ATTN_CASES)
def test_sparse_attn_paged(ic, oracle, case):
    seq_lens, Tq, Hq, d_qk, d_v, v_off, row, k_sel, page, Lk, holes = case
    say("paged attn lens=%s Tq=%d Hq=%d k=%d page=%d Lk=%d" % (seq_lens, Tq, Hq, k_sel, page, Lk))
    g = torch.Generator().manual_seed(700 + Tq + k_sel)
    B = len(seq_lens)
    Q = torch.randn((B, Tq, Hq, d_qk), generator=g).to(torch.bfloat16)
    KVs = [torch.randn((int(n), row), generator=g).to(torch.bfloat16) for n in seq_lens]
    idx = _rand_idx_ragged(41 + Tq, seq_lens, Tq, k_sel, holes)
    # one entry beyond each sequence's own length (but inside the bound) must be skipped, not read
    idx_dev = idx.copy()
    for b, n in enumerate(seq_lens):
        if n < Lk and k_sel > min(n, k_sel):
            idx_dev[b, 0, k_sel - 1] = n
    sl = torch.tensor(seq_lens, dtype=torch.int32).cuda()
    if page:
        max_pages = -(-Lk // page)
        pt, n_phys = _page_table(17 + page, seq_lens, page, max_pages)
        pool = _to_pool(KVs, pt, page, n_phys, 3.0e4).cuda()
        pc = ic.paged_cache(sl, torch.from_numpy(pt).cuda(), page)
    else:
        pool = _dense(KVs, Lk, 3.0e4).cuda()
        pc = ic.paged_cache(sl)
    scale = 1.0 / math.sqrt(d_qk)
    O, lse = ic.sparse_attn_paged(Q.cuda(), pool, torch.from_numpy(idx_dev).cuda(), Lk, d_v, v_off, scale, pc, want_lse=True)
    torch.cuda.synchronize()
    Oc, lc = O.float().cpu().numpy(), lse.cpu().numpy()
    for b in range(B):
        if seq_lens[b] == 0:
            assert np.all(Oc[b] == 0) and np.all(np.isneginf(lc[b]))
            continue
        want, want_lse = oracle.sparse_attn(synth.bits(Q[b:b + 1]), synth.bits(KVs[b][None]), idx[b:b + 1], d_v, v_off, scale)
        parity.check_attn(Oc[b:b + 1], want)
        assert np.allclose(lc[b:b + 1], want_lse, rtol=0, atol=2e-2)


def test_forward_stack_paged_decode(ic, oracle):
    # FSSF pattern, batch of ragged sequences, every layer with its own pools behind one page table
    seq_lens, Tq, page, Lk, k_sel = [700, 130, 385, 64], 1, 64, 704, 96
    H, d, Hq, d_qk, d_v, row = 32, 128, 32, 576, 512, 576
    say("paged stack lens=%s" % (seq_lens,))
    B, n_layers = len(seq_lens), 4
    mask = ic.pattern_from_string("FSSF")
    pt, n_phys = _page_table(3, seq_lens, page, Lk // page)
    ptd = torch.from_numpy(pt).cuda()
    sl = torch.tensor(seq_lens, dtype=torch.int32).cuda()
    pc = ic.paged_cache(sl, ptd, page)
    scale = 1.0 / math.sqrt(d_qk)
    host, dev, outs = [], [], []
    for l in range(n_layers):
        q, w, ks = _mk_seqs(50 + l, seq_lens, Tq, H, d)
        g = torch.Generator().manual_seed(80 + l)
        Q = torch.randn((B, Tq, Hq, d_qk), generator=g).to(torch.bfloat16)
        KVs = [torch.randn((int(n), row), generator=g).to(torch.bfloat16) for n in seq_lens]
        host.append(dict(q=q, w=w, ks=ks, Q=Q, KVs=KVs))
        dev.append(dict(q=q.cuda(), w=w.cuda(), k=_to_pool(ks, pt, page, n_phys, 60.0).cuda(), Q=Q.cuda(),
                        KV=_to_pool(KVs, pt, page, n_phys, 3.0e4).cuda()))
        outs.append(torch.empty((B, Tq, Hq, d_v), dtype=torch.bfloat16, device="cuda"))
    arr = ic.make_layers(dev, k_sel, 0, d_v, 0, scale, outs, Lk=Lk)
    ws = torch.empty(ic.forward_stack_workspace(arr), dtype=torch.uint8, device="cuda")
    cache = torch.full((B, Tq, k_sel), -7, dtype=torch.int32, device="cuda")
    ic.forward_stack_paged(arr, mask, pc, cache, ws)
    torch.cuda.synchronize()
    # indices of each Full layer through the entry point the stack uses; the cache keeps the last
    gpu_idx = {l: ic.indexer_topk_paged(dev[l]["q"], dev[l]["k"], dev[l]["w"], k_sel, Lk, pc) for l in (0, 3)}
    torch.cuda.synchronize()
    assert torch.equal(cache, gpu_idx[3])
    for l, gi in gpu_idx.items():
        _oracle_idx_check(oracle, host[l]["q"], host[l]["w"], host[l]["ks"], seq_lens, Tq, k_sel, gi.cpu().numpy())
    for l in range(n_layers):
        used = gpu_idx[oracle.source_layer(list(mask), l)].cpu().numpy()
        h = host[l]
        for b in range(B):
            want, _ = oracle.sparse_attn(synth.bits(h["Q"][b:b + 1]), synth.bits(h["KVs"][b][None]), used[b:b + 1], d_v, 0, scale)
            parity.check_attn(outs[l][b:b + 1].float().cpu().numpy(), want)
