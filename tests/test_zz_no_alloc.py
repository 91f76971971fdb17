"""The entry point that allocates nothing: ic_sparse_attn_static against ic_sparse_attn, through the C ABI."""
import ctypes as C
import math
import sys

import numpy as np
import pytest
import torch

from tests import parity
import synth


def say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


def test_static_scratch_rejects_oversized_shapes_without_a_gpu():
    import paper_2603_12201_amd as ic
    L, S = ic.lib(), ic.Status
    one = C.c_void_p(4096)
    # 255 queries x 2 splits x 32 heads x 512 values in bf16 is a little over 16 MiB of partials
    big = ic.AttnDesc(255, 1, 65536, 32, 576, 512, 0, 576, 2048, 1.0 / 24.0)
    assert L.ic_sparse_attn_workspace(C.byref(big)) > ic.STATIC_SCRATCH_BYTES
    assert L.ic_sparse_attn_static(C.byref(big), one, one, one, one, None, None) == S.ERR_WORKSPACE
    assert b"static scratch" in L.ic_last_error()
    ok = ic.AttnDesc(32, 1, 65536, 32, 576, 512, 0, 576, 2048, 1.0 / 24.0)
    assert 0 < L.ic_sparse_attn_workspace(C.byref(ok)) <= ic.STATIC_SCRATCH_BYTES
    assert L.ic_sparse_attn_static(C.byref(ok), None, one, one, one, None, None) == S.ERR_NULL
    bad = ic.AttnDesc(32, 1, 65536, 33, 576, 512, 0, 576, 2048, 1.0 / 24.0)
    assert L.ic_sparse_attn_static(C.byref(bad), one, one, one, one, None, None) == S.ERR_UNSUPPORTED


def _case(seed, B, Tq, Lk, ks):
    g = torch.Generator().manual_seed(seed)
    Q = torch.randn((B, Tq, 32, 576), generator=g).to(torch.bfloat16)
    KV = torch.randn((B, Lk, 576), generator=g).to(torch.bfloat16)
    rng = np.random.default_rng(seed)
    idx = np.full((B, Tq, ks), -1, dtype=np.int32)
    for b in range(B):
        for t in range(Tq):
            idx[b, t] = np.sort(rng.choice(Lk, size=ks, replace=False))
    idx[0, 0, ks // 2:] = -1                     # a row with empty slots
    return Q, KV, idx


@pytest.mark.gpu
def test_static_scratch_matches_the_workspace_entry_point_on_two_calls_in_a_row(oracle):
    import paper_2603_12201_amd as ic
    ic.lib()
    scale = 1.0 / math.sqrt(576)
    # first a decode-shaped call (8 queries x 32 splits), then a smaller one (3 queries, fewer rows): the
    # second call finds the first one's partials in the scratch and must not be disturbed by them
    for seed, B, Tq, Lk, ks in ((11, 8, 1, 3000, 2048), (12, 3, 1, 700, 320)):
        say("static scratch B=%d Tq=%d Lk=%d k=%d" % (B, Tq, Lk, ks))
        Q, KV, idx = _case(seed, B, Tq, Lk, ks)
        Qd, KVd, idxd = Q.cuda(), KV.cuda(), torch.from_numpy(idx).cuda()
        want_O, want_lse = ic.sparse_attn(Qd, KVd, idxd, 512, 0, scale, want_lse=True)
        out = torch.full((B, Tq, 32, 512), 7.0, dtype=torch.bfloat16, device="cuda")
        lse = torch.full((B, Tq, 32), 7.0, dtype=torch.float32, device="cuda")
        ic.sparse_attn_static(Qd, KVd, idxd, 512, 0, scale, out, lse)
        torch.cuda.synchronize()
        assert torch.equal(out, want_O) and torch.equal(lse, want_lse)        # same kernels, same bits
        ref, ref_lse = oracle.sparse_attn(synth.bits(Q), synth.bits(KV), idx, 512, 0, scale)
        parity.check_attn(out.float().cpu().numpy(), ref)
        assert np.allclose(lse.cpu().numpy(), ref_lse, rtol=0, atol=2e-2)
    # a shape that needs no scratch at all (one workgroup per query) goes through as well
    Q, KV, idx = _case(13, 1, 300, 400, 130)
    Qd, KVd, idxd = Q.cuda(), KV.cuda(), torch.from_numpy(idx).cuda()
    want_O = ic.sparse_attn(Qd, KVd, idxd, 512, 0, scale)
    out = torch.empty_like(want_O)
    ic.sparse_attn_static(Qd, KVd, idxd, 512, 0, scale, out)
    torch.cuda.synchronize()
    assert torch.equal(out, want_O)
