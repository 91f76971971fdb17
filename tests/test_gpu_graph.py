"""GPU: the layer loop is capturable.  ic_forward_stack allocates nothing, clears nothing with a
memset and never synchronises, so a decode step (one launch sequence per token) can be recorded in
a HIP graph and replayed.  The test replays it several times, with eager work and new inputs
between the replays, and compares every replay bit for bit with the eager call on the same inputs."""
import sys

import pytest
import torch

import synth

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


def _decode_cfg():
    cfg = dict(synth.config("c2"))
    cfg.update(B=4, Lk=4096, q_pos0=4095, k_sel=512, n_layers=4, pattern="FSSS")
    return cfg


def test_decode_step_replayed_from_a_graph(ic):
    cfg = _decode_cfg()
    say("graph replay of a decode step: B=%d ctx=%d layers=%s" % (cfg["B"], cfg["Lk"], cfg["pattern"]))
    layers = [{k: v.cuda() for k, v in l.items()} for l in synth.stack_layers(cfg)]
    mask = ic.pattern_from_string(cfg["pattern"])
    B, Tq, ks = cfg["B"], cfg["Tq"], cfg["k_sel"]

    def buffers():
        outs = [torch.zeros((B, Tq, cfg["H_q"], cfg["d_v"]), dtype=torch.bfloat16, device="cuda") for _ in layers]
        idx = torch.full((B, Tq, ks), -7, dtype=torch.int32, device="cuda")
        return outs, idx

    outs_e, idx_e = buffers()
    outs_g, idx_g = buffers()
    arr_e = ic.make_layers(layers, ks, cfg["q_pos0"], cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg), outs_e)
    arr_g = ic.make_layers(layers, ks, cfg["q_pos0"], cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg), outs_g)
    nws = max(ic.forward_stack_workspace(arr_e), 256)
    ws_e = torch.empty(nws, dtype=torch.uint8, device="cuda")
    ws_g = torch.empty(nws, dtype=torch.uint8, device="cuda")

    # eager once first: one-time function attributes are set outside the capture
    ic.forward_stack(arr_e, mask, idx_e, ws_e)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ic.forward_stack(arr_g, mask, idx_g, ws_g)       # the binding launches on torch's current (capturing) stream
    torch.cuda.synchronize()

    gen = torch.Generator(device="cuda").manual_seed(11)
    for rep in range(4):
        if rep:
            # new token: fresh query-side inputs, written in place (the graph holds the addresses)
            for l in layers:
                l["Q"].copy_(torch.randn(l["Q"].shape, generator=gen, device="cuda").to(l["Q"].dtype))
                if l.get("q") is not None:
                    l["q"].copy_((torch.randn(l["q"].shape, generator=gen, device="cuda") / 11.3).to(l["q"].dtype))
        for o in outs_g:
            o.fill_(1.0)                                  # eager work between the replays
        idx_g.fill_(-9)
        ic.forward_stack(arr_e, mask, idx_e, ws_e)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(idx_g, idx_e), "replay %d: index cache differs" % rep
        for l, (a, b) in enumerate(zip(outs_g, outs_e)):
            assert torch.equal(a, b), "replay %d: layer %d output differs" % (rep, l)
    assert int((idx_e >= 0).sum()) == B * Tq * ks
