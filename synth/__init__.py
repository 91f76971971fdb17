"""Seeded synthetic inputs shaped like long-context DSA prefill / decode workloads.

This module only draws random tensors and packs them into the layouts the library
and the CPU oracle both read (it holds none of the method's arithmetic).  The same
bytes go to both sides: tensors are created here once, handed to the GPU library as
device pointers and to the oracle as numpy bit patterns (`bits`).

Recipe (per layer l, all streams derived from (seed, l, tensor name)):
  indexer  q[t,j,:] ~ N(0, 1/d_I) -> bf16          w[t,j] ~ U(0,1) fp32
           k_l[s,:] = sqrt(rho) k_base[s,:] + sqrt(1-rho) n_l[s,:], k_base, n_l ~ N(0,1) -> bf16
           (rho = 0.8 correlates the keys of different layers; rho = 0 gives plain N(0,1))
  attention Q ~ N(0,1) bf16; KV row ~ N(0,1) bf16 (MLA: 512 latent + 64 rope in one row;
           tiny config: separate K and V of 64 packed as one row [K | V])
  fp8      q and k are quantised per token to OCP e4m3 with scale = amax/448 (fp32).
"""
import math

import numpy as np
import torch

BASE_SEED = 2603122010

_TENSOR_ID = {"q": 1, "k_base": 2, "k_noise": 3, "w": 4, "Q": 5, "KV": 6, "q_chain": 7, "k_chain": 8}

# The workload shapes this build is measured and tested on.
CONFIGS = {
    # tiny stack the oracle finishes in seconds
    "c0": dict(kind="prefill", B=1, Tq=512, Lk=512, q_pos0=0, n_layers=4, pattern="FSFS",
               H_I=4, d_I=64, k_sel=64, H_q=4, d_qk=64, d_v=64, v_off=64, row_elems=128,
               dtype="bf16", rho=0.8, seed=BASE_SEED + 0),
    # single-layer indexer + top-k prefill
    "c1": dict(kind="prefill", B=1, Tq=16384, Lk=16384, q_pos0=0, n_layers=1, pattern="F",
               H_I=32, d_I=128, k_sel=2048, H_q=32, d_qk=576, d_v=512, v_off=0, row_elems=576,
               dtype="bf16", rho=0.0, seed=BASE_SEED + 1),
    # batched decode: the new token's key is already appended, so all 65536 keys are visible
    "c2": dict(kind="decode", B=32, Tq=1, Lk=65536, q_pos0=65535, n_layers=4, pattern="FSSS",
               H_I=32, d_I=128, k_sel=2048, H_q=32, d_qk=576, d_v=512, v_off=0, row_elems=576,
               dtype="bf16", rho=0.0, seed=BASE_SEED + 2),
    # 48-layer stack prefill (pattern chosen by the caller: all-F or 1-in-4)
    "c3": dict(kind="prefill", B=1, Tq=32768, Lk=32768, q_pos0=0, n_layers=48, pattern=None,
               H_I=32, d_I=128, k_sel=2048, H_q=32, d_qk=576, d_v=512, v_off=0, row_elems=576,
               dtype="bf16", rho=0.8, seed=BASE_SEED + 3),
    # long-context fp8 prefill
    "c4": dict(kind="prefill", B=1, Tq=131072, Lk=131072, q_pos0=0, n_layers=48, pattern=None,
               H_I=64, d_I=128, k_sel=2048, H_q=32, d_qk=576, d_v=512, v_off=0, row_elems=576,
               dtype="fp8", rho=0.8, seed=BASE_SEED + 4),
}


def config(name, **overrides):
    cfg = dict(CONFIGS[name])
    cfg.update(overrides)
    return cfg


def _gen(seed, layer, name, device):
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1000003 + layer * 7919 + _TENSOR_ID[name]) % (2 ** 62))
    return g


def _randn(shape, seed, layer, name, device):
    return torch.randn(shape, generator=_gen(seed, layer, name, device), device=device,
                       dtype=torch.float32)


def quantize_e4m3(x):
    """Per-token (last-dim rows flattened over everything but the token axes) e4m3 quantiser.

    x: [..., d] or [..., H, d] fp32 with one scale per leading `token` index; the caller passes
    a view shaped [tokens, features].  Returns (uint8-viewable float8 tensor, fp32 scales)."""
    amax = x.abs().amax(dim=-1, keepdim=True).clamp_min(1e-12)
    scale = (amax / 448.0).to(torch.float32)
    y = (x / scale).clamp(-448.0, 448.0).to(torch.float8_e4m3fn)
    return y, scale.squeeze(-1)


def indexer_layer(cfg, layer, device="cpu"):
    """q [B,Tq,H_I,d_I], k [B,Lk,d_I], w [B,Tq,H_I] (+ q_scale [B,Tq], k_scale [B,Lk] for fp8)."""
    B, Tq, Lk, H, d = cfg["B"], cfg["Tq"], cfg["Lk"], cfg["H_I"], cfg["d_I"]
    seed, rho = cfg["seed"], cfg.get("rho", 0.0)
    q = _randn((B, Tq, H, d), seed, layer, "q", device) * (1.0 / math.sqrt(d))
    if rho > 0.0:
        kb = _randn((B, Lk, d), seed, 0, "k_base", device)
        kn = _randn((B, Lk, d), seed, layer, "k_noise", device)
        k = math.sqrt(rho) * kb + math.sqrt(1.0 - rho) * kn
        del kb, kn
    else:
        k = _randn((B, Lk, d), seed, layer, "k_noise", device)
    w = torch.rand((B, Tq, H), generator=_gen(seed, layer, "w", device), device=device,
                   dtype=torch.float32)
    out = {"w": w.contiguous()}
    if cfg["dtype"] == "bf16":
        out["q"] = q.to(torch.bfloat16).contiguous()
        out["k"] = k.to(torch.bfloat16).contiguous()
    elif cfg["dtype"] == "fp8":
        q8, qs = quantize_e4m3(q.reshape(B, Tq, H * d))
        k8, ks = quantize_e4m3(k)
        out["q"] = q8.reshape(B, Tq, H, d).contiguous()
        out["k"] = k8.contiguous()
        out["q_scale"] = qs.contiguous()
        out["k_scale"] = ks.contiguous()
    else:
        raise ValueError(cfg["dtype"])
    return out


def chain_indexer_layers(cfg, n_layers, device="cpu", rho=0.8):
    """Generator of bf16 indexer inputs whose q AND k drift from layer to layer as an AR(1) chain,
    x_0 = n_0, x_l = sqrt(rho) x_(l-1) + sqrt(1-rho) n_l, so the correlation of two layers decays
    with their distance.  Only the cross-layer overlap diagnostic uses it (a stand-in for a trained
    model's slowly drifting token selection); the graded configs keep the base+noise recipe above."""
    B, Tq, Lk, H, d = cfg["B"], cfg["Tq"], cfg["Lk"], cfg["H_I"], cfg["d_I"]
    seed = cfg["seed"]
    q = k = None
    a, b = math.sqrt(rho), math.sqrt(1.0 - rho)
    for l in range(n_layers):
        nq = _randn((B, Tq, H, d), seed, l, "q_chain", device)
        nk = _randn((B, Lk, d), seed, l, "k_chain", device)
        q = nq if q is None else a * q + b * nq
        k = nk if k is None else a * k + b * nk
        del nq, nk
        w = torch.rand((B, Tq, H), generator=_gen(seed, l, "w", device), device=device, dtype=torch.float32)
        yield {"q": (q * (1.0 / math.sqrt(d))).to(torch.bfloat16).contiguous(),
               "k": k.to(torch.bfloat16).contiguous(), "w": w.contiguous()}


def attn_layer(cfg, layer, device="cpu", parts=("Q", "KV")):
    """Q [B,Tq,H_q,d_qk] bf16 and KV [B,Lk,row_elems] bf16 (each has its own random stream, so either can
    be drawn alone with `parts`)."""
    B, Tq, Lk = cfg["B"], cfg["Tq"], cfg["Lk"]
    seed = cfg["seed"]
    out = {}
    if "Q" in parts:
        out["Q"] = torch.randn((B, Tq, cfg["H_q"], cfg["d_qk"]), generator=_gen(seed, layer, "Q", device),
                               device=device, dtype=torch.bfloat16).contiguous()
    if "KV" in parts:
        out["KV"] = torch.randn((B, Lk, cfg["row_elems"]), generator=_gen(seed, layer, "KV", device),
                                device=device, dtype=torch.bfloat16).contiguous()
    return out


def stack_layers(cfg, device="cpu", n_layers=None):
    """One dict per layer with the indexer and attention tensors of that layer."""
    n = cfg["n_layers"] if n_layers is None else n_layers
    layers = []
    for l in range(n):
        d = indexer_layer(cfg, l, device)
        d.update(attn_layer(cfg, l, device))
        layers.append(d)
    return layers


def sm_scale(cfg):
    """Default softmax scale 1/sqrt(d_qk): unit-variance logits on N(0,1) inputs."""
    return 1.0 / math.sqrt(cfg["d_qk"])


def bits(t):
    """The exact bit patterns of a bf16 / fp8 / fp32 / int32 tensor as a C-contiguous numpy array."""
    t = t.detach().contiguous().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.float8_e4m3fn:
        return t.view(torch.uint8).numpy()
    return t.numpy()


def bits_layer(layer):
    """numpy bit-pattern view of every tensor of a layer dict (for the oracle)."""
    return {name: bits(t) for name, t in layer.items()}
