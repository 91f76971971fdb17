#!/usr/bin/env python3
"""Benchmark of the IndexCache / DSA attention-side hot path on one MI355X.

A step is one pass of the whole path (indexer score + top-k on Full layers, sparse MQA
attention on every layer) through ic_forward_stack over the 48-layer, L = 32768 prefill stack
with the 1-in-4 Full pattern (FSSS...).  The all-Full arm (standard DSA) and one batched decode
step (batch 32, context 65536, 4 layers FSSS / FFFF) are timed beside it and reported in
"arms".  Inputs are synthetic, seeded and resident in HBM before the timed region.

Prints ONE JSON line (see the keys below); progress goes to stderr.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# HBM bytes per launch of the kernels at the configs[3] per-layer shape, from rocprofv3 FETCH_SIZE +
# WRITE_SIZE scaled by a plain-copy reference (profiles/attn_score_select_prefill32k_hbm_traffic.txt).
MEASURED_TRAFFIC_BYTES = {"sparse_attn": 18.88e9 + 1.07e9, "indexer_score": 0.452e9 + 0.566e9,
                          "topk_select": 0.672e9 + 0.068e9}
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published
KERNELS = ["indexer_score", "topk_select", "sparse_attn", "attn_merge"]


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def ensure_built():
    import paper_2603_12201_amd as ic
    if not os.path.exists(ic.lib_path()):
        from paper_2603_12201_amd import build
        log("libindexcache.so missing: building")
        build.build()
    ic.lib()
    return ic


def time_steps(fn, steps, warmup):
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def prof_snapshot(ic):
    ic.prof_collect()
    return {name: ic.prof_get(i) for i, name in enumerate(KERNELS)}


class Stack:
    """Device-resident layer tensors + the host layer array for ic_forward_stack."""

    def __init__(self, ic, synth, cfg, n_layers, share_q_every):
        import torch
        self.cfg, self.ic = cfg, ic
        B, Tq = cfg["B"], cfg["Tq"]
        t0 = time.perf_counter()
        self.layers = []
        for l in range(n_layers):
            d = synth.indexer_layer(cfg, l, device="cuda")
            if l < share_q_every:
                d.update(synth.attn_layer(cfg, l, device="cuda"))
            else:   # cycle the big attention inputs (they do not influence the indices)
                src = self.layers[l % share_q_every]
                d["Q"], d["KV"] = src["Q"], src["KV"]
            self.layers.append(d)
            if l % 8 == 7:
                torch.cuda.synchronize()
                log("generated %d/%d layers (%.1f s)" % (l + 1, n_layers, time.perf_counter() - t0))
        self.O = torch.empty((B, Tq, cfg["H_q"], cfg["d_v"]), dtype=torch.bfloat16, device="cuda")
        self.arr = ic.make_layers(self.layers, cfg["k_sel"], cfg["q_pos0"], cfg["d_v"], cfg["v_off"],
                                  synth.sm_scale(cfg), [self.O] * n_layers)
        self.ws = torch.empty(max(ic.forward_stack_workspace(self.arr), 256), dtype=torch.uint8, device="cuda")
        self.idx_cache = torch.empty((B, Tq, cfg["k_sel"]), dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()

    def step(self, mask):
        self.ic.forward_stack(self.arr, mask, self.idx_cache, self.ws)


def algorithmic(cfg):
    """Algorithmic work of ONE layer's kernels: flops per causal pair, bytes per key / score / query token."""
    B, Tq, Lk, p0 = cfg["B"], cfg["Tq"], cfg["Lk"], cfg["q_pos0"]
    pairs = sum(max(0, min(Lk, p0 + i + 1)) for i in range(Tq)) * B if Tq <= 4096 else \
        B * (Tq * (Tq + 1) // 2 if p0 == 0 and Tq == Lk else Tq * Lk)
    return {
        "indexer_flop": 2.0 * cfg["H_I"] * cfg["d_I"] * pairs,                 # 2*H_I*d_I per causal pair
        "indexer_key_bytes": float(B) * Lk * cfg["d_I"] * 2,                   # decode: the key cache once
        "select_bytes": 4.0 * pairs + 4.0 * B * Tq * cfg["k_sel"],             # one read of the scores + idx
        "attn_bytes": float(B) * Tq * (min(cfg["k_sel"], Lk) * cfg["row_elems"] * 2
                                       + cfg["H_q"] * cfg["d_qk"] * 2 + cfg["H_q"] * cfg["d_v"] * 2),
        "attn_flop": 2.0 * B * Tq * cfg["H_q"] * min(cfg["k_sel"], Lk) * (cfg["d_qk"] + cfg["d_v"]),
    }


def cpu_baseline(synth, cfg, layer_gpu, n_full, n_layers, budget_s=15.0):
    """The oracle, as it stands, on a strided sample of query rows of one layer; extrapolated to
    the whole 1-in-4 stack by the row count (a strided sample is unbiased for the causal work)."""
    from oracle import oracle as orc
    import numpy as np
    Tq = cfg["Tq"]
    lb = synth.bits_layer(layer_gpu)

    def run(rows):
        t0 = time.perf_counter()
        r = orc.indexer_topk(lb["q"], lb["k"], lb["w"], cfg["q_pos0"], cfg["k_sel"], rows=rows)
        t1 = time.perf_counter()
        orc.sparse_attn(lb["Q"], lb["KV"], r["idx"], cfg["d_v"], cfg["v_off"], synth.sm_scale(cfg),
                        rows=rows, idx_is_subset=True)
        t2 = time.perf_counter()
        return t1 - t0, t2 - t1

    def strided(n):
        return sorted(set(int(x) for x in np.linspace(0, Tq - 1, n)))

    rows = strided(32)
    ti, ta = run(rows)
    per_row = (ti + ta) / len(rows)
    n = int(max(32, min(Tq, budget_s / max(per_row, 1e-6))))
    rows = strided(n)
    ti, ta = run(rows)
    layer_idx_s = ti / len(rows) * Tq
    layer_att_s = ta / len(rows) * Tq
    total_s = n_full * layer_idx_s + n_layers * layer_att_s
    return {
        "value": cfg["B"] * Tq / total_s, "unit": "tokens/s", "cores": orc.num_threads(), "kind": "oracle",
        "sample": "%d strided query rows of one layer (indexer+top-k %.2f s, attention %.2f s), "
                  "extrapolated by row count to %d Full + %d attention layers"
                  % (len(rows), ti, ta, n_full, n_layers),
        "extrapolated": True,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--layers", type=int, default=48, help="layers of the prefill stack (48 = the metric's workload)")
    ap.add_argument("--distinct-attn-inputs", type=int, default=4,
                    help="distinct per-layer Q/KV buffers to generate; later layers cycle through them")
    ap.add_argument("--decode-steps", type=int, default=20)
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle baseline leg")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--greedy-layers", type=int, default=6)
    ap.add_argument("--no-fp8", action="store_true")
    ap.add_argument("--distill-targets", type=int, default=4)
    ap.add_argument("--no-overlap", action="store_true", help="skip the cross-layer overlap diagnostic arm")
    ap.add_argument("--overlap-layers", type=int, default=48)
    ap.add_argument("--similarity-layers", type=int, default=8)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain device copies of 1 GiB (reference dispatches for scaling rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    ic = ensure_built()
    import synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---------------- prefill: 48-layer stack, L = 32768 ----------------
    cfg = synth.config("c3", n_layers=args.layers)
    n_layers = args.layers
    mask_14 = ic.pattern_uniform(n_layers, 4)
    mask_all = [True] * n_layers
    stack = Stack(ic, synth, cfg, n_layers, max(1, min(args.distinct_attn_inputs, n_layers)))
    alg = algorithmic(cfg)
    tokens = cfg["B"] * cfg["Tq"]

    log("prefill 1-in-4 arm")
    ic.prof_reset()
    for _ in range(args.warmup):
        stack.step(mask_14)
    torch.cuda.synchronize()
    ic.prof_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        stack.step(mask_14)
    torch.cuda.synchronize()
    ms_14 = (time.perf_counter() - t0) * 1e3 / args.steps
    ic.prof_enable(False)
    prof_14 = prof_snapshot(ic)

    log("prefill all-Full arm")
    ms_all = time_steps(lambda: stack.step(mask_all), max(1, args.steps - 1), 1)

    def per_launch(prof, name):
        n, ms = prof[name]
        return (ms / n) if n else None

    # per-layer kernel time (one layer = all its launches of that class)
    n_full = sum(mask_14)
    t_score = prof_14["indexer_score"][1] / (args.steps * n_full)
    t_select = prof_14["topk_select"][1] / (args.steps * n_full)
    t_attn = prof_14["sparse_attn"][1] / (args.steps * n_layers)
    kernels = {
        "indexer_score": {"bound": "mfma", "ms_per_layer": t_score,
                          "achieved": alg["indexer_flop"] / (t_score * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                          "unit": "TFLOP/s", "launches_per_layer": prof_14["indexer_score"][0] / (args.steps * n_full)},
        "topk_select": {"bound": "hbm", "ms_per_layer": t_select,
                        "achieved": alg["select_bytes"] / (t_select * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                        "unit": "GB/s", "launches_per_layer": prof_14["topk_select"][0] / (args.steps * n_full)},
        "sparse_attn": {"bound": "hbm", "ms_per_layer": t_attn,
                        "achieved": alg["attn_bytes"] / (t_attn * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                        "unit": "GB/s", "launches_per_layer": prof_14["sparse_attn"][0] / (args.steps * n_layers),
                        "mfma_tflops": alg["attn_flop"] / (t_attn * 1e-3) / 1e12},
    }
    for k in kernels.values():
        k["frac"] = k["achieved"] / k["peak"]
    # dominant kernel of the timed step = largest share of the step's time
    share = {"indexer_score": t_score * n_full, "topk_select": t_select * n_full, "sparse_attn": t_attn * n_layers}
    dom = max(share, key=share.get)
    roofline = {"kernel": dom, "bound": kernels[dom]["bound"], "achieved": kernels[dom]["achieved"],
                "peak": kernels[dom]["peak"], "unit": kernels[dom]["unit"], "frac": kernels[dom]["frac"],
                "traffic": MEASURED_TRAFFIC_BYTES.get(dom) if cfg["Tq"] == 32768 else None,
                "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE+WRITE_SIZE, scaled; see profiles/)",
                "avg_launch_ms": per_launch(prof_14, dom),
                "share_of_step": share[dom] / sum(share.values())}
    if dom == "sparse_attn":
        # the gathered rows of neighbouring queries are re-used out of L2 / Infinity Cache (unique KV is
        # 37.7 MB), so the algorithmic gather rate may exceed the HBM peak; the kernel's own bounds are
        # the MFMA rate of its flops and the LDS data path every gathered byte crosses
        roofline["mfma_frac"] = kernels[dom]["mfma_tflops"] / MFMA_BF16_PEAK_TFLOPS
        roofline["note"] = ("achieved = algorithmic gathered bytes / time; HBM traffic (field traffic) is 4x smaller "
                            "because selected rows are re-used out of L2, so frac can exceed 1")

    arms = {
        "prefill_1in4": {"ms_per_step": ms_14, "tokens_per_s": tokens / (ms_14 * 1e-3), "full_layers": n_full},
        "prefill_all_full": {"ms_per_step": ms_all, "tokens_per_s": tokens / (ms_all * 1e-3), "full_layers": n_layers},
        "prefill_speedup_1in4_vs_all_full": ms_all / ms_14,
    }

    cpu = None
    if not args.no_cpu:
        log("cpu baseline (oracle, bounded sample)")
        cpu = cpu_baseline(synth, cfg, stack.layers[0], n_full, n_layers)

    del stack
    torch.cuda.empty_cache()

    # ---------------- decode: batch 32, context 65536, 4 layers ----------------
    if not args.no_decode:
        dcfg = synth.config("c2")
        log("decode inputs")
        dstack = Stack(ic, synth, dcfg, dcfg["n_layers"], dcfg["n_layers"])
        dalg = algorithmic(dcfg)
        m_fsss = ic.pattern_from_string("FSSS")
        m_ffff = [True] * 4
        ms_d14 = time_steps(lambda: dstack.step(m_fsss), args.decode_steps, 3)
        ms_dall = time_steps(lambda: dstack.step(m_ffff), args.decode_steps, 3)
        # the same FSSS step recorded in a HIP graph (the library allocates, clears and synchronises nothing)
        dgraph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(dgraph):
            dstack.step(m_fsss)
        ms_d14_graph = time_steps(dgraph.replay, args.decode_steps, 3)
        # per layer-step, from the two step times (launch gaps included; event pairs around 20 us
        # kernels would add their own few us each): FFFF - FSSS = three indexer + top-k runs
        d_idx = (ms_dall - ms_d14) / 3.0
        d_att = (ms_d14 - d_idx) / 4.0
        arms.update({
            "decode_1in4": {"ms_per_step": ms_d14, "tokens_per_s": dcfg["B"] / (ms_d14 * 1e-3), "pattern": "FSSS"},
            "decode_1in4_graph_replay": {"ms_per_step": ms_d14_graph, "tokens_per_s": dcfg["B"] / (ms_d14_graph * 1e-3),
                                         "pattern": "FSSS"},
            "decode_all_full": {"ms_per_step": ms_dall, "tokens_per_s": dcfg["B"] / (ms_dall * 1e-3), "pattern": "FFFF"},
            "decode_speedup_1in4_vs_all_full": ms_dall / ms_d14,
            "decode_kernels": {
                "note": "per layer-step, derived from the FFFF and FSSS step times (launch gaps included)",
                "indexer_plus_topk": {"bound": "hbm", "ms_per_layer": d_idx,
                                      "achieved": dalg["indexer_key_bytes"] / (d_idx * 1e-3) / 1e9,
                                      "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                      "frac": dalg["indexer_key_bytes"] / (d_idx * 1e-3) / 1e9 / HBM_PEAK_GBS},
                "sparse_attn_plus_merge": {"bound": "hbm", "ms_per_layer": d_att,
                                           "achieved": dalg["attn_bytes"] / (d_att * 1e-3) / 1e9,
                                           "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                           "frac": dalg["attn_bytes"] / (d_att * 1e-3) / 1e9 / HBM_PEAK_GBS},
            },
        })
        # the same caches read through a page table (64-position pages in random physical order),
        # first with every sequence at full length, then with a seeded mix of lengths in [Lk/2, Lk]
        log("paged decode arm")
        g = torch.Generator().manual_seed(2603)
        page, Lk_d = 64, dcfg["Lk"]
        pt = torch.randperm(dcfg["B"] * Lk_d // page, generator=g).to(torch.int32).reshape(dcfg["B"], Lk_d // page).cuda()
        arr_p = ic.make_layers(dstack.layers, dcfg["k_sel"], 0, dcfg["d_v"], dcfg["v_off"], synth.sm_scale(dcfg),
                               [dstack.O] * dcfg["n_layers"], Lk=Lk_d)
        paged = {"page_size": page}
        for name, lens in (("full_length", torch.full((dcfg["B"],), Lk_d, dtype=torch.int32)),
                           ("ragged", torch.randint(Lk_d // 2, Lk_d + 1, (dcfg["B"],), generator=g).to(torch.int32))):
            pc = ic.paged_cache(lens.cuda(), pt, page)
            ms14 = time_steps(lambda: ic.forward_stack_paged(arr_p, m_fsss, pc, dstack.idx_cache, dstack.ws), args.decode_steps, 3)
            msall = time_steps(lambda: ic.forward_stack_paged(arr_p, m_ffff, pc, dstack.idx_cache, dstack.ws), args.decode_steps, 3)
            paged[name] = {"mean_len": float(lens.float().mean()), "ms_per_step_1in4": ms14, "ms_per_step_all_full": msall,
                           "tokens_per_s_1in4": dcfg["B"] / (ms14 * 1e-3), "speedup_1in4_vs_all_full": msall / ms14}
        arms["decode_paged"] = paged
        del dstack, arr_p

    # ---------------- cross-layer overlap of the index sets (the paper's App. A diagnostic) ----------------
    if not args.no_overlap:
        log("overlap arm: %d layers with drifting q/k" % args.overlap_layers)
        ocfg = synth.config("c3")
        idxs = []
        for lay in synth.chain_indexer_layers(ocfg, args.overlap_layers, device="cuda"):
            idxs.append(ic.indexer_topk(lay["q"], lay["k"], lay["w"], ocfg["k_sel"], 0))
            del lay
        ows = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
        ic.topk_overlap(idxs, ocfg["Lk"], workspace=ows)
        torch.cuda.synchronize()
        ms_ov = time_steps(lambda: ic.topk_overlap(idxs, ocfg["Lk"], workspace=ows), 3, 0)
        ov = ic.topk_overlap(idxs, ocfg["Lk"], workspace=ows)[0].cpu()
        n_ov = len(idxs)
        by_dist = {}
        for dist in (1, 2, 4, 8, 16, 32):
            if dist < n_ov:
                by_dist[str(dist)] = float(torch.diagonal(ov, dist).mean())
        # one membership test = one 4-byte LDS gather lane; the LDS serves a 64-lane gather in about 16
        # clocks per CU (measured), i.e. 4 tests per clock and CU: 256 CUs x 2.4 GHz x 4
        ov_tests = n_ov * (n_ov + 1) / 2 * ocfg["Tq"] * ocfg["k_sel"]
        ov_peak = 256 * 2.4e9 * 4 / 1e12
        arms["topk_overlap"] = {"layers": n_ov, "ms": ms_ov, "bound": "alu",
                                "achieved": ov_tests / (ms_ov * 1e-3) / 1e12, "peak": ov_peak,
                                "unit": "T membership tests/s", "frac": ov_tests / (ms_ov * 1e-3) / 1e12 / ov_peak,
                                "index_bytes_read_GBs": n_ov * ocfg["Tq"] * ocfg["k_sel"] * 4 / (ms_ov * 1e-3) / 1e9,
                                "mean_overlap_by_layer_distance": by_dist,
                                "data": "q and k drift as an AR(1) chain over the layers (rho 0.8)"}
        # similarity-based pattern search (App. C) on the first layers of the same stack: S[i][j] from the
        # attention outputs under own vs reused indices, then the exact dynamic program
        n_sim = min(args.similarity_layers, n_ov)
        if n_sim >= 2:
            log("similarity arm: %d layers" % n_sim)
            at = [synth.attn_layer(ocfg, l, device="cuda") for l in range(min(n_sim, 2))]
            at = [at[l % len(at)] for l in range(n_sim)]           # the big Q/KV inputs are cycled, the indices are not
            o_own = torch.empty((ocfg["B"], ocfg["Tq"], ocfg["H_q"], ocfg["d_v"]), dtype=torch.bfloat16, device="cuda")
            arr = ic.make_layers(at, ocfg["k_sel"], 0, ocfg["d_v"], ocfg["v_off"], synth.sm_scale(ocfg), [o_own] * n_sim)
            t0 = time.perf_counter()
            S = ic.similarity_matrix(arr, idxs[:n_sim])
            torch.cuda.synchronize()
            ms_sim = (time.perf_counter() - t0) * 1e3
            o_b = torch.empty_like(o_own)
            o_b.copy_(o_own)
            a2, b2 = o_own.view(ocfg["Tq"], -1), o_b.view(ocfg["Tq"], -1)
            ms_cos = time_steps(lambda: ic.cosine_rows(a2, b2), 5, 1)
            cos_bytes = 2 * a2.numel() * 2
            Sh = S.cpu().numpy()
            t0 = time.perf_counter()
            mask, total = ic.pattern_search_dp(Sh, max(1, n_sim // 4))
            ms_dp = (time.perf_counter() - t0) * 1e3
            arms["similarity_search"] = {
                "layers": n_sim, "matrix_ms": ms_sim, "attention_launches": n_sim * (n_sim + 1) // 2,
                "cosine_kernel": {"ms": ms_cos, "bound": "hbm", "achieved": cos_bytes / (ms_cos * 1e-3) / 1e9,
                                  "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": cos_bytes / (ms_cos * 1e-3) / 1e9 / HBM_PEAK_GBS},
                "mean_similarity_by_layer_distance": {str(d): float(np.mean([Sh[i, i - d] for i in range(d, n_sim)]))
                                                      for d in (1, 2, 4) if d < n_sim},
                "dp_pattern": "".join("F" if m else "S" for m in mask), "dp_total": total, "dp_host_ms": ms_dp}
            del at, o_own, o_b
        del idxs

    # ---------------- greedy layer selection by forward passes (Alg. 1 with the surrogate loss) ----------------
    if not args.no_overlap and args.greedy_layers >= 2:
        n_g = args.greedy_layers
        k_g = n_g // 2
        log("greedy search arm: %d layers, %d flips" % (n_g, k_g))
        gcfg = synth.config("c3")
        at2 = [synth.attn_layer(gcfg, l, device="cuda") for l in range(2)]
        lay_g = []
        for l, ixl in enumerate(synth.chain_indexer_layers(gcfg, n_g, device="cuda")):
            d = dict(ixl)
            d.update(at2[l % 2])                                  # the big Q/KV inputs are cycled, the indexer inputs are not
            lay_g.append(d)
        o_shape = (gcfg["B"], gcfg["Tq"], gcfg["H_q"], gcfg["d_v"])
        outs_g = [torch.empty(o_shape, dtype=torch.bfloat16, device="cuda") for _ in range(n_g)]
        arr_g = ic.make_layers(lay_g, gcfg["k_sel"], 0, gcfg["d_v"], gcfg["v_off"], synth.sm_scale(gcfg), outs_g)
        ws_g = torch.empty(max(int(ic.lib().ic_greedy_search_forward_workspace(arr_g, n_g)), 256), dtype=torch.uint8, device="cuda")
        cache_g = torch.empty((gcfg["B"], gcfg["Tq"], gcfg["k_sel"]), dtype=torch.int32, device="cuda")
        ic.forward_stack(arr_g, [True] * n_g, cache_g, ws_g)
        torch.cuda.synchronize()
        ref_g = [o.clone() for o in outs_g]
        t0 = time.perf_counter()
        gmask, gorder, gcurve = ic.greedy_search_forward(arr_g, k_g, ref_g, cache_g, workspace=ws_g)
        ms_g = (time.perf_counter() - t0) * 1e3
        passes = sum(n_g - 1 - s for s in range(k_g))
        arms["greedy_search"] = {
            "layers": n_g, "flips": k_g, "forward_passes": passes, "total_ms": ms_g, "ms_per_forward_pass": ms_g / passes,
            "tokens_per_s_inside_search": passes * gcfg["Tq"] / (ms_g * 1e-3),
            "order": gorder, "loss_curve": gcurve, "pattern": "".join("F" if m else "S" for m in gmask),
            "loss": "1/N sum_l (1 - mean per-token cosine of layer l's output under the pattern vs all-Full)"}
        del lay_g, outs_g, ref_g, at2, arr_g

    # ---------------- forward of the multi-layer distillation loss (Sec. 3.3, Eq. 1 / Eq. 2) ----------------
    if not args.no_overlap and args.distill_targets >= 1:
        m1 = args.distill_targets
        log("distillation arm: one Full layer serving %d layers" % m1)
        dcfg3 = synth.config("c3")
        ixd = synth.indexer_layer(dcfg3, 0, device="cuda")
        idx_d, sel_d = ic.indexer_topk(ixd["q"], ixd["k"], ixd["w"], dcfg3["k_sel"], 0, want_scores=True)
        del ixd
        atd = synth.attn_layer(dcfg3, 0, device="cuda")
        _, lse_d = ic.sparse_attn(atd["Q"], atd["KV"], idx_d, dcfg3["d_v"], dcfg3["v_off"], synth.sm_scale(dcfg3), want_lse=True)
        ms_probs = time_steps(lambda: ic.attn_probs(atd["Q"], atd["KV"], idx_d, synth.sm_scale(dcfg3), lse_d), 3, 1)
        probs_d = [ic.attn_probs(atd["Q"], atd["KV"], idx_d, synth.sm_scale(dcfg3), lse_d) for _ in range(m1)]
        ws_d = torch.empty(int(ic.lib().ic_distill_loss_workspace(dcfg3["Tq"])), dtype=torch.uint8, device="cuda")
        ms_kl = time_steps(lambda: ic.distill_loss(probs_d, sel_d, workspace=ws_d), 5, 1)
        lm_d, la_d = ic.distill_loss(probs_d, sel_d, workspace=ws_d)
        torch.cuda.synchronize()
        flop_p = 2.0 * dcfg3["H_q"] * dcfg3["k_sel"] * dcfg3["d_qk"] * dcfg3["Tq"]
        bytes_kl = (m1 + 1) * 4.0 * dcfg3["Tq"] * dcfg3["k_sel"]
        arms["distill_forward"] = {
            "served_layers": m1,
            "attn_probs": {"ms": ms_probs, "bound": "mfma", "achieved": flop_p / (ms_probs * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                           "unit": "TFLOP/s", "frac": flop_p / (ms_probs * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                           "gathered_GBs": dcfg3["Tq"] * dcfg3["k_sel"] * dcfg3["row_elems"] * 2 / (ms_probs * 1e-3) / 1e9},
            "kl_kernel": {"ms": ms_kl, "bound": "hbm", "achieved": bytes_kl / (ms_kl * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                          "unit": "GB/s", "frac": bytes_kl / (ms_kl * 1e-3) / 1e9 / HBM_PEAK_GBS},
            "loss_multi": float(lm_d), "loss_avg": float(la_d),
            "note": "identical targets here, so Eq. 1 = Eq. 2; timing only"}
        del probs_d, atd, idx_d, sel_d

    # ---------------- the FP8 indexer at configs[4] (L = 131072, 64 heads, e4m3 + per-token scales) ----------------
    if not args.no_fp8:
        log("fp8 indexer arm (configs[4], one Full layer)")
        c4 = synth.config("c4")
        l4 = synth.indexer_layer(c4, 0, device="cuda")
        from paper_2603_12201_amd import binding as icb
        ws4 = torch.empty(ic.indexer_topk_workspace(icb.indexer_desc(l4["q"], l4["k"], l4["w"], c4["k_sel"], 0,
                                                                     l4["q_scale"], l4["k_scale"])), dtype=torch.uint8, device="cuda")
        idx4 = torch.empty((c4["B"], c4["Tq"], c4["k_sel"]), dtype=torch.int32, device="cuda")
        run4 = lambda: ic.indexer_topk(l4["q"], l4["k"], l4["w"], c4["k_sel"], 0, q_scale=l4["q_scale"], k_scale=l4["k_scale"],
                                       idx=idx4, workspace=ws4)
        ms4 = time_steps(run4, 2, 1)
        flop4 = 2.0 * c4["H_I"] * c4["d_I"] * (c4["Tq"] * (c4["Tq"] + 1) / 2)
        arms["indexer_fp8_c4"] = {
            "L": c4["Tq"], "H_I": c4["H_I"], "ms_indexer_plus_topk": ms4,
            "tokens_per_s_one_full_layer": c4["Tq"] / (ms4 * 1e-3),
            "score_flop": flop4, "PFLOPs_incl_topk": flop4 / (ms4 * 1e-3) / 1e15, "peak_PFLOPs": 5.0,
            "note": "wall time of ic_indexer_topk; per-kernel split in profiles/indexer_fp8_131k_kernel_trace.txt"}
        del l4, ws4, idx4

    out = {
        "metric": "prefill & decode tokens/s, 48-layer DSA stack L=32K, 1-in-4 Full vs all-Full",
        "value": tokens / (ms_14 * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_14,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[3]: 48-layer attention-only DSA stack prefill, 1 sequence, L=32768, "
                               "H_I=32 d_I=128 k=2048, MQA 32 heads, KV row 576 bf16, 1-in-4 Full (value); "
                               "all-Full and decode (configs[2]) in arms",
                   "layers": n_layers, "pattern": "FSSS x%d" % (n_layers // 4), "L": cfg["Tq"], "k_sel": cfg["k_sel"],
                   "distinct_attn_inputs": min(args.distinct_attn_inputs, n_layers)},
        "roofline": roofline,
        "kernels": kernels,
        "arms": arms,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
