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

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
MFMA_FP8_PEAK_TFLOPS = 5000.0    # MI355X dense fp8 MFMA, published
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")
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


def event_ms(fn, reps=5, warmup=1):
    """Average duration of fn's device work in ms, between two events on torch's current stream (the
    stream the binding hands to the library)."""
    import torch
    for _ in range(warmup):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) / reps


def measured_traffic():
    """HBM bytes per launch from the tracked rocprofv3 counter summary (lines 'traffic <kernel> <workload>
    fetch_bytes=<f> write_bytes=<w>'); the file names the runs the figures come from."""
    out = {"source": os.path.relpath(TRAFFIC_FILE, ROOT)}
    try:
        for line in open(TRAFFIC_FILE):
            t = line.split()
            if len(t) >= 5 and line.startswith("traffic "):
                kv = dict(x.split("=") for x in t[3:] if "=" in x)
                try:
                    out[(t[1], t[2])] = float(kv["fetch_bytes"]) + float(kv["write_bytes"])
                except (KeyError, ValueError):
                    pass
    except OSError:
        out["source"] = None
    return out


def prof_snapshot(ic):
    ic.prof_collect()
    return {name: ic.prof_get(i) for i, name in enumerate(KERNELS)}


class Stack:
    """Device-resident layer tensors + the host layer array for ic_forward_stack.  Every layer has its own
    indexer inputs and its own KV cache; Q is distinct for the first `distinct_q` layers and cycled after
    that (all layers by default; the long-context workload aliases it because 48 x 4.8 GB of Q and as much
    of O do not fit beside the rest, and Q does not influence the indices).  Every layer writes its output to one
    shared buffer (a layer's output is consumed at once in a model)."""

    def __init__(self, ic, synth, cfg, n_layers, distinct_q):
        import torch
        self.cfg, self.ic = cfg, ic
        B, Tq = cfg["B"], cfg["Tq"]
        t0 = time.perf_counter()
        self.layers = []
        for l in range(n_layers):
            d = synth.indexer_layer(cfg, l, device="cuda")
            if l < distinct_q:
                d.update(synth.attn_layer(cfg, l, device="cuda"))
            else:
                d.update(synth.attn_layer(cfg, l, device="cuda", parts=("KV",)))
                d["Q"] = self.layers[l % distinct_q]["Q"]
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


def profile_pass(ic, stack, mask):
    """Per-kernel durations of ONE step, from HIP events the library records around its launches on the
    caller's stream.  A pass of its own, outside every timed region."""
    import torch
    ic.prof_reset()
    torch.cuda.synchronize()
    ic.prof_enable(True)
    stack.step(mask)
    torch.cuda.synchronize()
    ic.prof_enable(False)
    return prof_snapshot(ic)


def kernel_table(alg, prof, n_full, n_layers, traffic, workload, fp8):
    """Per-layer time and roofline position of the three kernels of a prefill step."""
    t_score = prof["indexer_score"][1] / n_full
    t_select = prof["topk_select"][1] / n_full
    t_attn = prof["sparse_attn"][1] / n_layers
    mfma_peak_ix = MFMA_FP8_PEAK_TFLOPS if fp8 else MFMA_BF16_PEAK_TFLOPS
    k = {
        "indexer_score": {"bound": "mfma", "ms_per_layer": t_score, "achieved": alg["indexer_flop"] / (t_score * 1e-3) / 1e12,
                          "peak": mfma_peak_ix, "unit": "TFLOP/s", "launches_per_layer": prof["indexer_score"][0] / n_full},
        "topk_select": {"bound": "hbm", "ms_per_layer": t_select, "achieved": alg["select_bytes"] / (t_select * 1e-3) / 1e9,
                        "peak": HBM_PEAK_GBS, "unit": "GB/s", "launches_per_layer": prof["topk_select"][0] / n_full},
        # score and select together, priced as the one fused kernel they stand for: its flops against the MFMA peak
        "indexer_plus_topk": {"bound": "mfma", "ms_per_layer": t_score + t_select,
                              "achieved": alg["indexer_flop"] / ((t_score + t_select) * 1e-3) / 1e12, "peak": mfma_peak_ix,
                              "unit": "TFLOP/s"},
        # the gather is served out of L2 / Infinity Cache (a layer's KV is 38-151 MB, every row is fetched by
        # many queries), so its arithmetic intensity against compulsory bytes is far above the ridge:
        # the binding roofline is the MFMA rate of its flops
        "sparse_attn": {"bound": "mfma", "ms_per_layer": t_attn, "achieved": alg["attn_flop"] / (t_attn * 1e-3) / 1e12,
                        "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "launches_per_layer": prof["sparse_attn"][0] / n_layers,
                        "gathered_GBs": alg["attn_bytes"] / (t_attn * 1e-3) / 1e9,
                        "compulsory_bytes": alg["attn_unique_bytes"]},
    }
    for name, v in k.items():
        v["frac"] = v["achieved"] / v["peak"]
        t = traffic.get((name, workload))
        if t is not None:
            v["traffic"] = t
            # what the HBM side of L2 moved per second for this kernel (profiler counters of a tracked run over this
            # kernel's time in THIS run): near the chip's stream rate means the kernel waits for memory beyond L2
            v["traffic_GBs"] = t / (v["ms_per_layer"] * 1e-3) / 1e9
            v["traffic_frac_of_hbm_peak"] = v["traffic_GBs"] / HBM_PEAK_GBS
    return k


def algorithmic(cfg):
    """Algorithmic work of ONE layer's kernels: flops per causal pair, bytes per key / score / query token."""
    B, Tq, Lk, p0 = cfg["B"], cfg["Tq"], cfg["Lk"], cfg["q_pos0"]
    pairs = sum(max(0, min(Lk, p0 + i + 1)) for i in range(Tq)) * B if Tq <= 4096 else \
        B * (Tq * (Tq + 1) // 2 if p0 == 0 and Tq == Lk else Tq * Lk)
    # selected entries over all query rows: a row near the start of a sequence sees fewer keys than k_sel
    ks = min(cfg["k_sel"], Lk)
    n_short = max(0, min(Tq, ks - 1 - p0))                                  # rows i with p0 + i + 1 < ks
    entries = B * ((Tq - n_short) * ks + sum(max(0, p0 + i + 1) for i in range(n_short)))
    return {
        "indexer_flop": 2.0 * cfg["H_I"] * cfg["d_I"] * pairs,                 # 2*H_I*d_I per causal pair
        "indexer_key_bytes": float(B) * Lk * cfg["d_I"] * 2,                   # decode: the key cache once
        "select_bytes": 4.0 * pairs + 4.0 * B * Tq * cfg["k_sel"],             # one read of the scores + idx
        "attn_bytes": float(entries) * cfg["row_elems"] * 2
                      + float(B) * Tq * (cfg["H_q"] * cfg["d_qk"] * 2 + cfg["H_q"] * cfg["d_v"] * 2),
        "attn_flop": 2.0 * entries * cfg["H_q"] * (cfg["d_qk"] + cfg["d_v"]),
        # what a layer must move at least: its KV once, Q, O and the index tensor
        "attn_unique_bytes": float(B) * (Lk * cfg["row_elems"] * 2 + Tq * (cfg["H_q"] * (cfg["d_qk"] + cfg["d_v"]) * 2
                                                                         + cfg["k_sel"] * 4)),
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


def calibration(ic, synth, idx_prefill, kv_rows):
    """What the chip sustains on the hot path's access and issue patterns, through the library's own
    calibration kernels: the second denominator beside the published peaks."""
    import torch
    out = {}
    scratch = torch.empty(1 << 22, dtype=torch.uint8, device="cuda")
    n = 2 << 30
    src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1)
    ms = event_ms(lambda: ic.calibrate(ic.CALIB_READ, src, scratch, n=n, wgs=4096))
    out["stream_read"] = {"bytes": n, "ms": ms, "GBs": n / (ms * 1e-3) / 1e9, "frac_of_hbm_peak": n / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    dst = torch.empty(n // 2, dtype=torch.uint8, device="cuda")
    ms = event_ms(lambda: ic.calibrate(ic.CALIB_COPY, src, dst, n=n // 2, wgs=4096))
    out["copy"] = {"bytes_read_plus_written": n, "ms": ms, "GBs": n / (ms * 1e-3) / 1e9}
    del dst
    # decode indexer: one pass over the index-key cache of configs[2] (32 x 65536 keys x 256 B)
    nk = 32 * 65536 * 256
    ms = event_ms(lambda: ic.calibrate(ic.CALIB_READ, src, scratch, n=nk, wgs=2048), reps=20, warmup=3)
    out["decode_key_stream"] = {"bytes": nk, "us": ms * 1e3, "GBs": nk / (ms * 1e-3) / 1e9,
                                "frac_of_hbm_peak": nk / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    del src
    # decode attention: 32 sequences x 2048 random rows of 1152 B out of a 2.4 GB cache (configs[2])
    g = torch.Generator().manual_seed(77)
    table = torch.empty((32 * 65536, 1152), dtype=torch.uint8, device="cuda").fill_(3)
    rows = (torch.randint(0, 65536, (32, 2048), generator=g) + 65536 * torch.arange(32)[:, None]).to(torch.int32).cuda()
    # (a launch of about 13 us: 20 of them recorded in a HIP graph, so that the host's own time per call does not count)
    def decode_gather():
        ic.calibrate(ic.CALIB_GATHER, table, scratch, idx=rows, n=rows.numel(), table_rows=table.shape[0], row_bytes=1152, wgs=2048)
    decode_gather()
    torch.cuda.synchronize()
    note = "no compute attached, every row in flight at once; 20 launches per graph replay"
    try:
        cgraph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(cgraph):
            for _ in range(20):
                decode_gather()
        torch.cuda.synchronize()
        ms = event_ms(cgraph.replay, reps=5, warmup=2) / 20
        del cgraph
    except Exception as e:                                   # no graph: plain launches, the host's time per call included
        log("decode gather probe: graph capture failed (%s), timing plain launches" % e)
        torch.cuda.synchronize()
        ms = event_ms(decode_gather, reps=20, warmup=3)
        note = "no compute attached, every row in flight at once; plain launches, host time per call included"
    gb = rows.numel() * 1152
    out["decode_row_gather"] = {"bytes": gb, "us": ms * 1e3, "GBs": gb / (ms * 1e-3) / 1e9,
                                "frac_of_hbm_peak": gb / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "note": note}
    # prefill attention: the rows one L=32768 layer really selects, out of its 37.7 MB cache
    if idx_prefill is not None:
        flat = idx_prefill.reshape(-1)
        ms = event_ms(lambda: ic.calibrate(ic.CALIB_GATHER, table, scratch, idx=flat, n=flat.numel(), table_rows=kv_rows,
                                           row_bytes=1152, wgs=512), reps=2, warmup=1)
        gb = flat.numel() * 1152
        out["prefill_row_gather"] = {"bytes": gb, "ms": ms, "GBs": gb / (ms * 1e-3) / 1e9, "workgroups": 512,
                                     "note": "served out of L2 / Infinity Cache; no compute attached; 512 workgroups of 4 waves "
                                             "(about 72 KB in flight per CU) is the fastest schedule found: 256 give 11, 8192 give 10.8 TB/s"}
        # the attention kernel's tile loop without its arithmetic: the same rows through the same registers and LDS
        tp = {}
        for kind, name in ((ic.CALIB_TILE_GATHER, "gather_into_registers"), (ic.CALIB_TILE_STORE, "plus_lds_store"),
                           (ic.CALIB_TILE_READ, "plus_score_operand_reads"), (ic.CALIB_TILE_READ2, "plus_both_lds_reads"),
                           (ic.CALIB_TILE_INTERLEAVED, "same_bytes_phases_merged"), (ic.CALIB_TILE_8WAVES, "same_bytes_eight_waves")):
            tp[name + "_ms"] = event_ms(lambda: ic.calibrate(kind, table, scratch, idx=flat, n=flat.numel(), table_rows=kv_rows,
                                                             row_bytes=1152, wgs=256), reps=2, warmup=1)
        tp["note"] = ("64-row tiles, 4 waves, one workgroup per CU, one tile of gathers ahead, one barrier per tile: what the data "
                      "movement of the prefill attention kernel takes with no MFMA and no softmax (what is read is folded with XORs); "
                      "same_bytes_phases_merged: stores and gathers spread between the reads; same_bytes_eight_waves: the work "
                      "dealt to eight waves, no byte read twice")
        out["prefill_attn_tile_path"] = tp
    del table, rows
    for kind, name, flop, peak in ((ic.CALIB_MFMA_BF16, "mfma_bf16", 2.0 * 32 * 32 * 16, MFMA_BF16_PEAK_TFLOPS),
                                   (ic.CALIB_MFMA_FP8, "mfma_fp8", 2.0 * 32 * 32 * 64, MFMA_FP8_PEAK_TFLOPS)):
        rounds, wgs = 20000, 512
        ms = event_ms(lambda: ic.calibrate(kind, None, scratch, n=rounds, wgs=wgs), reps=3, warmup=1)
        tf = flop * 4 * rounds * 4 * wgs / (ms * 1e-3) / 1e12
        out[name] = {"TFLOPs": tf, "frac_of_published_peak": tf / peak, "waves_per_simd": 2,
                     "note": "constant operands; under random operands the shader clock settles lower"}
    # LDS access patterns of the attention tile, nothing else running: time per 64-lane instruction and CU
    lds = {}
    for kind, name, nbytes in ((ic.CALIB_LDS_READ16_PADDED, "read16_rows_1184_apart", 1024),
                               (ic.CALIB_LDS_READ16_SWIZZLED, "read16_rows_1152_apart_xor_swizzled", 1024),
                               (ic.CALIB_LDS_TR8_ROWS2, "transpose_read8_rows_two_apart", 512),
                               (ic.CALIB_LDS_TR8_ROWS1, "transpose_read8_consecutive_rows", 512)):
        rounds, wgs = 4000, 256
        ms = event_ms(lambda: ic.calibrate(kind, None, scratch, n=rounds, wgs=wgs), reps=3, warmup=1)
        ns = ms * 1e6 / (rounds * 16 * 16)                  # 16 reads per round and wave, 16 waves per CU
        lds[name] = {"ns_per_instruction_per_cu": ns, "bytes_per_ns_per_cu": nbytes / ns}
    lds["note"] = ("16 waves per CU issue nothing but one kind of LDS read (the LDS fill at kernel start and the launch are in the "
                   "figure: a few per cent); the first and the third are the patterns of the attention tile as it is laid out, "
                   "the second is the layout it had before, the fourth what its transpose reads would cost over consecutive rows")
    out["lds_access_patterns"] = lds
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--layers", type=int, default=48, help="layers of the prefill stack (48 = the metric's workload)")
    ap.add_argument("--distinct-attn-inputs", type=int, default=48,
                    help="layers with a Q tensor of their own (every layer has its own KV and indexer inputs); "
                         "later layers cycle through those Q")
    ap.add_argument("--decode-steps", type=int, default=20)
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle baseline leg")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-calibrate", action="store_true", help="skip the calibration arm (stream, copy, gather, MFMA rounds)")
    ap.add_argument("--greedy-layers", type=int, default=6)
    ap.add_argument("--no-fp8", action="store_true", help="skip the configs[4] long-context fp8 stack arm")
    ap.add_argument("--fp8-layers", type=int, default=48)
    ap.add_argument("--fp8-distinct-q", type=int, default=2)
    ap.add_argument("--distill-targets", type=int, default=4)
    ap.add_argument("--no-overlap", action="store_true", help="skip the diagnostic arms (overlap, similarity, greedy, distillation)")
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
    t_start = time.perf_counter()
    traffic = measured_traffic()

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
    n_full = sum(mask_14)

    # the timed regions carry no event records; the per-kernel split comes from a pass of its own
    log("prefill 1-in-4 arm")
    ms_14 = time_steps(lambda: stack.step(mask_14), args.steps, args.warmup)
    log("prefill all-Full arm")
    ms_all = time_steps(lambda: stack.step(mask_all), max(1, args.steps - 1), 1)
    log("per-kernel pass")
    prof_14 = profile_pass(ic, stack, mask_14)
    workload = "prefill32k" if cfg["Tq"] == 32768 else "other"
    kernels = kernel_table(alg, prof_14, n_full, n_layers, traffic, workload, fp8=False)

    # dominant kernel of the timed step = largest share of the step's time
    share = {"indexer_score": kernels["indexer_score"]["ms_per_layer"] * n_full,
             "topk_select": kernels["topk_select"]["ms_per_layer"] * n_full,
             "sparse_attn": kernels["sparse_attn"]["ms_per_layer"] * n_layers}
    dom = max(share, key=share.get)
    kd = kernels[dom]
    roofline = {"kernel": dom, "bound": kd["bound"], "achieved": kd["achieved"], "peak": kd["peak"], "unit": kd["unit"],
                "frac": kd["frac"], "traffic": kd.get("traffic"),
                "traffic_unit": "HBM bytes per launch: rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a plain copy",
                "traffic_source": traffic.get("source"),
                "avg_launch_ms": kd["ms_per_layer"] / kd["launches_per_layer"],
                "timing": "HIP events around every launch of one 1-in-4 step, a pass of its own after the timed region",
                "share_of_step": share[dom] / sum(share.values())}
    if dom == "sparse_attn":
        roofline["gathered_GBs"] = kd["gathered_GBs"]
        roofline["compulsory_bytes"] = kd["compulsory_bytes"]
        roofline["note"] = ("algorithmic flops per launch (2 * H_q * (d_qk + d_v) per selected entry: k per query token, fewer on the first k - 1 rows of a sequence) against the bf16 MFMA peak; "
                            "the gathered rows (gathered_GBs, algorithmic) come out of L2 / Infinity Cache, the HBM side "
                            "moves only `traffic`")

    arms = {
        "prefill_1in4": {"ms_per_step": ms_14, "tokens_per_s": tokens / (ms_14 * 1e-3), "full_layers": n_full},
        "prefill_all_full": {"ms_per_step": ms_all, "tokens_per_s": tokens / (ms_all * 1e-3), "full_layers": n_layers},
        "prefill_speedup_1in4_vs_all_full": ms_all / ms_14,
    }

    if not args.no_calibrate:
        log("calibration arm")
        stack.step([True] + [False] * (n_layers - 1))           # idx_cache = layer 0's selection
        torch.cuda.synchronize()
        arms["calibration"] = calibration(ic, synth, stack.idx_cache if cfg["Tq"] == 32768 else None, cfg["Lk"])
        cal = arms["calibration"]
        if "prefill_attn_tile_path" in cal:
            # the kernel's own ceilings: its rows fetched in its own order with nothing done to them, and all of its
            # data movement (gather, LDS stores, both operand reads) with no arithmetic, in its best four-wave order
            tp = cal["prefill_attn_tile_path"]
            kernels["sparse_attn"]["gather_only_ms"] = min(tp["gather_into_registers_ms"], tp["plus_lds_store_ms"])
            kernels["sparse_attn"]["data_movement_only_ms"] = tp["same_bytes_phases_merged_ms"]
            kernels["sparse_attn"]["frac_of_data_movement_only"] = tp["same_bytes_phases_merged_ms"] / kernels["sparse_attn"]["ms_per_layer"]
        elif "prefill_row_gather" in cal:
            kernels["sparse_attn"]["gather_only_ms"] = cal["prefill_row_gather"]["ms"]
        kernels["sparse_attn"]["frac_of_measured_mfma"] = kernels["sparse_attn"]["achieved"] / cal["mfma_bf16"]["TFLOPs"]
        kernels["indexer_score"]["frac_of_measured_mfma"] = kernels["indexer_score"]["achieved"] / cal["mfma_bf16"]["TFLOPs"]

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
        try:
            dgraph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(dgraph):
                dstack.step(m_fsss)
            ms_d14_graph = time_steps(dgraph.replay, args.decode_steps, 3)
        except Exception as e:                               # an arm of its own: the headline does not depend on it
            log("decode graph arm failed: %s" % e)
            torch.cuda.synchronize()
            ms_d14_graph = None
        # per layer-step, from the two step times (launch gaps included; event pairs around 20 us
        # kernels would add their own few us each): FFFF - FSSS = three indexer + top-k runs
        d_idx = (ms_dall - ms_d14) / 3.0
        d_att = (ms_d14 - d_idx) / 4.0
        arms.update({
            "decode_1in4": {"ms_per_step": ms_d14, "tokens_per_s": dcfg["B"] / (ms_d14 * 1e-3), "pattern": "FSSS"},
            "decode_1in4_graph_replay": {"ms_per_step": ms_d14_graph,
                                         "tokens_per_s": dcfg["B"] / (ms_d14_graph * 1e-3) if ms_d14_graph else None,
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
        if "calibration" in arms:
            # the same bytes with no compute attached, through the library's calibration kernels
            dk, cal = arms["decode_kernels"], arms["calibration"]
            dk["indexer_plus_topk"]["stream_only_ms"] = cal["decode_key_stream"]["us"] * 1e-3
            dk["indexer_plus_topk"]["frac_of_stream_only"] = cal["decode_key_stream"]["us"] * 1e-3 / d_idx
            dk["sparse_attn_plus_merge"]["gather_only_ms"] = cal["decode_row_gather"]["us"] * 1e-3
            dk["sparse_attn_plus_merge"]["frac_of_gather_only"] = cal["decode_row_gather"]["us"] * 1e-3 / d_att
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
        # the bitmap form costs one AND and one population count per pair of layers (i <= j) and 32 positions, on
        # the vector ALUs: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-operations per second
        ov_ops = n_ov * (n_ov + 1) / 2 * ((ocfg["Lk"] + 31) // 32) * 2.0 * ocfg["Tq"]
        ov_peak = 256 * 64 * 2.4e9 / 1e12
        idx_bytes = n_ov * ocfg["Tq"] * ocfg["k_sel"] * 4
        arms["topk_overlap"] = {"layers": n_ov, "ms": ms_ov, "bound": "alu",
                                "achieved": ov_ops / (ms_ov * 1e-3) / 1e12, "peak": ov_peak,
                                "unit": "T lane-operations/s", "frac": ov_ops / (ms_ov * 1e-3) / 1e12 / ov_peak,
                                "index_bytes": idx_bytes, "index_bytes_GBs": idx_bytes / (ms_ov * 1e-3) / 1e9,
                                "note": "algorithmic work = pairs x ceil(Lk/32) words x (AND + popcount); the index rows are "
                                        "read once per chunk of the position range (two chunks at Lk = 32768)",
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

    # ---------------- configs[4]: the long-context fp8 stack (L = 131072, 64 fp8 indexer heads, 48 layers, 12 Full) ----------------
    if not args.no_fp8:
        torch.cuda.empty_cache()
        c4 = synth.config("c4", n_layers=args.fp8_layers)
        n4 = args.fp8_layers
        log("configs[4] stack: %d layers at L = %d (fp8 indexer)" % (n4, c4["Tq"]))
        s4 = Stack(ic, synth, c4, n4, max(1, min(args.fp8_distinct_q, n4)))
        m4_14 = ic.pattern_uniform(n4, 4)
        m4_all = [True] * n4
        alg4 = algorithmic(c4)
        ms4_14 = time_steps(lambda: s4.step(m4_14), 1, 1)
        ms4_all = time_steps(lambda: s4.step(m4_all), 1, 0)
        prof4 = profile_pass(ic, s4, m4_14)
        k4 = kernel_table(alg4, prof4, sum(m4_14), n4, traffic, "prefill131k_fp8", fp8=True)
        # the rows the last Full layer really selects out of its 151 MB cache, fetched with no compute attached (the
        # index tensor left by the profiled step is that layer's)
        l_last = max(l for l in range(n4) if m4_14[l])
        flat4 = s4.idx_cache.reshape(-1)
        scratch4 = torch.empty((1 << 16,), dtype=torch.int32, device="cuda")
        ms_g4 = event_ms(lambda: ic.calibrate(ic.CALIB_GATHER, s4.layers[l_last]["KV"], scratch4, idx=flat4, n=flat4.numel(),
                                              table_rows=c4["Lk"], row_bytes=1152, wgs=512), reps=2, warmup=1)
        k4["sparse_attn"]["gather_only_ms"] = ms_g4
        k4["sparse_attn"]["frac_of_gather_only"] = ms_g4 / k4["sparse_attn"]["ms_per_layer"]
        arms["prefill_fp8_131k"] = {
            "workload": "configs[4]: 1 sequence, L=131072, %d layers, H_I=64 d_I=128 e4m3 q/k with per-token scales, k=2048, "
                        "MQA 32 heads, KV row 576 bf16; every layer has its own KV and indexer inputs, Q cycles over %d tensors "
                        "and O is one buffer (48 x 4.8 GB of Q and 4.3 GB of O per layer do not fit beside the rest)"
                        % (n4, min(args.fp8_distinct_q, n4)),
            "prefill_1in4": {"ms_per_step": ms4_14, "tokens_per_s": c4["Tq"] / (ms4_14 * 1e-3), "full_layers": sum(m4_14), "steps": 1},
            "prefill_all_full": {"ms_per_step": ms4_all, "tokens_per_s": c4["Tq"] / (ms4_all * 1e-3), "full_layers": n4, "steps": 1},
            "prefill_speedup_1in4_vs_all_full": ms4_all / ms4_14,
            "kernels": k4,
        }
        del s4

    out = {
        "metric": "prefill & decode tokens/s, 48-layer DSA stack L=32K, 1-in-4 Full vs all-Full",
        "value": tokens / (ms_14 * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_14,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[3]: 48-layer attention-only DSA stack prefill, 1 sequence, L=32768, "
                               "H_I=32 d_I=128 k=2048, MQA 32 heads, KV row 576 bf16, 1-in-4 Full (value); "
                               "all-Full, decode (configs[2]) and the fp8 long-context stack (configs[4]) in arms",
                   "layers": n_layers, "pattern": "FSSS x%d" % (n_layers // 4), "L": cfg["Tq"], "k_sel": cfg["k_sel"],
                   "distinct_q_tensors": min(args.distinct_attn_inputs, n_layers), "distinct_kv_and_indexer_inputs": n_layers},
        "roofline": roofline,
        "kernels": kernels,
        "arms": arms,
        "cpu_baseline": cpu,
        "bench_wall_s": time.perf_counter() - t_start,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
