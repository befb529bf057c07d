#!/usr/bin/env python3
"""Benchmark of the AWEQ calibration + quantization hot path on one MI355X.

A step = one pass of the whole path (statistics, equalization, weight quantizer,
activation quantizer + W8A8 int8 GEMM, bias correction) over every linear layer of one
decoder block, on synthetic inputs already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--cfg 2] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_PEAK_TOPS = 5000.0   # MI355X dense int8 MFMA, published
HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, published
F16_PEAK_TFLOPS = 2500.0  # MI355X dense fp16 MFMA, published

# HBM bytes per GEMM launch, measured with `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE`
# on this workload (profiles/gemm_i8_fast_opt6.7b_hbm_traffic.txt), scaled by what the same
# counters read for a plain 1 GiB device copy (FETCH x2.0, WRITE x1.0).  Keyed by (N, K), T = 262144.
GEMM_TRAFFIC_BYTES = {
    (4096, 4096): (6.79e9, 4.57e9),
    (16384, 4096): (26.0e9, 18.3e9),
    (4096, 16384): (29.1e9, 4.56e9),
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--cfg", type=int, default=2, help="workload number (1 single 512x512 layer, 2 OPT-6.7B block, 3 LLaMA-7B block, 5 LLaMA-65B block)")
    ap.add_argument("--tokens", type=int, default=0, help="override the number of calibration tokens (debug)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--out-deq", action="store_true", help="GEMM writes the de-quantised fp16 output instead of int32")
    ap.add_argument("--weight-only", type=int, default=0, choices=(0, 3, 4),
                    help="weight-only calibration (workload 4, LLaMA-7B shapes): W4 or W3 per group of 128, fp16 activations "
                         "(statistics, equalization, weight quantizer, bias correction; no GEMM); implies --cfg 4")
    ap.add_argument("--block", action="store_true",
                    help="run the block with its real data flow: linears that read the same activation (q/k/v, gate/up) "
                         "share one statistics pass, one equalization scale and one activation quantization")
    ap.add_argument("--layers", default="", help="comma-separated layer names to keep (profiling runs)")
    ap.add_argument("--mfma-probe", action="store_true",
                    help="only measure the sustained shader clock / MFMA rate for three kinds of operand data and exit")
    ap.add_argument("--library-gemm", action="store_true",
                    help="context, not the product: time the ROCm library's int8 GEMM (torch._int_mm) and fp16 GEMM on "
                         "the operands one calibrated layer produces, next to aweq_w8a8_gemm / aweq_wonly_gemm")
    ap.add_argument("--fused-chain", action="store_true",
                    help="OPT-6.7B fc1 -> ReLU -> fc2: the statistics pass and the activation quantizer of fc2's input as "
                         "passes of their own over fc1's output, against aweq_w8a8_gemm_fused doing them in fc1's epilogue")
    ap.add_argument("--ablation", action="store_true",
                    help="context: output error of the quantised layer on the synthetic workload for the AWE x BC grid "
                         "(W8A8, and W4 / W3 weight-only), first linear of --cfg at 32768 tokens")
    ap.add_argument("--copy-probe", type=int, default=0,
                    help="only run a plain device copy of this many bytes (reference for the HBM counters) and exit")
    return ap.parse_args()


SHARED_INPUT_GROUPS = (("q_proj", "k_proj", "v_proj"), ("gate_proj", "up_proj"))


def block_bench(args, torch, B, pipeline, synth, dev):
    """W8A8 calibration of a block with shared inputs (Sec. 3.1: equalization sits at the entrance of
    the attention block and of the MLP): the call sequence of pipeline.calibrate_group with the GEMMs
    bracketed by events."""
    wl = synth.WORKLOADS[args.cfg]
    T = args.tokens or wl.T
    tdt = torch.float16 if wl.dtype == "f16" else torch.float32
    dt = B.AWEQ_F16 if wl.dtype == "f16" else B.AWEQ_F32
    groups, seen = [], set()
    for li, lin in enumerate(wl.linears):
        if lin.name in seen:
            continue
        names = next((g for g in SHARED_INPUT_GROUPS if lin.name in g), (lin.name,))
        members = [(j, l) for j, l in enumerate(wl.linears) if l.name in names]
        seen.update(l.name for _, l in members)
        seed = synth.layer_seed(wl.cfg, li)
        X = synth.make_act_torch(seed, T, lin.K, wl, dev)
        Ws = [synth.make_weight_torch(synth.layer_seed(wl.cfg, j), l.N, l.K, wl.dtype, dev) for j, l in members]
        bs = []
        for j, l in members:
            b = synth.make_bias_np(synth.layer_seed(wl.cfg, j), l.N, wl.has_bias)
            bs.append(torch.from_numpy(b).to(dev) if b is not None else None)
        gb = pipeline.GroupBuffers(T, lin.K, tuple(l.N for _, l in members), tdt, want_out_i32=True, device=dev)
        groups.append(([l for _, l in members], X, Ws, bs, gb))
    torch.cuda.synchronize()
    n_layers = sum(len(g[0]) for g in groups)

    def run_group(lins, X, Ws, bs, gb, ev=None):
        t, K, st = gb.t, gb.K, gb.t["status"]
        B.aweq_calib_stats(X, dt, T, K, K, t["xmin"], t["xmax"], t["xsum"], t["count"], 0, 1, t["r_x"], t["R_x"],
                           t["p_x"], t["ws"], st)
        for i, W in enumerate(Ws):
            B.aweq_calib_stats(W, dt, W.shape[0], K, K, t["wmin"], t["wmax"], None, t["wcount"], int(i > 0),
                               int(i == len(Ws) - 1), t["r_w"], t["R_w"], t["p_w"], t["ws"], st)
        for W, p in zip(Ws, gb.per):
            N = W.shape[0]
            B.aweq_equalize(t["xmin"], t["xmax"], t["xsum"], T, t["wmin"], t["wmax"], K, 1, t["s"], t["inv_s"], W,
                            p["W_hat"], dt, N, K, None, t["xhat_range"], t["mu_xhat"], t["act_step"], t["act_zero"], st)
            B.aweq_quant_weight(p["W_hat"], dt, N, K, K, 8, 0, p["codes"], p["step_w"], p["zero_w"], p["rowsum_w"],
                                t["ws"], st)
        B.aweq_quant_act(X, dt, T, K, K, t["inv_s"], t["act_step"], t["act_zero"], t["xq"], t["rowsum_x"],
                         t["colsum_xq"], st)
        for i, (W, b, p) in enumerate(zip(Ws, bs, gb.per)):
            N = W.shape[0]
            if ev is not None:
                ev[i][0].record()
            B.aweq_w8a8_gemm(t["xq"], B.AWEQ_I8, T, K, K, None, t["act_step"], t["act_zero"], None, t["rowsum_x"], None,
                             p["codes"], N, p["step_w"], p["zero_w"], p["rowsum_w"], b, p["out_i32"], None, dt, N,
                             p["colsum_acc"], None, st)
            if ev is not None:
                ev[i][1].record()
            B.aweq_bias_correct(B.BIAS_W8A8, p["W_hat"], dt, N, K, K, t["mu_xhat"], T, p["colsum_acc"], t["colsum_xq"],
                                p["rowsum_w"], t["act_step"], t["act_zero"], None, 8, 0, p["step_w"], p["zero_w"], b,
                                p["delta"], p["bias_out"], 1, None, st)

    for _ in range(args.warmup):
        for g in groups:
            run_group(*g)
    torch.cuda.synchronize()
    evs = [[[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in g[0]] for g in groups]
           for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        for gi, g in enumerate(groups):
            run_group(*g, evs[k][gi])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    gemm_ms = sum(e0.elapsed_time(e1) for k in range(args.steps) for gi in range(len(groups)) for e0, e1 in evs[k][gi])
    gemm_ops = args.steps * sum(2.0 * T * l.N * l.K for g in groups for l in g[0])
    gemm_tops = gemm_ops / (gemm_ms * 1e-3) / 1e12
    status_bits = 0
    for g in groups:
        status_bits |= int(g[4].t["status"].item())
    return {
        "metric": "calibration tokens/sec per layer (stats+equalize+quant+bias); W8A8 GEMM TOPS",
        "value": n_layers * T / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"cfg{wl.cfg} {wl.name}: {n_layers} linears on {len(groups)} distinct inputs (shared-input "
                               f"groups {[[l.name for l in g[0]] for g in groups]}), T={T} calibration tokens, {wl.dtype} in, "
                               "W8 per-channel / A8 per-tensor, GEMM output int32 + column sums",
                   "value_is": "layers * T / step time, whole block with one statistics pass and one activation "
                               "quantization per distinct input"},
        "gemm_tops": gemm_tops,
        "roofline": {"bound": "mfma", "kernel": "gemm_i8_fast", "achieved": gemm_tops, "peak": INT8_PEAK_TOPS,
                     "unit": "TFLOP/s", "frac": gemm_tops / INT8_PEAK_TOPS, "traffic": None,
                     "note": "int8 multiply-add = 2 ops (TOP/s); achieved = sum 2*T*N*K / sum of event-timed GEMM launches"},
        "status_bits": status_bits,
    }


def weight_only_bench(args, torch, B, pipeline, synth, dev):
    """Workload 4 (weight-only): every linear of the LLaMA-7B-shaped block through statistics, equalization,
    the W4 / W3 group-128 weight quantizer and the weight-only bias correction."""
    wl = synth.WORKLOADS[4]
    T = args.tokens or wl.T
    bits = args.weight_only
    layers = []
    for li, lin in enumerate(wl.linears):
        seed = synth.layer_seed(wl.cfg, li)
        X = synth.make_act_torch(seed, T, lin.K, wl, dev)
        W = synth.make_weight_torch(seed, lin.N, lin.K, wl.dtype, dev)
        buf = pipeline.LayerBuffers(T, lin.K, lin.N, torch.float16, bits=bits, group=128, w8a8=False, device=dev)
        buf.t["y"] = torch.empty((T, lin.N), dtype=torch.float16, device=dev)
        buf.t["ws_fw"] = torch.empty(B.aweq_workspace_size(B.OP_WONLY_GEMM, T, lin.K, lin.N), dtype=torch.uint8, device=dev)
        layers.append((lin, X, W, buf))
    torch.cuda.synchronize()
    dt = B.AWEQ_F16
    stages = ("stats_x", "stats_w", "equalize", "quant_weight", "bias", "forward")

    def run_layer(lin, X, W, buf, ev=None):
        t, K, N, st = buf.t, lin.K, lin.N, buf.t["status"]

        def mark(i):
            if ev is not None:
                ev[i].record()
        mark(0)
        B.aweq_calib_stats(X, dt, T, K, K, t["xmin"], t["xmax"], t["xsum"], t["count"], 0, 1, t["r_x"], t["R_x"],
                           t["p_x"], t["ws"], st)
        mark(1)
        B.aweq_calib_stats(W, dt, N, K, K, t["wmin"], t["wmax"], None, t["wcount"], 0, 1, t["r_w"], t["R_w"],
                           t["p_w"], t["ws"], st)
        mark(2)
        B.aweq_equalize(t["xmin"], t["xmax"], t["xsum"], T, t["wmin"], t["wmax"], K, 1, t["s"], t["inv_s"], W,
                        t["W_hat"], dt, N, K, None, t["xhat_range"], t["mu_xhat"], t["act_step"], t["act_zero"], st)
        mark(3)
        B.aweq_quant_weight(t["W_hat"], dt, N, K, K, bits, 128, t["codes"], t["step_w"], t["zero_w"], None, t["ws"], st)
        mark(4)
        B.aweq_bias_correct(B.BIAS_WEIGHT_ONLY, t["W_hat"], dt, N, K, K, t["mu_xhat"], T, None, None, None, None, None,
                            t["codes"], bits, 128, t["step_w"], t["zero_w"], None, t["delta"], t["bias_out"], 1, None, st)
        mark(5)
        # the quantised layer's forward with the corrected bias; the synthetic X stands in for the
        # equalised binary16 activations the preceding block would deliver
        B.aweq_wonly_gemm(X, T, K, K, t["codes"], bits, 128, t["step_w"], t["zero_w"], N, t["bias_out"], t["y"],
                          B.AWEQ_F16, N, t["ws_fw"], st)
        mark(6)

    for _ in range(args.warmup):
        for lay in layers:
            run_layer(*lay)
    torch.cuda.synchronize()
    evs = [[[torch.cuda.Event(enable_timing=True) for _ in range(7)] for _ in layers] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        for i, lay in enumerate(layers):
            run_layer(*lay, evs[k][i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    per_layer, sx_ms, sx_bytes, fw_ms, fw_flops, calib_ms = [], 0.0, 0.0, 0.0, 0.0, 0.0
    for i, (lin, *_r) in enumerate(layers):
        ms = {s: sum(evs[k][i][j].elapsed_time(evs[k][i][j + 1]) for k in range(args.steps)) / args.steps
              for j, s in enumerate(stages)}
        sx_ms += ms["stats_x"]
        sx_bytes += 2.0 * T * lin.K
        fw_ms += ms["forward"]
        fw_flops += 2.0 * T * lin.N * lin.K
        calib_ms += sum(v for s, v in ms.items() if s != "forward")
        per_layer.append({"name": lin.name, "N": lin.N, "K": lin.K, "ms": {s: round(v, 4) for s, v in ms.items()},
                          "stats_x_GBs": round(2.0 * T * lin.K / (ms["stats_x"] * 1e-3) / 1e9, 1),
                          "forward_TFLOPs": round(2.0 * T * lin.N * lin.K / (ms["forward"] * 1e-3) / 1e12, 1)})
    status_bits = 0
    for *_r, buf in layers:
        status_bits |= int(buf.t["status"].item())
    achieved = sx_bytes / (sx_ms * 1e-3) / 1e9
    fw_tflops = fw_flops / (fw_ms * 1e-3) / 1e12
    return {
        "metric": "calibration tokens/sec per layer (stats+equalize+quant+bias); W8A8 GEMM TOPS",
        "value": len(layers) * T / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"cfg4 {wl.name}: {len(layers)} linears, T={T} calibration tokens, f16, weight-only "
                               f"W{bits} per group of 128, fp16 activations, equalization + bias correction, then "
                               "the de-quantising fp16 forward GEMM",
                   "value_is": "layers * T / step time, whole path incl. the weight-only forward"},
        "calib_tokens_per_s_per_layer_excl_forward": T * len(layers) / (calib_ms * 1e-3),
        "forward_tflops": fw_tflops,
        "roofline": {"bound": "mfma", "kernel": "gemm_f16_kernel<true> (after dequant_weight_h_kernel)", "achieved": fw_tflops,
                     "peak": F16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": fw_tflops / F16_PEAK_TFLOPS, "traffic": None,
                     "note": "achieved = sum 2*T*N*K / sum of event-timed aweq_wonly_gemm launches"},
        "roofline_stats": {"bound": "hbm", "kernel": "col_stats_partial_f16 (+ merge, finalize: the whole aweq_calib_stats call on X)",
                           "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                           "note": "achieved = 2 B x T x K of X over the event-timed aweq_calib_stats calls (3 kernels each)"},
        "layers": per_layer, "status_bits": status_bits,
    }


def cpu_baseline(wl, lin, seed, tokens):
    """The oracle, as it stands, on a bounded sample of the same workload (host cores)."""
    import numpy as np
    from oracle import aweq_oracle as orc
    from paper_2311_01305_amd import synth
    X = synth.make_act_np(seed, tokens, lin.K, wl)
    W = synth.make_weight_np(seed, lin.N, lin.K, wl.dtype)
    b = synth.make_bias_np(seed, lin.N, wl.has_bias)
    t0 = time.perf_counter()
    sx, sw = orc.col_stats(X), orc.col_stats(W, want_sum=False)
    r_x, _, _ = orc.ranges(sx["cmin"], sx["cmax"])
    r_w, _, _ = orc.ranges(sw["cmin"], sw["cmax"])
    s, inv_s, _ = orc.scales(r_x, r_w)
    Wh = orc.fold_weight(W, s)
    lo, hi, mu = orc.xhat_stats(sx["cmin"], sx["cmax"], sx["csum"], sx["count"], inv_s)
    step, zero, _ = orc.qparams(lo, hi, 8)
    q = orc.quant_weight(Wh, 8, 0)
    wq = orc.pack_codes(q["codes_u"], 8)
    a = orc.quant_act(X, inv_s, step, zero)
    acc = orc.gemm_i8(a["xq"], wq)
    csa = acc.astype(np.int64).sum(axis=0)
    orc.bias_w8a8(Wh, mu, tokens, csa, a["colsum_xq"], q["rowsum_w"], step, zero, q["step"], q["zero"], b)
    dt = time.perf_counter() - t0
    return {"value": tokens / dt, "unit": "tokens/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"{lin.name} {lin.N}x{lin.K} of cfg {wl.cfg}, {tokens} of {wl.T} calibration tokens, "
                      f"all stages incl. int8 GEMM, {dt:.2f} s"}


def mfma_probe(torch, B, dev, iters=20000, reps=12):
    """Sustained shader clock and int8 MFMA rate with no memory traffic, per kind of operand data."""
    out = torch.zeros(3, dtype=torch.int64, device=dev)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    res = {}
    for mode, name, ops in ((0, "constant_bytes", 65536), (1, "random_bytes", 65536), (2, "small_signed_codes", 65536),
                            (3, "f16_32x32x16_random_values", 32768)):
        for _ in range(reps):  # the clock settles over a few tens of milliseconds
            B.aweq_probe_mfma_clock(iters, mode, out)
        cyc, ticks = int(out[0].item()), int(out[1].item())
        res[name] = {"shader_clock_GHz": cyc / ticks * 0.1, "cycles_per_mfma": cyc / (16.0 * iters),
                     "TOPs": cus * 4 * 16.0 * iters * ops / (ticks * 1e-8) / 1e12}
    return {"mfma_probe": res, "compute_units": cus}


def library_gemm(args, torch, B, pipeline, synth, dev):
    """The vendor library's GEMMs on the same operands and the same box, as context for the
    rooflines: int8 (torch._int_mm) against aweq_w8a8_gemm on the codes a calibrated layer
    produces, fp16 (torch.matmul) against aweq_wonly_gemm.  Nothing of the product runs through
    the library; this only says what its tuned kernels reach here."""
    wl = synth.WORKLOADS[args.cfg]
    T = args.tokens or wl.T
    keep = set(x for x in args.layers.split(",") if x) or {wl.linears[0].name}
    out = []

    def timed(fn, n=10, w=4):
        for _ in range(w):
            fn()
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for a, b in ev:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) for a, b in ev)
        return ts[len(ts) // 2]

    for li, lin in enumerate(wl.linears):
        if lin.name not in keep:
            continue
        seed = synth.layer_seed(wl.cfg, li)
        X = synth.make_act_torch(seed, T, lin.K, wl, dev)
        W = synth.make_weight_torch(seed, lin.N, lin.K, wl.dtype, dev)
        buf = pipeline.LayerBuffers(T, lin.K, lin.N, torch.float16, device=dev)
        t = pipeline.calibrate_layer(X, W, None, buf, fused_weight_pass=True)
        torch.cuda.synchronize()
        K, N = lin.K, lin.N
        ops = 2.0 * T * N * K
        ours = timed(lambda: B.aweq_w8a8_gemm(t["xq"], B.AWEQ_I8, T, K, K, None, None, None, None, None, None, t["codes"], N,
                                              None, None, None, None, t["out_i32"], None, B.AWEQ_F16, N, None, None))
        ours_cs = timed(lambda: B.aweq_w8a8_gemm(t["xq"], B.AWEQ_I8, T, K, K, None, None, None, None, None, None, t["codes"], N,
                                                 None, None, None, None, t["out_i32"], None, B.AWEQ_F16, N, t["colsum_acc"], None))
        xq_rm = torch.empty((T, K), dtype=torch.int8, device=dev)
        wq_rm = torch.empty((N, K), dtype=torch.int8, device=dev)
        B.aweq_unpack_panels_i8(t["xq"], T, K, xq_rm, K)
        B.aweq_unpack_panels_i8(t["codes"], N, K, wq_rm, K)
        ref_out = t["out_i32"].clone()
        lib_ms = timed(lambda: torch._int_mm(xq_rm, wq_rm.t(), out=t["out_i32"]))
        same = bool(torch.equal(ref_out, t["out_i32"]))
        del ref_out, xq_rm, wq_rm
        # fp16: the library on X and the folded weight, ours on W4 codes of the same weight
        y = torch.empty((T, N), dtype=torch.float16, device=dev)
        lib_h = timed(lambda: torch.matmul(X, t["W_hat"].t(), out=y))
        bw = pipeline.LayerBuffers(T, K, N, torch.float16, bits=4, group=128, w8a8=False, device=dev)
        tw = pipeline.calibrate_layer(X, W, None, bw)
        ws = torch.empty(B.aweq_workspace_size(B.OP_WONLY_GEMM, T, K, N), dtype=torch.uint8, device=dev)
        ours_h = timed(lambda: B.aweq_wonly_gemm(X, T, K, K, tw["codes"], 4, 128, tw["step_w"], tw["zero_w"], N, None, y,
                                                 B.AWEQ_F16, N, ws))
        out.append({"name": lin.name, "T": T, "N": N, "K": K,
                    "int8_TOPs": {"aweq_w8a8_gemm_int32_out": ops / ours / 1e9, "aweq_w8a8_gemm_int32_out_colsum": ops / ours_cs / 1e9,
                                  "library_int_mm": ops / lib_ms / 1e9, "outputs_identical": same},
                    "fp16_TFLOPs": {"aweq_wonly_gemm_w4": ops / ours_h / 1e9, "library_matmul": ops / lib_h / 1e9}})
        del X, W, buf, t, bw, tw, y, ws
        torch.cuda.empty_cache()
    return {"library_gemm": out, "workload": f"cfg{wl.cfg} {wl.name}"}


def fused_chain(args, torch, B, pipeline, synth, dev):
    """fc1 -> ReLU -> fc2 of the OPT-6.7B-shaped block: what the fused epilogues save.
    Calibration flow: fc2's statistics come out of fc1's GEMM (its output is still stored and
    quantised by a pass of its own once fc2's scales exist).  Deployed flow (static scales
    known): fc1's GEMM writes fc2's int8 codes directly and no binary16 output at all."""
    wl = synth.WORKLOADS[2]
    T = args.tokens or wl.T
    fc1, fc2 = wl.linears[4], wl.linears[5]
    seed = synth.layer_seed(wl.cfg, 4)
    X = synth.make_act_torch(seed, T, fc1.K, wl, dev)
    W1 = synth.make_weight_torch(seed, fc1.N, fc1.K, wl.dtype, dev)
    b1 = torch.from_numpy(synth.make_bias_np(seed, fc1.N, True)).to(dev)
    W2 = synth.make_weight_torch(synth.layer_seed(wl.cfg, 5), fc2.N, fc2.K, wl.dtype, dev)
    buf = pipeline.LayerBuffers(T, fc1.K, fc1.N, torch.float16, want_out_i32=False, want_out_deq=True, device=dev)
    t = pipeline.calibrate_layer(X, W1, b1, buf, fused_weight_pass=True)
    torch.cuda.synchronize()
    del X
    K, N = fc1.K, fc1.N
    y = t["out_deq"]
    y.clamp_(min=0)                       # ReLU: fc2's input for the separate passes
    b2 = pipeline.LayerBuffers(T, fc2.K, fc2.N, torch.float16, want_out_i32=False, device=dev)
    u = b2.t
    f32, i32, i64 = torch.float32, torch.int32, torch.int64
    e = lambda *shape, dtype: torch.empty(shape, dtype=dtype, device=dev)
    ws = e(B.aweq_workspace_size(B.OP_W8A8_GEMM, T, K, N), dtype=torch.uint8)
    fmin, fmax, fsum, fcnt = e(N, dtype=f32), e(N, dtype=f32), e(N, dtype=torch.float64), torch.zeros(1, dtype=i64, device=dev)
    yq, rsy, csy = e(B.aweq_panel_bytes(T, N), dtype=torch.int8), e(T, dtype=i32), e(N, dtype=i64)

    def gemm_plain():
        B.aweq_w8a8_gemm(t["xq"], B.AWEQ_I8, T, K, K, None, t["act_step"], t["act_zero"], None, t["rowsum_x"], None, t["codes"],
                         N, t["step_w"], t["zero_w"], t["rowsum_w"], b1, None, y, B.AWEQ_F16, N, t["colsum_acc"], None)

    def stats_y():
        B.aweq_calib_stats(y, B.AWEQ_F16, T, N, N, u["xmin"], u["xmax"], u["xsum"], u["count"], 0, 1, u["r_x"], u["R_x"],
                           u["p_x"], u["ws"])

    def quant_y():
        B.aweq_quant_act(y, B.AWEQ_F16, T, N, N, u["inv_s"], u["act_step"], u["act_zero"], u["xq"], u["rowsum_x"], u["colsum_xq"])

    def fused(store, stats, quant):
        B.aweq_w8a8_gemm_fused(t["xq"], T, K, t["codes"], N, t["act_step"], t["act_zero"], t["step_w"], t["zero_w"],
                               t["rowsum_x"], t["rowsum_w"], b1, 1, y if store else None, N, t["colsum_acc"],
                               fmin if stats else None, fmax if stats else None, fsum if stats else None,
                               fcnt if stats else None, 0, u["inv_s"] if quant else None, u["act_step"] if quant else None,
                               u["act_zero"] if quant else None, yq if quant else None, rsy if quant else None,
                               csy if quant else None, ws)

    # fc2's scales from the separate statistics pass (the fused statistics must agree: checked below)
    stats_y()
    B.aweq_calib_stats(W2, B.AWEQ_F16, fc2.N, fc2.K, fc2.K, u["wmin"], u["wmax"], None, u["wcount"], 0, 1, u["r_w"], u["R_w"],
                       u["p_w"], u["ws"])
    B.aweq_equalize(u["xmin"], u["xmax"], u["xsum"], T, u["wmin"], u["wmax"], fc2.K, 1, u["s"], u["inv_s"], None, u["W_hat"],
                    B.AWEQ_F16, fc2.N, fc2.K, None, u["xhat_range"], u["mu_xhat"], u["act_step"], u["act_zero"])
    quant_y()
    fused(True, True, True)
    torch.cuda.synchronize()
    same = bool(torch.equal(fmin, u["xmin"]) and torch.equal(fmax, u["xmax"]) and torch.equal(yq, u["xq"])
                and torch.equal(rsy, u["rowsum_x"]) and torch.equal(csy, u["colsum_xq"]))

    def timed(fn, n=6, w=3):
        for _ in range(w):
            fn()
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for a, b in ev:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) for a, b in ev)
        return ts[len(ts) // 2]

    ms = {"gemm_fp16_out": timed(gemm_plain), "stats_pass_over_y": timed(stats_y), "quant_act_pass_over_y": timed(quant_y),
          "gemm_fused_statistics_fp16_out": timed(lambda: fused(True, True, False)),
          "gemm_fused_codes_no_fp16_out": timed(lambda: fused(False, False, True)),
          "gemm_fused_statistics_and_codes_fp16_out": timed(lambda: fused(True, True, True))}
    ops = 2.0 * T * N * K
    return {"fused_chain": {"layers": "cfg2 fc1 (16384 x 4096) -> ReLU -> fc2 input", "T": T, "ms": {k: round(v, 4) for k, v in ms.items()},
                            "calibration_flow_ms": {"separate": round(ms["gemm_fp16_out"] + ms["stats_pass_over_y"], 4),
                                                    "fused": round(ms["gemm_fused_statistics_fp16_out"], 4)},
                            "deployed_flow_ms": {"separate": round(ms["gemm_fp16_out"] + ms["quant_act_pass_over_y"], 4),
                                                 "fused": round(ms["gemm_fused_codes_no_fp16_out"], 4)},
                            "gemm_TOPs": {k: round(ops / v / 1e9, 1) for k, v in ms.items() if k.startswith("gemm")},
                            "fused_results_identical_to_separate_passes": same}}


def ablation(args, torch, B, pipeline, synth, dev):
    """The switches of the paper's ablation (equalization on / off, bias correction on / off) on one
    synthetic layer: relative RMS error and mean error of the quantised layer's output against the
    fp64 product of the un-quantised layer.  Context only: synthetic tensors, not the paper's tasks."""
    wl = synth.WORKLOADS[args.cfg]
    T = args.tokens or 32768
    lin = wl.linears[0]
    seed = synth.layer_seed(wl.cfg, 0)
    X = synth.make_act_torch(seed, T, lin.K, wl, dev)
    W = synth.make_weight_torch(seed, lin.N, lin.K, wl.dtype, dev)
    b_np = synth.make_bias_np(seed, lin.N, wl.has_bias)
    b = None if b_np is None else torch.from_numpy(b_np).to(dev)
    K, N = lin.K, lin.N
    y = X.to(torch.float64) @ W.to(torch.float64).t()        # the reference the error is measured against
    if b is not None:
        y += b.to(torch.float64)
    rms_y = float(y.pow(2).mean().sqrt())
    rows = []
    for mode, bits in (("w8a8", 8), ("w4 g128, fp16 activations", 4), ("w3 g128, fp16 activations", 3)):
        for awe in (0, 1):
            for bc in (0, 1):
                if bits == 8:
                    buf = pipeline.LayerBuffers(T, K, N, torch.float16, want_out_i32=False, want_out_deq=True, device=dev)
                    t = pipeline.calibrate_layer(X, W, b, buf, enable_awe=bool(awe), enable_bc=bool(bc))
                    yq = t["out_deq"].to(torch.float64)
                    if b is not None:
                        yq -= b.to(torch.float64)
                    yq += t["bias_out"].to(torch.float64)
                else:
                    buf = pipeline.LayerBuffers(T, K, N, torch.float16, bits=bits, group=128, w8a8=False, device=dev)
                    t = pipeline.calibrate_layer(X, W, b, buf, enable_awe=bool(awe), enable_bc=bool(bc))
                    # the deployed layer sees the equalised activation: X diag(s)^-1 in binary16
                    Xh = (X.to(torch.float32) * t["inv_s"]).to(torch.float16)
                    yh = torch.empty((T, N), dtype=torch.float32, device=dev)
                    ws = torch.empty(B.aweq_workspace_size(B.OP_WONLY_GEMM, T, K, N), dtype=torch.uint8, device=dev)
                    B.aweq_wonly_gemm(Xh, T, K, K, t["codes"], bits, 128, t["step_w"], t["zero_w"], N, t["bias_out"], yh,
                                      B.AWEQ_F32, N, ws)
                    yq = yh.to(torch.float64)
                e = yq - y
                rows.append({"mode": mode, "awe": awe, "bc": bc, "rel_rms_error": float(e.pow(2).mean().sqrt()) / rms_y,
                             "max_abs_channel_mean_error": float(e.mean(dim=0).abs().max()),
                             "status_bits": int(t["status"].item())})
                del buf, t, yq, e
    return {"ablation": rows, "layer": f"cfg{wl.cfg} {lin.name} {N}x{K}", "T": T, "rms_of_reference_output": rms_y}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU; --gpus must be 1 (no multi-GPU path exists: the "
              "calibration path shards over tokens or layers without changing the kernels)", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2311_01305_amd import binding as B
    from paper_2311_01305_amd import pipeline, synth

    B.load_library()  # raises if libaweq.so is missing: no fallback
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.mfma_probe:
        print(json.dumps(mfma_probe(torch, B, dev)))
        return
    if args.library_gemm:
        print(json.dumps(library_gemm(args, torch, B, pipeline, synth, dev)))
        return
    if args.ablation:
        print(json.dumps(ablation(args, torch, B, pipeline, synth, dev)))
        return
    if args.fused_chain:
        print(json.dumps(fused_chain(args, torch, B, pipeline, synth, dev)))
        return
    if args.copy_probe:
        # a plain copy kernel of known size: what FETCH_SIZE / WRITE_SIZE read for it gives the
        # factor that turns those counters into bytes
        src = torch.empty(args.copy_probe, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        dst.copy_(src)
        e0.record()
        for _ in range(5):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 5
        print(json.dumps({"copy_probe_bytes": args.copy_probe, "ms": ms,
                          "GBs_read_plus_write": 2 * args.copy_probe / ms / 1e6}))
        return
    if args.weight_only:
        print(json.dumps(weight_only_bench(args, torch, B, pipeline, synth, dev)))
        return
    if args.block:
        print(json.dumps(block_bench(args, torch, B, pipeline, synth, dev)))
        return
    wl = synth.WORKLOADS[args.cfg]
    T = args.tokens or wl.T
    tdt = torch.float16 if wl.dtype == "f16" else torch.float32
    dt = B.AWEQ_F16 if wl.dtype == "f16" else B.AWEQ_F32

    layers = []
    keep = set(x for x in args.layers.split(",") if x)
    for li, lin in enumerate(wl.linears):
        if keep and lin.name not in keep:
            continue
        seed = synth.layer_seed(wl.cfg, li)
        X = synth.make_act_torch(seed, T, lin.K, wl, dev)
        W = synth.make_weight_torch(seed, lin.N, lin.K, wl.dtype, dev)
        b = synth.make_bias_np(seed, lin.N, wl.has_bias)
        b = torch.from_numpy(b).to(dev) if b is not None else None
        buf = pipeline.LayerBuffers(T, lin.K, lin.N, tdt, want_out_i32=not args.out_deq, want_out_deq=args.out_deq,
                                    device=dev)
        layers.append((lin, X, W, b, buf))
    torch.cuda.synchronize()

    stages = ("stats_x", "stats_w", "equalize", "quant_weight", "quant_act", "gemm", "bias")

    def run_layer(lin, X, W, b, buf, ev=None):
        """The same call sequence as pipeline.calibrate_layer, with the activation quantizer and
        the GEMM issued as two calls so that each can be bracketed by events."""
        t = buf.t
        K, N = lin.K, lin.N
        st = t["status"]

        def mark(i):
            if ev is not None:
                ev[i].record()
        mark(0)
        B.aweq_calib_stats(X, dt, T, K, K, t["xmin"], t["xmax"], t["xsum"], t["count"], 0, 1, t["r_x"], t["R_x"],
                           t["p_x"], t["ws"], st)
        mark(1)
        B.aweq_calib_stats(W, dt, N, K, K, t["wmin"], t["wmax"], None, t["wcount"], 0, 1, t["r_w"], t["R_w"],
                           t["p_w"], t["ws"], st)
        mark(2)
        B.aweq_equalize(t["xmin"], t["xmax"], t["xsum"], T, t["wmin"], t["wmax"], K, 1, t["s"], t["inv_s"], None,
                        None, dt, N, K, None, t["xhat_range"], t["mu_xhat"], t["act_step"], t["act_zero"], st)
        mark(3)
        # fold (Eq. 3) and per-channel quantizer in one pass over W
        B.aweq_fold_quant_weight(W, dt, N, K, K, t["s"], t["W_hat"], 8, t["codes"], t["step_w"], t["zero_w"],
                                 t["rowsum_w"], st)
        mark(4)
        B.aweq_quant_act(X, dt, T, K, K, t["inv_s"], t["act_step"], t["act_zero"], t["xq"], t["rowsum_x"],
                         t["colsum_xq"], st)
        mark(5)
        B.aweq_w8a8_gemm(t["xq"], B.AWEQ_I8, T, K, K, None, t["act_step"], t["act_zero"], None, t["rowsum_x"], None,
                         t["codes"], N, t["step_w"], t["zero_w"], t["rowsum_w"], b, t.get("out_i32"), t.get("out_deq"),
                         dt, N, t["colsum_acc"], None, st)
        mark(6)
        B.aweq_bias_correct(B.BIAS_W8A8, t["W_hat"], dt, N, K, K, t["mu_xhat"], T, t["colsum_acc"], t["colsum_xq"],
                            t["rowsum_w"], t["act_step"], t["act_zero"], None, 8, 0, t["step_w"], t["zero_w"], b,
                            t["delta"], t["bias_out"], 1, None, st)
        mark(7)

    def step(evs=None):
        for i, (lin, X, W, b, buf) in enumerate(layers):
            run_layer(lin, X, W, b, buf, None if evs is None else evs[i])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    all_evs = [[[torch.cuda.Event(enable_timing=True) for _ in range(8)] for _ in layers] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(all_evs[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_per_step = wall * 1e3 / args.steps

    # the same layers calibrated without the forward (outside the timed region of `value`): the bias
    # correction takes the accumulator's sums over tokens from the weight codes, the activation
    # quantizer only forms its sums
    def calib_only_step():
        for lin, X, W, b, buf in layers:
            t, K, N, st = buf.t, lin.K, lin.N, buf.t["status"]
            B.aweq_calib_stats(X, dt, T, K, K, t["xmin"], t["xmax"], t["xsum"], t["count"], 0, 1, t["r_x"], t["R_x"],
                               t["p_x"], t["ws"], st)
            B.aweq_calib_stats(W, dt, N, K, K, t["wmin"], t["wmax"], None, t["wcount"], 0, 1, t["r_w"], t["R_w"],
                               t["p_w"], t["ws"], st)
            B.aweq_equalize(t["xmin"], t["xmax"], t["xsum"], T, t["wmin"], t["wmax"], K, 1, t["s"], t["inv_s"], None,
                            None, dt, N, K, None, t["xhat_range"], t["mu_xhat"], t["act_step"], t["act_zero"], st)
            B.aweq_fold_quant_weight(W, dt, N, K, K, t["s"], t["W_hat"], 8, t["codes"], t["step_w"], t["zero_w"],
                                     t["rowsum_w"], st)
            B.aweq_quant_act(X, dt, T, K, K, t["inv_s"], t["act_step"], t["act_zero"], None, None, t["colsum_xq"], st)
            B.aweq_bias_correct(B.BIAS_W8A8, t["W_hat"], dt, N, K, K, t["mu_xhat"], T, None, t["colsum_xq"],
                                t["rowsum_w"], t["act_step"], t["act_zero"], t["codes"], 8, 0, t["step_w"], t["zero_w"], b,
                                t["delta"], t["bias_out"], 1, None, st)

    ref_bias = [buf.t["bias_out"].clone() for *_r, buf in layers]
    calib_only_step()
    torch.cuda.synchronize()
    calib_same = all(torch.equal(r, buf.t["bias_out"]) for r, (*_r, buf) in zip(ref_bias, layers))
    t0 = time.perf_counter()
    for _ in range(args.steps):
        calib_only_step()
    torch.cuda.synchronize()
    calib_only_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    # per-stage device time from the events (ms, summed over steps)
    stage_ms = {s: [0.0] * len(layers) for s in stages}
    for k in range(args.steps):
        for i in range(len(layers)):
            for j, s in enumerate(stages):
                stage_ms[s][i] += all_evs[k][i][j].elapsed_time(all_evs[k][i][j + 1])
    n_gemm = args.steps * len(layers)
    gemm_ms_total = sum(stage_ms["gemm"])
    gemm_ops_total = args.steps * sum(2.0 * T * lin.N * lin.K for lin, *_ in layers)
    gemm_tops = gemm_ops_total / (gemm_ms_total * 1e-3) / 1e12
    calib_ms = sum(sum(stage_ms[s]) for s in ("stats_x", "stats_w", "equalize", "quant_weight", "bias"))
    tokens_per_s = len(layers) * T / (ms_per_step * 1e-3)

    esz = 2 if wl.dtype == "f16" else 4
    per_layer = []
    for i, (lin, *_rest) in enumerate(layers):
        ms = {s: stage_ms[s][i] / args.steps for s in stages}
        per_layer.append({
            "name": lin.name, "N": lin.N, "K": lin.K,
            "ms": {s: round(v, 4) for s, v in ms.items()},
            "stats_x_GBs": round(T * lin.K * esz / (ms["stats_x"] * 1e-3) / 1e9, 1),
            "quant_act_GBs": round(T * lin.K * (esz + 1) / (ms["quant_act"] * 1e-3) / 1e9, 1),
            "gemm_TOPs": round(2.0 * T * lin.N * lin.K / (ms["gemm"] * 1e-3) / 1e12, 1),
        })

    # the two streaming passes over X against the HBM peak (event-timed calls, all layers of the step)
    sx_bytes = sum(T * lin.K * esz for lin, *_ in layers)
    qa_bytes = sum(T * lin.K * (esz + 1) for lin, *_ in layers)
    sx_ms = sum(pl["ms"]["stats_x"] for pl in per_layer)
    qa_ms = sum(pl["ms"]["quant_act"] for pl in per_layer)
    hbm_passes = [
        {"bound": "hbm", "kernel": "col_stats_partial_f16 + merge + finalize (the aweq_calib_stats call on X)",
         "achieved": sx_bytes / (sx_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
         "frac": sx_bytes / (sx_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "bytes_per_element": esz},
        {"bound": "hbm", "kernel": "quant_act_kernel (+ two fill kernels: the aweq_quant_act call)",
         "achieved": qa_bytes / (qa_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
         "frac": qa_bytes / (qa_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "bytes_per_element": esz + 1}]

    traffic = None
    if T == 262144 and all((lin.N, lin.K) in GEMM_TRAFFIC_BYTES for lin, *_ in layers):
        traffic = sum(sum(GEMM_TRAFFIC_BYTES[(lin.N, lin.K)]) for lin, *_ in layers) / len(layers) / 1e9
    algorithmic_gb = sum(T * lin.K + lin.N * lin.K + 4.0 * T * lin.N for lin, *_ in layers) / len(layers) / 1e9

    status_bits = 0
    for _lin, _X, _W, _b, buf in layers:
        status_bits |= int(buf.t["status"].item())

    out = {
        "metric": "calibration tokens/sec per layer (stats+equalize+quant+bias); W8A8 GEMM TOPS",
        "value": tokens_per_s,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": f"cfg{wl.cfg} {wl.name}: {len(layers)} linears, T={T} calibration tokens, "
                               f"{wl.dtype} in, W8 per-channel / A8 per-tensor, "
                               f"GEMM output {'fp16 de-quantised' if args.out_deq else 'int32'} + column sums",
                   "value_is": "layers * T / step time, whole path incl. activation quantizer and int8 GEMM"},
        "calib_tokens_per_s_per_layer_excl_w8a8": T * len(layers) / (calib_ms / args.steps * 1e-3),
        "gemm_tops": gemm_tops,
        "roofline": {"bound": "mfma", "kernel": "gemm_i8_kernel", "achieved": gemm_tops, "peak": INT8_PEAK_TOPS,
                     "unit": "TFLOP/s", "frac": gemm_tops / INT8_PEAK_TOPS, "traffic": traffic,
                     "traffic_unit": "GB of HBM traffic per launch (fetch + write, mean over the layer shapes; "
                                     f"algorithmic {algorithmic_gb:.1f} GB: operands once + int32 output)",
                     "note": "int8 multiply-add = 2 ops (TOP/s); achieved = sum 2*T*N*K / sum of event-timed GEMM "
                             f"launches ({n_gemm} launches, avg {gemm_ms_total / n_gemm:.3f} ms)"},
        "calibration_without_forward": {
            "ms_per_step": calib_only_ms, "tokens_per_s_per_layer": T * len(layers) / (calib_only_ms * 1e-3),
            "bias_identical_to_the_run_with_the_gemm": calib_same,
            "note": "statistics, equalization, weight quantizer, sums-only activation quantizer, bias correction from "
                    "wq . colsum_xq (exact): what a W8A8 calibration needs when the forward itself is not wanted"},
        "roofline_hbm_passes": hbm_passes,
        "layers": per_layer,
        "status_bits": status_bits,
    }
    if not args.no_cpu_baseline:
        lin0 = wl.linears[0]
        out["cpu_baseline"] = cpu_baseline(wl, lin0, synth.layer_seed(wl.cfg, 0), min(T, 8192))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
