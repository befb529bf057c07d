#!/usr/bin/env python3
"""Benchmark of the AWEQ calibration + quantization hot path on one MI355X.

A step = one pass of the whole path (statistics, equalization, weight quantizer,
activation quantizer + W8A8 int8 GEMM, bias correction) over every linear layer of one
decoder block, on synthetic inputs already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

With no further flags the line is for the LLaMA-65B-shaped block (the largest workload that
fits one GPU), every linear with its own calibration input, and carries three more objects:
`north_star_block` (the LLaMA-7B-shaped block run with its real data flow: linears that read the
same activation share one statistics pass, one scale and one activation quantization),
`weight_only` (the LLaMA-7B shapes with W4 / W3 group-128 weights: calibration and the
de-quantising fp16 forward) and `cpu_baseline` (the CPU oracle timed stage by stage).
`--cfg N`, `--block`, `--weight-only B` select one of these as the line itself.
"""
import argparse
import ctypes
import glob
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_PEAK_TOPS = 5000.0   # MI355X dense int8 MFMA, published
HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, published
F16_PEAK_TFLOPS = 2500.0  # MI355X dense fp16 MFMA, published
METRIC = "calibration tokens/sec per layer (stats+equalize+quant+bias); W8A8 GEMM TOPS"
DEFAULT_CFG = 5
SHARED_INPUT_GROUPS = (("q_proj", "k_proj", "v_proj"), ("gate_proj", "up_proj"))


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--cfg", type=int, default=0,
                    help="only this workload (1 single 512x512 layer, 2 OPT-6.7B block, 3 LLaMA-7B block, 5 LLaMA-65B block); "
                         "default: 5 plus the north_star_block / weight_only objects")
    ap.add_argument("--tokens", type=int, default=0, help="override the number of calibration tokens (debug)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--out-deq", action="store_true", help="GEMM writes the de-quantised fp16 output instead of int32")
    ap.add_argument("--weight-only", type=int, default=0, choices=(0, 3, 4),
                    help="only the weight-only workload (4, LLaMA-7B shapes): W4 or W3 per group of 128, fp16 activations")
    ap.add_argument("--block", action="store_true",
                    help="run --cfg with the block's real data flow: linears that read the same activation (q/k/v, gate/up) "
                         "share one statistics pass, one equalization scale and one activation quantization")
    ap.add_argument("--layers", default="", help="comma-separated layer names to keep (profiling runs)")
    ap.add_argument("--mfma-probe", action="store_true",
                    help="only measure the sustained shader clock / MFMA rate for several kinds of operand data and exit")
    ap.add_argument("--stream-probe", action="store_true",
                    help="only measure what bare streaming kernels (read only, copy, 2 bytes read per byte written) reach "
                         "on this box and exit")
    ap.add_argument("--fused-chain", action="store_true",
                    help="OPT-6.7B fc1 -> ReLU -> fc2: the statistics pass and the activation quantizer of fc2's input as "
                         "passes of their own over fc1's output, against aweq_w8a8_gemm_fused doing them in fc1's epilogue")
    ap.add_argument("--ablation", action="store_true",
                    help="context: output error of the quantised layer on the synthetic workload for the AWE x BC grid "
                         "(W8A8, and W4 / W3 weight-only), first linear of --cfg at 32768 tokens")
    ap.add_argument("--copy-probe", type=int, default=0,
                    help="only run a plain device copy of this many bytes (reference for the HBM counters) and exit")
    return ap.parse_args()


# ------------------------------------------------------------------------------------ helpers

def measured_gemm_traffic():
    """HBM bytes per gemm_i8_fast launch from the rocprofv3 --pmc summaries under profiles/
    (lines `traffic: kernel=gemm_i8_fast T=.. N=.. K=.. fetch_GB=.. write_GB=..`), keyed by (T, N, K)."""
    table = {}
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*hbm_traffic*.txt"))):
        for line in open(path):
            if not line.startswith("traffic:") or "kernel=gemm_i8_fast" not in line:
                continue
            kv = dict(re.findall(r"(\w+)=([\w.+-]+)", line))
            try:
                table[(int(kv["T"]), int(kv["N"]), int(kv["K"]))] = (float(kv["fetch_GB"]), float(kv["write_GB"]),
                                                                     os.path.basename(path))
            except (KeyError, ValueError):
                pass
    return table


def gemm_roofline(shapes, T, gemm_ms_total, n_launches, out_bytes=4):
    """`roofline` of the dominant kernel.  shapes: (N, K) of every launch of one step; gemm_ms_total /
    n_launches: event-timed durations over all timed steps."""
    steps = n_launches / len(shapes)
    ops = steps * sum(2.0 * T * N * K for N, K in shapes)
    tops = ops / (gemm_ms_total * 1e-3) / 1e12
    table = measured_gemm_traffic()
    per_shape, src = {}, set()
    for N, K in sorted(set(shapes)):
        if (T, N, K) in table:
            f, w, name = table[(T, N, K)]
            per_shape[f"N={N},K={K}"] = {"fetch_GB": f, "write_GB": w,
                                         "algorithmic_GB": round((T * K + N * K + out_bytes * T * N) / 1e9, 2)}
            src.add(name)
    traffic = None
    if len(per_shape) == len(set(shapes)):
        traffic = sum(sum(table[(T, N, K)][:2]) for N, K in shapes) / len(shapes)
    algorithmic = sum(T * K + N * K + out_bytes * T * N for N, K in shapes) / len(shapes) / 1e9
    return {"bound": "mfma", "kernel": "aweq::fast::gemm_i8_fast (v_mfma_i32_32x32x32_i8)", "achieved": tops,
            "peak": INT8_PEAK_TOPS, "unit": "TOP/s", "frac": tops / INT8_PEAK_TOPS, "traffic": traffic,
            "traffic_unit": "GB of memory traffic per launch behind the L2 (rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE, scaled by a "
                            f"plain copy; mean over the step's launches; algorithmic {algorithmic:.1f} GB: operands once + output)",
            "traffic_by_shape": per_shape or None, "traffic_source": sorted(src) or None,
            "note": "int8 multiply-add = 2 ops; achieved = sum 2*T*N*K / sum of event-timed launch durations on the launch "
                    f"stream ({n_launches} launches, avg {gemm_ms_total / n_launches:.3f} ms)"}


def make_inputs(torch, synth, wl, T, dev, keep=()):
    """Per linear: its own calibration input X, weight W and bias (seeded, generated on the device)."""
    layers = []
    for li, lin in enumerate(wl.linears):
        if keep and lin.name not in keep:
            continue
        seed = synth.layer_seed(wl.cfg, li)
        X = synth.make_act_torch(seed, T, lin.K, wl, dev)
        W = synth.make_weight_torch(seed, lin.N, lin.K, wl.dtype, dev)
        b = synth.make_bias_np(seed, lin.N, wl.has_bias)
        layers.append((lin, X, W, torch.from_numpy(b).to(dev) if b is not None else None))
    return layers


# ---------------------------------------------------------------- W8A8, one input per linear

def layer_bench(args, torch, B, pipeline, synth, dev, cfg):
    """The whole path over every linear of the block, each with its own calibration input."""
    wl = synth.WORKLOADS[cfg]
    T = args.tokens or wl.T
    tdt = torch.float16 if wl.dtype == "f16" else torch.float32
    dt = B.AWEQ_F16 if wl.dtype == "f16" else B.AWEQ_F32
    keep = set(x for x in args.layers.split(",") if x)
    layers = []
    for lin, X, W, b in make_inputs(torch, synth, wl, T, dev, keep):
        buf = pipeline.LayerBuffers(T, lin.K, lin.N, tdt, want_out_i32=not args.out_deq, want_out_deq=args.out_deq, device=dev)
        layers.append((lin, X, W, b, buf))
    torch.cuda.synchronize()
    stages = ("stats_x", "stats_w", "equalize", "quant_weight", "quant_act", "gemm", "bias")

    def run_layer(lin, X, W, b, buf, ev=None):
        """The call sequence of pipeline.calibrate_layer, with the activation quantizer and the GEMM
        issued as two calls so that each can be bracketed by events."""
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
        B.aweq_equalize(t["xmin"], t["xmax"], t["xsum"], T, t["wmin"], t["wmax"], K, 1, t["s"], t["inv_s"], None,
                        None, dt, N, K, K, None, t["xhat_range"], t["mu_xhat"], t["act_step"], t["act_zero"], st)
        mark(3)
        # fold (Eq. 3) and per-channel quantizer in one pass over W
        B.aweq_fold_quant_weight(W, dt, N, K, K, t["s"], t["W_hat"], K, 8, t["codes"], t["step_w"], t["zero_w"],
                                 t["rowsum_w"], st)
        mark(4)
        B.aweq_quant_act(X, dt, T, K, K, t["inv_s"], t["act_step"], t["act_zero"], t["xq"], t["rowsum_x"],
                         t["colsum_xq"], t["ws"], st)
        mark(5)
        B.aweq_w8a8_gemm(t["xq"], B.AWEQ_I8, T, K, K, None, t["act_step"], t["act_zero"], None, t["rowsum_x"], None,
                         t["codes"], N, t["step_w"], t["zero_w"], 0, t["rowsum_w"], b, t.get("out_i32"), t.get("out_deq"),
                         dt, N, t["colsum_acc"], None, st)
        mark(6)
        B.aweq_bias_correct(B.BIAS_W8A8, t["W_hat"], dt, N, K, K, t["mu_xhat"], T, t["colsum_acc"], t["colsum_xq"],
                            t["rowsum_w"], t["act_step"], t["act_zero"], None, 8, 0, t["step_w"], t["zero_w"], b,
                            t["delta"], t["bias_out"], 1, st)
        mark(7)

    def step(evs=None):
        for i, lay in enumerate(layers):
            run_layer(*lay, None if evs is None else evs[i])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    all_evs = [[[torch.cuda.Event(enable_timing=True) for _ in range(8)] for _ in layers] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(all_evs[k])
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

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
                            None, dt, N, K, K, None, t["xhat_range"], t["mu_xhat"], t["act_step"], t["act_zero"], st)
            B.aweq_fold_quant_weight(W, dt, N, K, K, t["s"], t["W_hat"], K, 8, t["codes"], t["step_w"], t["zero_w"],
                                     t["rowsum_w"], st)
            B.aweq_quant_act(X, dt, T, K, K, t["inv_s"], t["act_step"], t["act_zero"], None, None, t["colsum_xq"], t["ws"], st)
            B.aweq_bias_correct(B.BIAS_W8A8, t["W_hat"], dt, N, K, K, t["mu_xhat"], T, None, t["colsum_xq"],
                                t["rowsum_w"], t["act_step"], t["act_zero"], t["codes"], 8, 0, t["step_w"], t["zero_w"], b,
                                t["delta"], t["bias_out"], 1, st)

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
    gemm_ms_total = sum(stage_ms["gemm"])
    calib_ms = sum(sum(stage_ms[s]) for s in ("stats_x", "stats_w", "equalize", "quant_weight", "bias"))
    esz = 2 if wl.dtype == "f16" else 4
    per_layer = []
    for i, (lin, *_rest) in enumerate(layers):
        ms = {s: stage_ms[s][i] / args.steps for s in stages}
        per_layer.append({
            "name": lin.name, "N": lin.N, "K": lin.K, "ms": {s: round(v, 4) for s, v in ms.items()},
            "stats_x_GBs": round(T * lin.K * esz / (ms["stats_x"] * 1e-3) / 1e9, 1),
            "quant_act_GBs": round(T * lin.K * (esz + 1) / (ms["quant_act"] * 1e-3) / 1e9, 1),
            "gemm_TOPs": round(2.0 * T * lin.N * lin.K / (ms["gemm"] * 1e-3) / 1e12, 1)})

    # the two streaming passes over X against the HBM peak (event-timed calls, all layers of the step)
    sx_bytes = sum(T * lin.K * esz for lin, *_ in layers)
    qa_bytes = sum(T * lin.K * (esz + 1) for lin, *_ in layers)
    sx_ms = sum(pl["ms"]["stats_x"] for pl in per_layer)
    qa_ms = sum(pl["ms"]["quant_act"] for pl in per_layer)
    hbm_passes = [
        {"bound": "hbm", "kernel": "col_stats_partial_f16 + merge + finalize (the aweq_calib_stats call on X)",
         "achieved": sx_bytes / (sx_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
         "frac": sx_bytes / (sx_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "bytes_per_element": esz},
        {"bound": "hbm", "kernel": "quant_act_kernel + quant_act_merge (the aweq_quant_act call)",
         "achieved": qa_bytes / (qa_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
         "frac": qa_bytes / (qa_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "bytes_per_element": esz + 1}]
    status_bits = 0
    for *_r, buf in layers:
        status_bits |= int(buf.t["status"].item())
    roof = gemm_roofline([(lin.N, lin.K) for lin, *_ in layers], T, gemm_ms_total, args.steps * len(layers),
                         out_bytes=2 if args.out_deq else 4)
    out = {
        "metric": METRIC, "value": len(layers) * T / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"cfg{wl.cfg} {wl.name}: {len(layers)} linears, each with its own calibration input, T={T} "
                               f"calibration tokens, {wl.dtype} in, W8 per-channel / A8 per-tensor, GEMM output "
                               f"{'fp16 de-quantised' if args.out_deq else 'int32'} + column sums",
                   "value_is": "layers * T / step time, whole path incl. activation quantizer and int8 GEMM"},
        "calib_tokens_per_s_per_layer_excl_w8a8": T * len(layers) / (calib_ms / args.steps * 1e-3),
        "gemm_tops": roof["achieved"], "roofline": roof,
        "calibration_without_forward": {
            "ms_per_step": calib_only_ms, "tokens_per_s_per_layer": T * len(layers) / (calib_only_ms * 1e-3),
            "bias_identical_to_the_run_with_the_gemm": calib_same,
            "note": "statistics, equalization, weight quantizer, sums-only activation quantizer, bias correction from "
                    "wq . colsum_xq (exact): what a W8A8 calibration needs when the forward itself is not wanted"},
        "roofline_hbm_passes": hbm_passes, "layers": per_layer, "status_bits": status_bits}
    del layers
    return out


# ---------------------------------------------------------------- W8A8, shared inputs (block)

def block_bench(args, torch, B, pipeline, synth, dev, cfg):
    """W8A8 calibration of a block with shared inputs (Sec. 3.1: equalization sits at the entrance of
    the attention block and of the MLP): the call sequence of pipeline.calibrate_group with every
    stage bracketed by events."""
    wl = synth.WORKLOADS[cfg]
    T = args.tokens or wl.T
    tdt = torch.float16 if wl.dtype == "f16" else torch.float32
    dt = B.AWEQ_F16 if wl.dtype == "f16" else B.AWEQ_F32
    esz = 2 if wl.dtype == "f16" else 4
    groups, seen = [], set()
    for li, lin in enumerate(wl.linears):
        if lin.name in seen:
            continue
        names = next((g for g in SHARED_INPUT_GROUPS if lin.name in g), (lin.name,))
        members = [(j, l) for j, l in enumerate(wl.linears) if l.name in names]
        seen.update(l.name for _, l in members)
        X = synth.make_act_torch(synth.layer_seed(wl.cfg, li), T, lin.K, wl, dev)
        Ws = [synth.make_weight_torch(synth.layer_seed(wl.cfg, j), l.N, l.K, wl.dtype, dev) for j, l in members]
        bs = []
        for j, l in members:
            b = synth.make_bias_np(synth.layer_seed(wl.cfg, j), l.N, wl.has_bias)
            bs.append(torch.from_numpy(b).to(dev) if b is not None else None)
        gb = pipeline.GroupBuffers(T, lin.K, tuple(l.N for _, l in members), tdt, want_out_i32=True, device=dev)
        groups.append(([l for _, l in members], X, Ws, bs, gb))
    torch.cuda.synchronize()
    n_layers = sum(len(g[0]) for g in groups)

    def run_group(lins, X, Ws, bs, gb, rec=None):
        t, K, st = gb.t, gb.K, gb.t["status"]

        def mark(name):
            if rec is not None:
                e = torch.cuda.Event(enable_timing=True)
                e.record()
                rec.append((name, e))
        mark("stats_x")
        B.aweq_calib_stats(X, dt, T, K, K, t["xmin"], t["xmax"], t["xsum"], t["count"], 0, 1, t["r_x"], t["R_x"],
                           t["p_x"], t["ws"], st)
        mark("weight_side")
        for i, W in enumerate(Ws):
            B.aweq_calib_stats(W, dt, W.shape[0], K, K, t["wmin"], t["wmax"], None, t["wcount"], int(i > 0),
                               int(i == len(Ws) - 1), t["r_w"], t["R_w"], t["p_w"], t["ws"], st)
        B.aweq_equalize(t["xmin"], t["xmax"], t["xsum"], T, t["wmin"], t["wmax"], K, 1, t["s"], t["inv_s"], None, None,
                        dt, 0, K, K, None, t["xhat_range"], t["mu_xhat"], t["act_step"], t["act_zero"], st)
        for W, p in zip(Ws, gb.per):
            B.aweq_fold_quant_weight(W, dt, W.shape[0], K, K, t["s"], p["W_hat"], K, 8, p["codes"], p["step_w"], p["zero_w"],
                                     p["rowsum_w"], st)
        mark("quant_act")
        B.aweq_quant_act(X, dt, T, K, K, t["inv_s"], t["act_step"], t["act_zero"], t["xq"], t["rowsum_x"],
                         t["colsum_xq"], t["ws"], st)
        for W, b, p in zip(Ws, bs, gb.per):
            N = W.shape[0]
            mark("gemm")
            B.aweq_w8a8_gemm(t["xq"], B.AWEQ_I8, T, K, K, None, t["act_step"], t["act_zero"], None, t["rowsum_x"], None,
                             p["codes"], N, p["step_w"], p["zero_w"], 0, p["rowsum_w"], b, p["out_i32"], None, dt, N,
                             p["colsum_acc"], None, st)
            mark("bias")
            B.aweq_bias_correct(B.BIAS_W8A8, p["W_hat"], dt, N, K, K, t["mu_xhat"], T, p["colsum_acc"], t["colsum_xq"],
                                p["rowsum_w"], t["act_step"], t["act_zero"], None, 8, 0, p["step_w"], p["zero_w"], b,
                                p["delta"], p["bias_out"], 1, st)
        mark("end")

    for _ in range(args.warmup):
        for g in groups:
            run_group(*g)
    torch.cuda.synchronize()
    recs = [[[] for _ in groups] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        for gi, g in enumerate(groups):
            run_group(*g, recs[k][gi])
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    tot = {}
    for k in range(args.steps):
        for gi in range(len(groups)):
            r = recs[k][gi]
            for (name, e0), (_n, e1) in zip(r[:-1], r[1:]):
                tot[name] = tot.get(name, 0.0) + e0.elapsed_time(e1)
    shapes = [(l.N, l.K) for g in groups for l in g[0]]
    roof = gemm_roofline(shapes, T, tot["gemm"], args.steps * n_layers)
    sx_bytes = args.steps * sum(T * g[4].K * esz for g in groups)
    qa_bytes = args.steps * sum(T * g[4].K * (esz + 1) for g in groups)
    status_bits = 0
    for g in groups:
        status_bits |= int(g[4].t["status"].item())
    out = {
        "metric": METRIC, "value": n_layers * T / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"cfg{wl.cfg} {wl.name}: {n_layers} linears on {len(groups)} distinct inputs (shared-input "
                               f"groups {[[l.name for l in g[0]] for g in groups]}), T={T} calibration tokens, {wl.dtype} in, "
                               "W8 per-channel / A8 per-tensor, GEMM output int32 + column sums",
                   "value_is": "layers * T / step time, whole block with one statistics pass and one activation "
                               "quantization per distinct input"},
        "calib_tokens_per_s_per_layer_excl_w8a8":
            n_layers * T / ((tot["stats_x"] + tot["weight_side"] + tot["bias"]) / args.steps * 1e-3),
        "gemm_tops": roof["achieved"], "roofline": roof,
        "stage_ms_per_step": {k: round(v / args.steps, 4) for k, v in tot.items()},
        "stats_x_GBs": sx_bytes / (tot["stats_x"] * 1e-3) / 1e9, "quant_act_GBs": qa_bytes / (tot["quant_act"] * 1e-3) / 1e9,
        "status_bits": status_bits}
    del groups
    return out


# ------------------------------------------------------------------------------ weight-only

def weight_only_bench(args, torch, B, pipeline, synth, dev, bits):
    """Workload 4 (weight-only): every linear of the LLaMA-7B-shaped block through statistics, equalization,
    the W4 / W3 group-128 weight quantizer, the weight-only bias correction and the de-quantising forward."""
    wl = synth.WORKLOADS[4]
    T = args.tokens or wl.T
    layers = []
    for lin, X, W, _b in make_inputs(torch, synth, wl, T, dev):
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
                        t["W_hat"], dt, N, K, K, None, t["xhat_range"], t["mu_xhat"], t["act_step"], t["act_zero"], st)
        mark(3)
        B.aweq_quant_weight(t["W_hat"], dt, N, K, K, bits, 128, t["codes"], t["step_w"], t["zero_w"], None, t["ws"], st)
        mark(4)
        B.aweq_bias_correct(B.BIAS_WEIGHT_ONLY, t["W_hat"], dt, N, K, K, t["mu_xhat"], T, None, None, None, None, None,
                            t["codes"], bits, 128, t["step_w"], t["zero_w"], None, t["delta"], t["bias_out"], 1, st)
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
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
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
    out = {
        "metric": METRIC, "value": len(layers) * T / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"cfg4 {wl.name}: {len(layers)} linears, T={T} calibration tokens, f16, weight-only "
                               f"W{bits} per group of 128, fp16 activations, equalization + bias correction, then "
                               "the de-quantising fp16 forward GEMM",
                   "value_is": "layers * T / step time, whole path incl. the weight-only forward"},
        "calib_tokens_per_s_per_layer_excl_forward": T * len(layers) / (calib_ms * 1e-3),
        "forward_tflops": fw_tflops,
        "roofline": {"bound": "mfma", "kernel": "aweq::gemm_f16_kernel (v_mfma_f32_32x32x16_f16, after dequant_weight_h_kernel)",
                     "achieved": fw_tflops, "peak": F16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": fw_tflops / F16_PEAK_TFLOPS,
                     "traffic": None, "note": "achieved = sum 2*T*N*K / sum of event-timed aweq_wonly_gemm calls"},
        "roofline_stats": {"bound": "hbm", "kernel": "col_stats_partial_f16 (+ merge, finalize: the whole aweq_calib_stats call on X)",
                           "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                           "note": "achieved = 2 B x T x K of X over the event-timed aweq_calib_stats calls"},
        "layers": per_layer, "status_bits": status_bits}
    del layers
    return out


# ------------------------------------------------------------------------------ CPU oracle

def cpu_baseline(wl, lin, X_dev, W_dev, b_dev, t_sub=1024):
    """The oracle, as it stands, timed stage by stage on the host cores: the streaming stages
    (statistics, equalization, weight quantizer, activation quantizer, bias correction through the
    linearity identities) on ALL calibration tokens of one layer of the benchmarked workload, its
    triple-loop int8 GEMM on the first t_sub tokens with the extrapolation to all tokens labelled."""
    import numpy as np
    from oracle import aweq_oracle as orc
    X = X_dev.cpu().numpy()
    W = W_dev.cpu().numpy()
    b = None if b_dev is None else b_dev.cpu().numpy()
    T = X.shape[0]
    sec = {}

    def timed(name, fn):
        t0 = time.perf_counter()
        r = fn()
        sec[name] = sec.get(name, 0.0) + time.perf_counter() - t0
        return r
    sx = timed("stats_x", lambda: orc.col_stats(X))
    sw = timed("stats_w", lambda: orc.col_stats(W, want_sum=False))

    def eq():
        r_x, _, _ = orc.ranges(sx["cmin"], sx["cmax"])
        r_w, _, _ = orc.ranges(sw["cmin"], sw["cmax"])
        s, inv_s, _ = orc.scales(r_x, r_w)
        lo, hi, mu = orc.xhat_stats(sx["cmin"], sx["cmax"], sx["csum"], sx["count"], inv_s)
        step, zero, _ = orc.qparams(lo, hi, 8)
        return s, inv_s, mu, step, zero
    s, inv_s, mu, step, zero = timed("equalize", eq)
    Wh = timed("equalize", lambda: orc.fold_weight(W, s))
    q = timed("quant_weight", lambda: orc.quant_weight(Wh, 8, 0))
    wq = timed("quant_weight", lambda: orc.pack_codes(q["codes_u"], 8))
    a = timed("quant_act", lambda: orc.quant_act(X, inv_s, step, zero))
    sub = min(t_sub, T)
    acc = timed("gemm_sub", lambda: orc.gemm_i8(np.ascontiguousarray(a["xq"][:sub]), wq))
    del acc
    csa = orc.colsum_acc_from_colsum_xq(wq, a["colsum_xq"])   # (the GEMM's column sums, by the identity the tests pin)
    timed("bias", lambda: orc.bias_w8a8(Wh, mu, T, csa, a["colsum_xq"], q["rowsum_w"], step, zero, q["step"], q["zero"], b))
    calib = sec["stats_x"] + sec["stats_w"] + sec["equalize"] + sec["quant_weight"] + sec["bias"]
    gemm_full = sec["gemm_sub"] * T / sub
    ops_sub = 2.0 * sub * lin.N * lin.K
    return {"value": T / calib, "unit": "tokens/s", "cores": orc.num_threads(), "kind": "oracle",
            "value_is": "the metric's first half for one layer: T / (statistics + equalization + weight quantizer + bias "
                        "correction), all T tokens, measured",
            "sample": f"{lin.name} {lin.N}x{lin.K} of cfg {wl.cfg}: streaming stages on all {T} calibration tokens "
                      f"({sum(v for k, v in sec.items() if k != 'gemm_sub'):.1f} s), int8 GEMM on the first {sub} tokens "
                      f"({sec['gemm_sub']:.1f} s)",
            "stage_seconds": {k: round(v, 3) for k, v in sec.items()},
            "quant_act_tokens_per_s": T / sec["quant_act"],
            "gemm": {"tokens": sub, "seconds": sec["gemm_sub"], "GOPs": ops_sub / sec["gemm_sub"] / 1e9,
                     "seconds_extrapolated_to_all_tokens": gemm_full,
                     "note": "linear extrapolation from the token subset, not measured"},
            "whole_path_tokens_per_s_extrapolated": T / (calib + sec["quant_act"] + gemm_full)}


# ------------------------------------------------------------------------------ probes

def load_probes():
    path = os.path.join(ROOT, "libbench_probes.so")
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -c 'import __graft_entry__ as g; g.build_probes()'`")
    import torch  # noqa: F401  (its HIP runtime must be the one in the process)
    lib = ctypes.CDLL(path)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    lib.bench_probe_mfma_clock.restype = i32
    lib.bench_probe_mfma_clock.argtypes = [i32, i32, vp, vp]
    lib.bench_probe_stream.restype = i32
    lib.bench_probe_stream.argtypes = [i32, vp, vp, i64, i32, vp, vp]
    return lib


def mfma_probe(torch, dev, iters=20000, reps=12):
    """Sustained shader clock and MFMA rate with no memory traffic, per kind of operand data."""
    lib = load_probes()
    out = torch.zeros(3, dtype=torch.int64, device=dev)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    st = torch.cuda.current_stream().cuda_stream
    res = {}
    for mode, name, ops in ((0, "constant_bytes", 65536), (1, "random_bytes", 65536), (2, "small_signed_codes", 65536),
                            (3, "f16_32x32x16_random_values", 32768), (4, "small_codes_first_operand_random_second", 65536),
                            (5, "random_first_operand_small_codes_second", 65536)):
        for _ in range(reps):  # the clock settles over a few tens of milliseconds
            assert lib.bench_probe_mfma_clock(iters, mode, out.data_ptr(), st) == 0
        cyc, ticks = int(out[0].item()), int(out[1].item())
        res[name] = {"shader_clock_GHz": cyc / ticks * 0.1, "cycles_per_mfma": cyc / (16.0 * iters),
                     "TOPs": cus * 4 * 16.0 * iters * ops / (ticks * 1e-8) / 1e12}
    return {"mfma_probe": res, "compute_units": cus}


def stream_probe(torch, dev, nbytes=1 << 32, reps=10):
    """What bare streaming kernels reach on this machine: the ceiling of an HBM-bound pass per read : write mix."""
    lib = load_probes()
    src = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    src.random_(0, 255)
    dst = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    st = torch.cuda.current_stream().cuda_stream
    res = {}
    for mode, name, moved in ((0, "read_only", nbytes), (1, "copy_1_read_1_written", 2 * nbytes),
                              (2, "2_read_1_written", nbytes + nbytes // 2)):
        best = None
        for blocks in (1024, 2048, 4096, 8192, 16384):
            for _ in range(2):
                assert lib.bench_probe_stream(mode, src.data_ptr(), dst.data_ptr(), nbytes, blocks, sink.data_ptr(), st) == 0
            torch.cuda.synchronize()
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
            for a, b in ev:
                a.record()
                lib.bench_probe_stream(mode, src.data_ptr(), dst.data_ptr(), nbytes, blocks, sink.data_ptr(), st)
                b.record()
            torch.cuda.synchronize()
            ts = sorted(a.elapsed_time(b) for a, b in ev)
            gbs = moved / (ts[len(ts) // 2] * 1e-3) / 1e9
            if best is None or gbs > best[0]:
                best = (gbs, blocks, ts[len(ts) // 2])
        res[name] = {"GBs": best[0], "frac_of_8000": best[0] / HBM_PEAK_GBS, "blocks": best[1], "ms": best[2],
                     "bytes_moved": moved}
    return {"stream_probe": res, "buffer_bytes": nbytes}


# ------------------------------------------------------------------- context modes (not the line)

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
                         N, t["step_w"], t["zero_w"], 0, t["rowsum_w"], b1, None, y, B.AWEQ_F16, N, t["colsum_acc"], None)

    def stats_y():
        B.aweq_calib_stats(y, B.AWEQ_F16, T, N, N, u["xmin"], u["xmax"], u["xsum"], u["count"], 0, 1, u["r_x"], u["R_x"],
                           u["p_x"], u["ws"])

    def quant_y():
        B.aweq_quant_act(y, B.AWEQ_F16, T, N, N, u["inv_s"], u["act_step"], u["act_zero"], u["xq"], u["rowsum_x"], u["colsum_xq"],
                         u["ws"])

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
                    B.AWEQ_F16, fc2.N, fc2.K, fc2.K, None, u["xhat_range"], u["mu_xhat"], u["act_step"], u["act_zero"])
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
    wl = synth.WORKLOADS[args.cfg or 2]
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
    scale_modes = ((0, "none"), (1, "awe (Eq. 10: channel ranges)"), (2, "abs-max (the definition Sec. 1 says AWE replaces)"))
    for mode, bits in (("w8a8", 8), ("w4 g128, fp16 activations", 4), ("w3 g128, fp16 activations", 3)):
        for awe, awe_name in scale_modes:
            for bc in (0, 1):
                if bits == 8:
                    buf = pipeline.LayerBuffers(T, K, N, torch.float16, want_out_i32=False, want_out_deq=True, device=dev)
                    t = pipeline.calibrate_layer(X, W, b, buf, enable_awe=awe, enable_bc=bool(bc))
                    yq = t["out_deq"].to(torch.float64)
                    if b is not None:
                        yq -= b.to(torch.float64)
                    yq += t["bias_out"].to(torch.float64)
                else:
                    buf = pipeline.LayerBuffers(T, K, N, torch.float16, bits=bits, group=128, w8a8=False, device=dev)
                    t = pipeline.calibrate_layer(X, W, b, buf, enable_awe=awe, enable_bc=bool(bc))
                    # the deployed layer sees the equalised activation: X diag(s)^-1 in binary16
                    Xh = (X.to(torch.float32) * t["inv_s"]).to(torch.float16)
                    yh = torch.empty((T, N), dtype=torch.float32, device=dev)
                    ws = torch.empty(B.aweq_workspace_size(B.OP_WONLY_GEMM, T, K, N), dtype=torch.uint8, device=dev)
                    B.aweq_wonly_gemm(Xh, T, K, K, t["codes"], bits, 128, t["step_w"], t["zero_w"], N, t["bias_out"], yh,
                                      B.AWEQ_F32, N, ws)
                    yq = yh.to(torch.float64)
                e = yq - y
                rows.append({"mode": mode, "scale": awe_name, "bc": bc, "rel_rms_error": float(e.pow(2).mean().sqrt()) / rms_y,
                             "max_abs_channel_mean_error": float(e.mean(dim=0).abs().max()),
                             "status_bits": int(t["status"].item())})
                del buf, t, yq, e
    return {"ablation": rows, "layer": f"cfg{wl.cfg} {lin.name} {N}x{K}", "T": T, "rms_of_reference_output": rms_y}


def copy_probe(torch, dev, nbytes):
    """A plain copy kernel of known size: what FETCH_SIZE / WRITE_SIZE read for it gives the factor that
    turns those counters into bytes."""
    src = torch.empty(nbytes, dtype=torch.uint8, device=dev).fill_(1)
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
    return {"copy_probe_bytes": nbytes, "ms": ms, "GBs_read_plus_write": 2 * nbytes / ms / 1e6}


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
    mods = (torch, B, pipeline, synth, dev)
    if args.mfma_probe:
        print(json.dumps(mfma_probe(torch, dev)))
        return
    if args.stream_probe:
        print(json.dumps(stream_probe(torch, dev)))
        return
    if args.ablation:
        print(json.dumps(ablation(args, *mods)))
        return
    if args.fused_chain:
        print(json.dumps(fused_chain(args, *mods)))
        return
    if args.copy_probe:
        print(json.dumps(copy_probe(torch, dev, args.copy_probe)))
        return
    if args.weight_only:
        print(json.dumps(weight_only_bench(args, *mods, args.weight_only)))
        return
    if args.block:
        print(json.dumps(block_bench(args, *mods, args.cfg or 3)))
        return
    cfg = args.cfg or DEFAULT_CFG
    wl = synth.WORKLOADS[cfg]
    cpu = None
    if not args.no_cpu_baseline:
        # the oracle leg needs one layer's inputs on the host; they are the bits the GPU run uses
        lin0 = wl.linears[0]
        T = args.tokens or wl.T
        seed = synth.layer_seed(wl.cfg, 0)
        X0 = synth.make_act_torch(seed, T, lin0.K, wl, dev)
        W0 = synth.make_weight_torch(seed, lin0.N, lin0.K, wl.dtype, dev)
        b0 = synth.make_bias_np(seed, lin0.N, wl.has_bias)
        host = (lin0, X0.cpu(), W0.cpu(), None if b0 is None else torch.from_numpy(b0))
        del X0, W0
    out = layer_bench(args, *mods, cfg)
    torch.cuda.empty_cache()
    if not args.cfg and not args.layers and not args.out_deq:
        # the spec block and the weight-only workload ride along in the default line
        nb = block_bench(args, *mods, 3)
        torch.cuda.empty_cache()
        out["north_star_block"] = {k: nb[k] for k in ("config", "value", "unit", "ms_per_step", "gemm_tops", "roofline",
                                                      "calib_tokens_per_s_per_layer_excl_w8a8", "stage_ms_per_step",
                                                      "stats_x_GBs", "quant_act_GBs", "status_bits")}
        wo = {}
        for bits in (4, 3):
            r = weight_only_bench(args, *mods, bits)
            torch.cuda.empty_cache()
            wo[f"w{bits}"] = {"config": r["config"], "value": r["value"], "unit": r["unit"], "ms_per_step": r["ms_per_step"],
                              "calib_tokens_per_s_per_layer_excl_forward": r["calib_tokens_per_s_per_layer_excl_forward"],
                              "forward_tflops": r["forward_tflops"], "roofline": r["roofline"],
                              "roofline_stats": r["roofline_stats"], "status_bits": r["status_bits"]}
        out["weight_only"] = wo
    if not args.no_cpu_baseline:
        lin0, Xh, Wh, bh = host
        out["cpu_baseline"] = cpu_baseline(wl, lin0, Xh, Wh, bh)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
