"""Convenience driver: allocate the buffers of one linear layer with torch and call the
five C-ABI stages in the order the method applies them (Sec. 3: statistics, equalization,
quantization, W8A8 forward, bias correction).  No arithmetic of the method happens here.
"""
from dataclasses import dataclass, field
from typing import Optional

import torch

from . import binding as B


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float16:
        return B.AWEQ_F16
    if t.dtype == torch.float32:
        return B.AWEQ_F32
    if t.dtype == torch.int8:
        return B.AWEQ_I8
    raise TypeError(f"unsupported dtype {t.dtype}")


@dataclass
class LayerBuffers:
    """Every device buffer one layer's calibration touches (allocated once, reused per step)."""
    T: int
    K: int
    N: int
    dtype: torch.dtype
    bits: int = 8
    group: int = 0
    w8a8: bool = True
    want_out_i32: bool = True
    want_out_deq: bool = False
    device: str = "cuda:0"
    t: dict = field(default_factory=dict)

    def __post_init__(self):
        d, T, K, N = self.device, self.T, self.K, self.N
        f32, i32, i64, f64 = torch.float32, torch.int32, torch.int64, torch.float64
        e = lambda *shape, dtype: torch.empty(shape, dtype=dtype, device=d)
        t = self.t
        for name in ("xmin", "xmax", "wmin", "wmax", "r_x", "p_x", "r_w", "p_w", "s", "inv_s", "mu_xhat"):
            t[name] = e(K, dtype=f32)
        t["xsum"] = e(K, dtype=f64)
        t["count"] = e(1, dtype=i64)
        t["wcount"] = e(1, dtype=i64)
        t["R_x"], t["R_w"] = e(1, dtype=f32), e(1, dtype=f32)
        t["xhat_range"] = e(2, dtype=f32)
        t["act_step"], t["act_zero"] = e(1, dtype=f32), e(1, dtype=i32)
        t["status"] = torch.zeros(1, dtype=i32, device=d)
        t["W_hat"] = e(N, K, dtype=self.dtype)
        ng = 1 if self.group < 0 else (N if self.group == 0 else N * (K // self.group))
        # 8-bit per-row / per-tensor codes are the GEMM operand: K-panel layout
        panel_w = self.bits == 8 and self.group <= 0
        t["codes"] = e(B.aweq_panel_bytes(N, K) if panel_w else N * K * self.bits // 8, dtype=torch.int8)
        t["step_w"], t["zero_w"] = e(ng, dtype=f32), e(ng, dtype=i32)
        t["rowsum_w"] = e(N, dtype=i32)
        t["delta"], t["bias_out"] = e(N, dtype=f32), e(N, dtype=f32)
        ws = max(B.aweq_workspace_size(B.OP_CALIB_STATS, T, K, N), B.aweq_workspace_size(B.OP_CALIB_STATS, N, K, N),
                 B.aweq_workspace_size(B.OP_QUANT_WEIGHT, N, K, N),
                 B.aweq_workspace_size(B.OP_W8A8_GEMM, T, K, N) if self.w8a8 else 0, 16)
        t["ws"] = e(ws, dtype=torch.uint8)
        if self.w8a8:
            t["xq"] = e(B.aweq_panel_bytes(T, K), dtype=torch.int8)
            t["rowsum_x"] = e(T, dtype=i32)
            t["colsum_xq"] = e(K, dtype=i64)
            t["colsum_acc"] = e(N, dtype=i64)
            if self.want_out_i32:
                t["out_i32"] = e(T, N, dtype=i32)
            if self.want_out_deq:
                t["out_deq"] = e(T, N, dtype=self.dtype)


def calibrate_layer(X: torch.Tensor, W: torch.Tensor, bias: Optional[torch.Tensor], buf: LayerBuffers,
                    enable_awe: bool = True, enable_bc: bool = True, stream=None, fused_weight_pass: bool = False,
                    forward: bool = True):
    """One pass of the whole hot path for one linear layer.  Everything is enqueued on the
    current (or given) stream; nothing synchronises.  forward = False (W8A8) calibrates without
    running the int8 GEMM: the activation quantizer only forms its sums and the bias correction
    takes the accumulator's sums over tokens from the weight codes (the same integers)."""
    t = buf.t
    T, K, N = buf.T, buf.K, buf.N
    dt = _dt(X)
    st = t["status"]
    # stage 1: statistics of X and of W
    B.aweq_calib_stats(X, dt, T, K, X.stride(0), t["xmin"], t["xmax"], t["xsum"], t["count"], 0, 1,
                       t["r_x"], t["R_x"], t["p_x"], t["ws"], st, stream)
    B.aweq_calib_stats(W, dt, N, K, W.stride(0), t["wmin"], t["wmax"], None, t["wcount"], 0, 1,
                       t["r_w"], t["R_w"], t["p_w"], t["ws"], st, stream)
    fused = fused_weight_pass and buf.group == 0
    ldw, ldwh = W.stride(0), t["W_hat"].stride(0)   # W may be a pitched view (a row slice of a fused qkv weight)
    # stage 2: equalization scales, fold into W, equalised activation range / mean / quantizer
    B.aweq_equalize(t["xmin"], t["xmax"], t["xsum"], T, t["wmin"], t["wmax"], K, enable_awe, t["s"], t["inv_s"],
                    None if fused else W, t["W_hat"], dt, N, ldw, ldwh, None, t["xhat_range"], t["mu_xhat"],
                    t["act_step"], t["act_zero"], st, stream)
    # stage 3: weight quantizer (fused: fold and quantise in one pass over W)
    if fused:
        B.aweq_fold_quant_weight(W, dt, N, K, ldw, t["s"], t["W_hat"], ldwh, buf.bits, t["codes"], t["step_w"], t["zero_w"],
                                 t["rowsum_w"] if buf.bits == 8 else None, st, stream)
    else:
        B.aweq_quant_weight(t["W_hat"], dt, N, K, ldwh, buf.bits, buf.group, t["codes"], t["step_w"], t["zero_w"],
                            t["rowsum_w"] if (buf.bits == 8 and buf.group <= 0) else None, t["ws"], st, stream)
    wg = -1 if buf.group < 0 else 0   # per-tensor weights (Sec. 3): one (Step, Z), read as such by stages 4 and 5
    if buf.w8a8 and not forward:
        B.aweq_quant_act(X, dt, T, K, X.stride(0), t["inv_s"], t["act_step"], t["act_zero"], None, None, t["colsum_xq"],
                         t["ws"], st, stream)
        B.aweq_bias_correct(B.BIAS_W8A8, t["W_hat"], dt, N, K, ldwh, t["mu_xhat"], T, None, t["colsum_xq"], t["rowsum_w"],
                            t["act_step"], t["act_zero"], t["codes"], 8, wg, t["step_w"], t["zero_w"], bias, t["delta"],
                            t["bias_out"], enable_bc, st, stream)
    elif buf.w8a8:
        # stage 4: activation quantizer + int8 GEMM (+ per-channel output sums for stage 5)
        B.aweq_w8a8_gemm(X, dt, T, K, X.stride(0), t["inv_s"], t["act_step"], t["act_zero"], t["xq"], t["rowsum_x"],
                         t["colsum_xq"], t["codes"], N, t["step_w"], t["zero_w"], wg, t["rowsum_w"], bias,
                         t.get("out_i32"), t.get("out_deq"), dt, N, t["colsum_acc"], t["ws"], st, stream)
        # stage 5: bias correction
        B.aweq_bias_correct(B.BIAS_W8A8, t["W_hat"], dt, N, K, ldwh, t["mu_xhat"], T, t["colsum_acc"], t["colsum_xq"],
                            t["rowsum_w"], t["act_step"], t["act_zero"], None, 8, wg, t["step_w"], t["zero_w"], bias,
                            t["delta"], t["bias_out"], enable_bc, st, stream)
    else:
        B.aweq_bias_correct(B.BIAS_WEIGHT_ONLY, t["W_hat"], dt, N, K, ldwh, t["mu_xhat"], T, None, None, None, None, None,
                            t["codes"], buf.bits, buf.group, t["step_w"], t["zero_w"], bias, t["delta"],
                            t["bias_out"], enable_bc, st, stream)
    return t


@dataclass
class GroupBuffers:
    """Buffers of a group of linears that read the same activation (q/k/v, gate/up): one
    statistics pass, one equalization scale (from the merged weight ranges), one activation
    quantization; per linear its folded weight, codes, GEMM output sums and bias."""
    T: int
    K: int
    Ns: tuple
    dtype: torch.dtype
    want_out_i32: bool = False
    want_out_deq: bool = False
    device: str = "cuda:0"
    t: dict = field(default_factory=dict)
    per: list = field(default_factory=list)

    def __post_init__(self):
        d, T, K = self.device, self.T, self.K
        f32, i32, i64, f64 = torch.float32, torch.int32, torch.int64, torch.float64
        e = lambda *shape, dtype: torch.empty(shape, dtype=dtype, device=d)
        t = self.t
        for name in ("xmin", "xmax", "wmin", "wmax", "r_x", "p_x", "r_w", "p_w", "s", "inv_s", "mu_xhat"):
            t[name] = e(K, dtype=f32)
        t["xsum"] = e(K, dtype=f64)
        t["count"], t["wcount"] = e(1, dtype=i64), e(1, dtype=i64)
        t["R_x"], t["R_w"] = e(1, dtype=f32), e(1, dtype=f32)
        t["xhat_range"] = e(2, dtype=f32)
        t["act_step"], t["act_zero"] = e(1, dtype=f32), e(1, dtype=i32)
        t["status"] = torch.zeros(1, dtype=i32, device=d)
        t["xq"] = e(B.aweq_panel_bytes(T, K), dtype=torch.int8)
        t["rowsum_x"] = e(T, dtype=i32)
        t["colsum_xq"] = e(K, dtype=i64)
        ws = max([B.aweq_workspace_size(B.OP_CALIB_STATS, T, K, 0), B.aweq_workspace_size(B.OP_QUANT_ACT, T, K, 0)] +
                 [B.aweq_workspace_size(B.OP_CALIB_STATS, N, K, N) for N in self.Ns] + [16])
        t["ws"] = e(ws, dtype=torch.uint8)
        for N in self.Ns:
            p = {"W_hat": e(N, K, dtype=self.dtype), "codes": e(B.aweq_panel_bytes(N, K), dtype=torch.int8), "step_w": e(N, dtype=f32),
                 "zero_w": e(N, dtype=i32), "rowsum_w": e(N, dtype=i32), "colsum_acc": e(N, dtype=i64),
                 "delta": e(N, dtype=f32), "bias_out": e(N, dtype=f32)}
            if self.want_out_i32:
                p["out_i32"] = e(T, N, dtype=i32)
            if self.want_out_deq:
                p["out_deq"] = e(T, N, dtype=self.dtype)
            self.per.append(p)


def calibrate_group(X: torch.Tensor, Ws, biases, gb: GroupBuffers, enable_awe: bool = True, enable_bc: bool = True,
                    stream=None):
    """W8A8 calibration of linears sharing the input X (Sec. 3.1: equalization sits at the
    entrance of the attention block and of the MLP, so layers with a common input share s)."""
    t, T, K = gb.t, gb.T, gb.K
    dt = _dt(X)
    st = t["status"]
    B.aweq_calib_stats(X, dt, T, K, X.stride(0), t["xmin"], t["xmax"], t["xsum"], t["count"], 0, 1,
                       t["r_x"], t["R_x"], t["p_x"], t["ws"], st, stream)
    # weight ranges of the group: min of mins / max of maxes over all its weights
    for i, W in enumerate(Ws):
        last = i == len(Ws) - 1
        B.aweq_calib_stats(W, dt, W.shape[0], K, W.stride(0), t["wmin"], t["wmax"], None, t["wcount"], int(i > 0),
                           int(last), t["r_w"], t["R_w"], t["p_w"], t["ws"], st, stream)
    # the scales (and the activation quantizer) depend on the group's merged ranges only: computed once
    B.aweq_equalize(t["xmin"], t["xmax"], t["xsum"], T, t["wmin"], t["wmax"], K, enable_awe, t["s"], t["inv_s"],
                    None, None, dt, 0, K, K, None, t["xhat_range"], t["mu_xhat"], t["act_step"], t["act_zero"], st, stream)
    for W, p in zip(Ws, gb.per):
        # fold (Eq. 3) and per-channel quantizer in one pass over each weight
        B.aweq_fold_quant_weight(W, dt, W.shape[0], K, W.stride(0), t["s"], p["W_hat"], p["W_hat"].stride(0), 8, p["codes"],
                                 p["step_w"], p["zero_w"], p["rowsum_w"], st, stream)
    B.aweq_quant_act(X, dt, T, K, X.stride(0), t["inv_s"], t["act_step"], t["act_zero"], t["xq"], t["rowsum_x"],
                     t["colsum_xq"], t["ws"], st, stream)
    for W, b, p in zip(Ws, biases, gb.per):
        N = W.shape[0]
        B.aweq_w8a8_gemm(t["xq"], B.AWEQ_I8, T, K, K, None, t["act_step"], t["act_zero"], None, t["rowsum_x"], None,
                         p["codes"], N, p["step_w"], p["zero_w"], 0, p["rowsum_w"], b, p.get("out_i32"),
                         p.get("out_deq"), dt, N, p["colsum_acc"], None, st, stream)
        B.aweq_bias_correct(B.BIAS_W8A8, p["W_hat"], dt, N, K, p["W_hat"].stride(0), t["mu_xhat"], T, p["colsum_acc"],
                            t["colsum_xq"], p["rowsum_w"], t["act_step"], t["act_zero"], None, 8, 0, p["step_w"], p["zero_w"], b,
                            p["delta"], p["bias_out"], enable_bc, st, stream)
    return gb
