"""Seeded synthetic inputs for the AWEQ calibration path.

Stand-ins for the paper's workloads (real LLaMA / OPT linear layers and their
calibration activations, Sec. 4.3), which are not available: only the layer shapes,
the storage type (FP16, Sec. 2) and the outlier-channel structure of activations
(Sec. 2, "Quantization Difficulty"; Fig. 1) are reproduced.

This module holds no arithmetic of the method: it only draws random tensors.  Both the
GPU tests/benchmark and the CPU oracle are fed from here, so both see the same bits.
"""
from dataclasses import dataclass
from typing import List, Optional, Tuple

import numpy as np

T_FULL = 262144  # 128 sequences x 2048 tokens


@dataclass(frozen=True)
class Linear:
    name: str
    N: int  # output channels
    K: int  # input channels


@dataclass(frozen=True)
class Workload:
    cfg: int
    name: str
    dtype: str  # "f32" | "f16"
    T: int
    linears: Tuple[Linear, ...]
    dist: str  # "normal" | "student_t3"
    outlier_frac: float  # fraction of K (0 -> use outlier_count)
    outlier_count: int
    outlier_lo: float
    outlier_hi: float
    has_bias: bool
    quant: str  # "w8a8" | "w4" | "w3"


def _lin(*items):
    return tuple(Linear(n, N, K) for n, N, K in items)


WORKLOADS = {
    1: Workload(1, "single-512", "f32", 2048, _lin(("fc", 512, 512)), "normal", 0.0, 4, 50.0, 50.0,
                False, "w8a8"),
    2: Workload(2, "opt-6.7b-block", "f16", T_FULL,
                _lin(("q_proj", 4096, 4096), ("k_proj", 4096, 4096), ("v_proj", 4096, 4096),
                     ("out_proj", 4096, 4096), ("fc1", 16384, 4096), ("fc2", 4096, 16384)),
                "normal", 0.001, 0, 20.0, 100.0, True, "w8a8"),
    3: Workload(3, "llama-7b-block", "f16", T_FULL,
                _lin(("q_proj", 4096, 4096), ("k_proj", 4096, 4096), ("v_proj", 4096, 4096),
                     ("o_proj", 4096, 4096), ("gate_proj", 11008, 4096), ("up_proj", 11008, 4096),
                     ("down_proj", 4096, 11008)),
                "student_t3", 0.001, 0, 50.0, 50.0, False, "w8a8"),
    4: Workload(4, "llama-7b-block-w4w3", "f16", T_FULL,
                _lin(("q_proj", 4096, 4096), ("k_proj", 4096, 4096), ("v_proj", 4096, 4096),
                     ("o_proj", 4096, 4096), ("gate_proj", 11008, 4096), ("up_proj", 11008, 4096),
                     ("down_proj", 4096, 11008)),
                "student_t3", 0.001, 0, 50.0, 50.0, False, "w4"),
    5: Workload(5, "llama-65b-block", "f16", T_FULL,
                _lin(("q_proj", 8192, 8192), ("k_proj", 8192, 8192), ("v_proj", 8192, 8192),
                     ("o_proj", 8192, 8192), ("gate_proj", 22016, 8192), ("up_proj", 22016, 8192),
                     ("down_proj", 8192, 22016)),
                "normal", 0.001, 0, 100.0, 100.0, False, "w8a8"),
}


def layer_seed(cfg: int, layer_index: int) -> int:
    return 1000 * cfg + layer_index


def n_outliers(wl: Workload, K: int) -> int:
    return wl.outlier_count if wl.outlier_frac == 0.0 else max(1, int(round(wl.outlier_frac * K)))


def outlier_channels(wl: Workload, K: int, seed: int):
    """Channel indices and per-channel factors; fixed for all tokens of a layer."""
    rng = np.random.default_rng(seed + 7919)
    n = n_outliers(wl, K)
    idx = np.sort(rng.choice(K, size=n, replace=False))
    fac = rng.uniform(wl.outlier_lo, wl.outlier_hi, size=n) if wl.outlier_hi > wl.outlier_lo \
        else np.full(n, wl.outlier_lo)
    return idx.astype(np.int64), fac.astype(np.float32)


FP16_CLAMP = 60000.0


def np_dtype(dtype: str):
    return np.float16 if dtype == "f16" else np.float32


def make_weight_np(seed: int, N: int, K: int, dtype: str, std: float = 0.02) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((N, K), dtype=np.float32) * np.float32(std)).astype(np_dtype(dtype))


def make_bias_np(seed: int, N: int, has_bias: bool, std: float = 0.02) -> Optional[np.ndarray]:
    if not has_bias:
        return None
    rng = np.random.default_rng(seed + 31337)
    return (rng.standard_normal(N, dtype=np.float32) * np.float32(std)).astype(np.float32)


def make_act_np(seed: int, T: int, K: int, wl: Workload) -> np.ndarray:
    """Calibration activations on the host (small / test sizes)."""
    rng = np.random.default_rng(seed + 104729)
    x = rng.standard_normal((T, K), dtype=np.float32)
    if wl.dist == "student_t3":
        chi = rng.chisquare(3.0, size=(T, K)).astype(np.float32)
        x = x / np.sqrt(chi / np.float32(3.0))
    idx, fac = outlier_channels(wl, K, seed)
    x[:, idx] *= fac[None, :]
    if wl.dtype == "f16":
        np.clip(x, -FP16_CLAMP, FP16_CLAMP, out=x)
    return x.astype(np_dtype(wl.dtype))


def make_act_torch(seed: int, T: int, K: int, wl: Workload, device, chunk_rows: int = 16384):
    """Calibration activations generated on the device in row chunks (full sizes).

    The bits depend on torch's generator; parity checks copy the rows they need back to
    the host, so they never rely on regenerating them."""
    import torch
    tdt = torch.float16 if wl.dtype == "f16" else torch.float32
    g = torch.Generator(device=device)
    g.manual_seed(seed + 104729)
    out = torch.empty((T, K), dtype=tdt, device=device)
    idx, fac = outlier_channels(wl, K, seed)
    idx_t = torch.from_numpy(idx).to(device)
    fac_t = torch.from_numpy(fac).to(device)
    for r0 in range(0, T, chunk_rows):
        r1 = min(T, r0 + chunk_rows)
        x = torch.randn((r1 - r0, K), generator=g, device=device, dtype=torch.float32)
        if wl.dist == "student_t3":
            chi = torch.zeros_like(x)
            for _ in range(3):
                z = torch.randn((r1 - r0, K), generator=g, device=device, dtype=torch.float32)
                chi += z * z
            x = x / torch.sqrt(chi / 3.0)
        x[:, idx_t] *= fac_t[None, :]
        if wl.dtype == "f16":
            x.clamp_(-FP16_CLAMP, FP16_CLAMP)
        out[r0:r1] = x.to(tdt)
    return out


def make_weight_torch(seed: int, N: int, K: int, dtype: str, device, std: float = 0.02):
    import torch
    tdt = torch.float16 if dtype == "f16" else torch.float32
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    w = torch.randn((N, K), generator=g, device=device, dtype=torch.float32) * std
    return w.to(tdt)


def scaled(wl: Workload, T: int, linears: List[Linear]) -> Workload:
    """Same recipe at a reduced size (parity tests)."""
    return Workload(wl.cfg, wl.name + "-small", wl.dtype, T, tuple(linears), wl.dist, wl.outlier_frac,
                    wl.outlier_count, wl.outlier_lo, wl.outlier_hi, wl.has_bias, wl.quant)
