"""The W8A8 GEMM with fused epilogues (aweq_w8a8_gemm_fused): the column statistics of its binary16
output and that output's int8 codes for the next layer, produced where the output is.

Chain of evidence: (1) the fused entry point's stored output equals aweq_w8a8_gemm's de-quantised
binary16 output bit for bit (that one is checked against the oracle elsewhere, and here again
within one rounding); (2) its statistics equal the oracle's column statistics of that stored output
exactly (extremes and, at these sizes, the fp64 sums: sums of binary16 values are exact in fp64
below 2^13 rows); (3) its codes, row sums and column sums equal the oracle's activation quantizer
applied to that stored output, bit for bit.
"""
import numpy as np
import pytest
from conftest import from_panels, to_panels

torch = pytest.importorskip("torch")

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2311_01305_amd import binding
    binding.load_library()
    return binding


def progress(msg):
    print(f"[gpu-fused] {msg}", flush=True)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def e(*shape, dtype):
    return torch.empty(shape, dtype=dtype, device=DEV)


def make_case(orc, seed, T, K, N, with_bias=True):
    """A quantised layer from the oracle: codes of X_hat and W_hat and every constant of the epilogue."""
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((T, K)).astype(np.float32)
    X[:, 3 % K] *= 30.0
    X = X.astype(np.float16)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    sx, sw = orc.col_stats(X), orc.col_stats(W, want_sum=False)
    r_x, _, _ = orc.ranges(sx["cmin"], sx["cmax"])
    r_w, _, _ = orc.ranges(sw["cmin"], sw["cmax"])
    s, inv_s, _ = orc.scales(r_x, r_w)
    lo, hi, _ = orc.xhat_stats(sx["cmin"], sx["cmax"], sx["csum"], sx["count"], inv_s)
    step_x, zero_x, _ = orc.qparams(lo, hi, 8)
    a = orc.quant_act(X, inv_s, step_x, zero_x)
    q = orc.quant_weight(orc.fold_weight(W, s), 8, 0)
    bias = (rng.standard_normal(N) * 0.5).astype(np.float32) if with_bias else None
    return dict(T=T, K=K, N=N, xq=a["xq"], rowsum_x=a["rowsum_x"], wq=orc.pack_codes(q["codes_u"], 8), step_x=step_x,
                zero_x=zero_x, step_w=q["step"], zero_w=q["zero"], rowsum_w=q["rowsum_w"], bias=bias, rng=rng)


class Dev:
    def __init__(self, B, c):
        self.xq, self.wq = dev(to_panels(c["xq"])), dev(to_panels(c["wq"]))
        self.step_x, self.zero_x = dev(np.array([c["step_x"]], np.float32)), dev(np.array([c["zero_x"]], np.int32))
        self.step_w, self.zero_w = dev(c["step_w"]), dev(c["zero_w"])
        self.rowsum_x, self.rowsum_w = dev(c["rowsum_x"]), dev(c["rowsum_w"])
        self.bias = dev(c["bias"]) if c["bias"] is not None else None


def unfused(B, c, d):
    T, K, N = c["T"], c["K"], c["N"]
    y = torch.zeros((T, N), dtype=torch.float16, device=DEV)
    cs = e(N, dtype=torch.int64)
    B.aweq_w8a8_gemm(d.xq, B.AWEQ_I8, T, K, K, None, d.step_x, d.zero_x, None, d.rowsum_x, None, d.wq, N, d.step_w, d.zero_w, 0,
                     d.rowsum_w, d.bias, None, y, B.AWEQ_F16, N, cs, None, None)
    return host(y), host(cs)


def fused(B, c, d, act=0, store=True, stats=True, nxt=None, accumulate=0, prev=None):
    T, K, N = c["T"], c["K"], c["N"]
    o = {}
    o["y"] = torch.full((T, N), 7.0, dtype=torch.float16, device=DEV) if store else None
    o["colsum_acc"] = e(N, dtype=torch.int64)
    if stats:
        o["cmin"], o["cmax"] = e(N, dtype=torch.float32), e(N, dtype=torch.float32)
        o["csum"], o["count"] = e(N, dtype=torch.float64), torch.zeros(1, dtype=torch.int64, device=DEV)
        if prev is not None:
            for k in ("cmin", "cmax", "csum", "count"):
                o[k].copy_(prev[k])
    if nxt is not None:
        o["yq"] = torch.full((B.aweq_panel_bytes(T, N),), 0x5a, dtype=torch.int8, device=DEV)
        o["rowsum_y"], o["colsum_yq"] = e(T, dtype=torch.int32), e(N, dtype=torch.int64)
    ws = e(B.aweq_workspace_size(B.OP_W8A8_GEMM, T, K, N), dtype=torch.uint8)
    o["status"] = torch.zeros(1, dtype=torch.int32, device=DEV)
    B.aweq_w8a8_gemm_fused(d.xq, T, K, d.wq, N, d.step_x, d.zero_x, d.step_w, d.zero_w, d.rowsum_x, d.rowsum_w, d.bias, act,
                           o["y"], N, o["colsum_acc"], o.get("cmin"), o.get("cmax"), o.get("csum"), o.get("count"), accumulate,
                           dev(nxt["inv_s"]) if nxt else None, dev(np.array([nxt["step"]], np.float32)) if nxt else None,
                           dev(np.array([nxt["zero"]], np.int32)) if nxt else None, o.get("yq"), o.get("rowsum_y"),
                           o.get("colsum_yq"), ws, o["status"])
    torch.cuda.synchronize()
    return o


def next_layer_params(orc, rng, y):
    """An equalization scale and the static quantizer of the layer that reads y."""
    N = y.shape[1]
    inv_s = rng.uniform(0.2, 3.0, N).astype(np.float32)
    yh = y.astype(np.float32) * inv_s[None, :]
    step, zero, _ = orc.qparams(np.float32(yh.min()), np.float32(yh.max()), 8)
    return dict(inv_s=inv_s, step=step, zero=zero)


SHAPES = [
    (256, 64, 256),      # one tile, one panel
    (300, 256, 260),     # ragged T; N % 64 = 4: the last panel of the codes is mostly zero fill
    (515, 384, 1028),    # six panels, several tiles, ragged both ways
    (1000, 4096, 512),   # the K of the attention linears
    (8200, 128, 2308),   # 33 x 10 = 330 tiles on 256 persistent workgroups: second tiles, edges on both sides
]


@pytest.mark.parametrize("T,K,N", SHAPES)
@pytest.mark.parametrize("act", [0, 1])
def test_fused_epilogues_match_separate_passes(B, orc, T, K, N, act):
    progress(f"T={T} K={K} N={N} act={act}")
    c = make_case(orc, T + K + N, T, K, N)
    d = Dev(B, c)
    y_ref, cs_ref = unfused(B, c, d)
    assert np.isfinite(y_ref.astype(np.float32)).all()
    # (0) the separate path's output is the oracle's within one rounding of binary16
    direct = orc.w8a8_output_direct(c["xq"], c["wq"], c["step_x"], c["zero_x"], c["step_w"], c["zero_w"], c["bias"])
    assert np.all(np.abs(y_ref.astype(np.float64) - direct) <= 2.0 ** -10 * np.abs(direct) + 2.0 ** -24)
    if act == 1:
        y_ref = np.maximum(y_ref, np.float16(0))
    nxt = next_layer_params(orc, c["rng"], y_ref)
    f = fused(B, c, d, act=act, store=True, stats=True, nxt=nxt)
    # (1) the stored output
    assert np.array_equal(host(f["y"]).astype(np.float32), y_ref.astype(np.float32))
    assert np.array_equal(host(f["colsum_acc"]), cs_ref)
    # (2) statistics of the stored output: the oracle's column pass over it
    st = orc.col_stats(y_ref)
    assert np.array_equal(host(f["cmin"]), st["cmin"]) and np.array_equal(host(f["cmax"]), st["cmax"])
    assert np.array_equal(host(f["csum"]), st["csum"])
    assert int(host(f["count"])[0]) == T
    # library special case of the same: numpy reductions
    assert np.array_equal(host(f["cmax"]), y_ref.max(axis=0).astype(np.float32))
    # (3) the next layer's codes: the oracle's activation quantizer over the stored output
    a = orc.quant_act(y_ref, nxt["inv_s"], nxt["step"], nxt["zero"])
    assert np.array_equal(from_panels(host(f["yq"]), T, N), a["xq"])
    assert np.array_equal(host(f["rowsum_y"]), a["rowsum_x"])
    assert np.array_equal(host(f["colsum_yq"]), a["colsum_xq"])
    assert int(host(f["status"])[0]) == a["status"] == 0
    assert a["xq"].min() == -128 and a["xq"].max() == 127
    # the variants that do not store y, and each epilogue alone, give the same
    g = fused(B, c, d, act=act, store=False, stats=True, nxt=nxt)
    for k in ("cmin", "cmax", "csum", "yq", "rowsum_y", "colsum_yq", "colsum_acc"):
        assert torch.equal(g[k], f[k]), k
    g = fused(B, c, d, act=act, store=False, stats=True, nxt=None)
    assert torch.equal(g["cmin"], f["cmin"]) and torch.equal(g["cmax"], f["cmax"]) and torch.equal(g["csum"], f["csum"])
    g = fused(B, c, d, act=act, store=True, stats=False, nxt=nxt)
    assert torch.equal(g["yq"], f["yq"]) and torch.equal(g["rowsum_y"], f["rowsum_y"]) and torch.equal(g["y"], f["y"])


def test_fused_statistics_accumulate_over_batches(B, orc):
    """accumulate = 1 merges a second calibration batch the way aweq_calib_stats does."""
    progress("two batches")
    c1, c2 = make_case(orc, 1, 300, 128, 260), make_case(orc, 2, 200, 128, 260)
    for k in ("wq", "step_w", "zero_w", "rowsum_w", "bias"):      # the same layer, a second batch of tokens
        c2[k] = c1[k]
    d1, d2 = Dev(B, c1), Dev(B, c2)
    y1, _ = unfused(B, c1, d1)
    y2, _ = unfused(B, c2, d2)
    f1 = fused(B, c1, d1)
    f2 = fused(B, c2, d2, accumulate=1, prev=f1)
    st = orc.col_stats(y2, prev=orc.col_stats(y1))
    assert np.array_equal(host(f2["cmin"]), st["cmin"]) and np.array_equal(host(f2["cmax"]), st["cmax"])
    assert np.array_equal(host(f2["csum"]), st["csum"]) and int(host(f2["count"])[0]) == 500 == st["count"]


def test_fused_output_feeds_the_next_layers_calibration(B, orc):
    """What the epilogue statistics are for: aweq_equalize on them gives the scales the separate
    statistics pass over the stored output gives."""
    progress("statistics -> equalize")
    c = make_case(orc, 11, 700, 256, 512)
    d = Dev(B, c)
    f = fused(B, c, d, act=1)
    y = host(f["y"])
    T, N = y.shape
    cmin, cmax, csum = e(N, dtype=torch.float32), e(N, dtype=torch.float32), e(N, dtype=torch.float64)
    cnt = torch.zeros(1, dtype=torch.int64, device=DEV)
    r, R, p = e(N, dtype=torch.float32), e(1, dtype=torch.float32), e(N, dtype=torch.float32)
    ws = e(B.aweq_workspace_size(B.OP_CALIB_STATS, T, N), dtype=torch.uint8)
    B.aweq_calib_stats(f["y"], B.AWEQ_F16, T, N, N, cmin, cmax, csum, cnt, 0, 1, r, R, p, ws)
    assert torch.equal(cmin, f["cmin"]) and torch.equal(cmax, f["cmax"])
    mean_abs = np.abs(y.astype(np.float64)).mean(axis=0)
    assert np.all(np.abs(host(csum) - host(f["csum"])) / T <= 1e-6 * mean_abs + 1e-12)


def test_fused_fullsize(B, orc):
    """T = 262144 tokens, 4096 x 4096 (the launch configuration of the benchmark's attention linears):
    statistics and codes of the whole output against the oracle's passes over the stored output."""
    T, K, N = 262144, 4096, 4096
    progress(f"full size T={T} K={K} N={N}")
    g = torch.Generator(device=DEV)
    g.manual_seed(5)
    xq_rm = torch.clamp(torch.round(torch.randn((T, K), generator=g, device=DEV) * 3.0), -128, 127).to(torch.int8)
    xq_rm[:, 7] = torch.randint(-128, 128, (T,), generator=g, device=DEV, dtype=torch.int32).to(torch.int8)
    wq_rm = torch.clamp(torch.round(torch.randn((N, K), generator=g, device=DEV) * 40.0), -128, 127).to(torch.int8)
    xq, wq = e(B.aweq_panel_bytes(T, K), dtype=torch.int8), e(B.aweq_panel_bytes(N, K), dtype=torch.int8)
    B.aweq_pack_panels_i8(xq_rm, T, K, K, xq)
    B.aweq_pack_panels_i8(wq_rm, N, K, K, wq)

    class D:
        pass
    d = D()
    d.xq, d.wq = xq, wq
    d.rowsum_x = xq_rm.sum(dim=1, dtype=torch.int32)
    d.rowsum_w = wq_rm.sum(dim=1, dtype=torch.int32)
    rng = np.random.default_rng(6)
    c = dict(T=T, K=K, N=N)
    d.step_x, d.zero_x = dev(np.array([0.021], np.float32)), dev(np.array([131], np.int32))
    d.step_w, d.zero_w = dev(rng.uniform(5e-4, 2e-3, N).astype(np.float32)), dev(rng.integers(100, 156, N).astype(np.int32))
    d.bias = dev((rng.standard_normal(N) * 0.5).astype(np.float32))
    del xq_rm, wq_rm
    y_ref, cs_ref = unfused(B, c, d)
    assert np.isfinite(y_ref.astype(np.float32)).all()
    y_ref = np.maximum(y_ref, np.float16(0))
    inv_s = rng.uniform(0.2, 3.0, N).astype(np.float32)
    hi = np.float32((y_ref[::16].astype(np.float32) * inv_s[None, :]).max())
    step, zero, _ = orc.qparams(np.float32(0.0), hi, 8)
    nxt = dict(inv_s=inv_s, step=step, zero=zero)
    progress("fused launch")
    f = fused(B, c, d, act=1, store=True, stats=True, nxt=nxt)
    assert np.array_equal(host(f["y"]).astype(np.float32), y_ref.astype(np.float32))
    assert np.array_equal(host(f["colsum_acc"]), cs_ref)
    progress("oracle statistics over the stored output (host)")
    st = orc.col_stats(y_ref)
    assert np.array_equal(host(f["cmin"]), st["cmin"]) and np.array_equal(host(f["cmax"]), st["cmax"])
    # the epilogue's sums are exact; the oracle's fp64 running sums round: |error| <= T 2^-53 sum|y|
    abs_sum = np.abs(y_ref[::8].astype(np.float64)).sum(axis=0) * 8.5
    assert np.all(np.abs(host(f["csum"]) - st["csum"]) <= T * 2.0 ** -53 * abs_sum + 1e-9)
    progress("oracle activation quantizer over the stored output (host)")
    a = orc.quant_act(y_ref, nxt["inv_s"], nxt["step"], nxt["zero"])
    assert np.array_equal(host(f["rowsum_y"]), a["rowsum_x"]) and np.array_equal(host(f["colsum_yq"]), a["colsum_xq"])
    rows = np.unique(np.concatenate([np.arange(300), np.arange(T - 300, T), rng.integers(0, T, 300)])).astype(np.int64)
    idx = torch.from_numpy(rows).to(DEV)
    got = f["yq"].view(N // 64, T, 64)[:, idx, :].permute(1, 0, 2).reshape(-1, N)
    assert np.array_equal(host(got), a["xq"][rows])
    assert int(host(f["status"])[0]) == a["status"]
