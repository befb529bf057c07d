"""Parity of the weight-only configuration at its full size and in the launch configuration
bench.py --weight-only times: down_proj of the LLaMA-7B-shaped block (4096 x 11008, T = 262144
heavy-tailed calibration tokens, W4 and W3 per group of 128, binary16 activations).

Statistics are checked over the full input, the weight quantizer and the weight-only bias
correction (Eq. 12-15) over the whole weight, the forward on sampled token rows the oracle
computes one by one (within the fp32-accumulation bound) plus, for every token, a random
0/1 combination of its outputs against the same combination of the oracle's weight rows.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def progress(msg):
    print(f"[gpu-fullsize-wonly] {msg}", flush=True)


def h(x):
    return x.cpu().numpy()


@pytest.fixture(scope="module")
def shared():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2311_01305_amd import binding, synth
    binding.load_library()
    cfg, li = 4, 6
    wl = synth.WORKLOADS[cfg]
    lin = wl.linears[li]
    seed = synth.layer_seed(cfg, li)
    progress(f"generating {lin.name} X[{wl.T} x {lin.K}] on the device")
    X = synth.make_act_torch(seed, wl.T, lin.K, wl, DEV)
    W = synth.make_weight_torch(seed, lin.N, lin.K, wl.dtype, DEV)
    return dict(B=binding, wl=wl, lin=lin, X=X, W=W, cache={})


@pytest.mark.parametrize("bits", [4, 3])
def test_fullsize_weight_only(shared, orc, bits):
    from paper_2311_01305_amd import pipeline
    B, wl, lin, X, W = shared["B"], shared["wl"], shared["lin"], shared["X"], shared["W"]
    T, K, N, group = wl.T, lin.K, lin.N, 128
    buf = pipeline.LayerBuffers(T, K, N, torch.float16, bits=bits, group=group, w8a8=False, device=DEV)
    progress(f"W{bits}: statistics, equalization, quantizer, bias correction")
    t = pipeline.calibrate_layer(X, W, None, buf)
    y = torch.empty((T, N), dtype=torch.float16, device=DEV)
    ws = torch.empty(B.aweq_workspace_size(B.OP_WONLY_GEMM, T, K, N), dtype=torch.uint8, device=DEV)
    progress(f"W{bits}: forward")
    B.aweq_wonly_gemm(X, T, K, K, t["codes"], bits, group, t["step_w"], t["zero_w"], N, t["bias_out"], y,
                      B.AWEQ_F16, N, ws, t["status"])
    torch.cuda.synchronize()
    assert int(h(t["status"])[0]) == 0

    # ---- statistics over the full input (once for both bit widths)
    c = shared["cache"]
    if "sx" not in c:
        progress("oracle statistics over the full X (host)")
        Xh = h(X)
        c["sx"] = orc.col_stats(Xh)
        c["sw"] = orc.col_stats(h(W), want_sum=False)
        c["mean_abs"] = np.abs(Xh[::64].astype(np.float64)).mean(axis=0)
        del Xh
    sx, sw = c["sx"], c["sw"]
    assert np.array_equal(h(t["xmin"]), sx["cmin"]) and np.array_equal(h(t["xmax"]), sx["cmax"])
    assert np.all(np.abs(h(t["xsum"]) - sx["csum"]) / T <= 1e-6 * c["mean_abs"] + 1e-12)
    assert np.array_equal(h(t["wmin"]), sw["cmin"]) and np.array_equal(h(t["wmax"]), sw["cmax"])
    r_x, _, _ = orc.ranges(sx["cmin"], sx["cmax"])
    r_w, _, _ = orc.ranges(sw["cmin"], sw["cmax"])
    s, inv_s, _ = orc.scales(r_x, r_w)
    np.testing.assert_allclose(h(t["s"]), s, rtol=1e-5)
    _, _, mu = orc.xhat_stats(sx["cmin"], sx["cmax"], sx["csum"], sx["count"], h(t["inv_s"]))
    np.testing.assert_allclose(h(t["mu_xhat"]), mu, rtol=1e-5, atol=1e-9)

    # ---- fold + quantizer over the whole weight, given the GPU's fp32 scales
    progress(f"W{bits}: oracle fold + quantizer + bias correction")
    Wh = orc.fold_weight(h(W), h(t["s"]))
    assert np.array_equal(h(t["W_hat"]).view(np.uint16), Wh.view(np.uint16))
    q = orc.quant_weight(Wh, bits, group)
    assert np.array_equal(h(t["step_w"]), q["step"].reshape(-1)) and np.array_equal(h(t["zero_w"]), q["zero"].reshape(-1))
    assert np.array_equal(h(t["codes"]).view(np.uint8), orc.pack_codes(q["codes_u"], bits).view(np.uint8).reshape(-1))
    assert q["codes_u"].min() == 0 and q["codes_u"].max() == (1 << bits) - 1
    d_ref, b_ref = orc.bias_wonly(Wh, h(t["mu_xhat"]), q["codes_u"], group, q["step"], q["zero"], None)
    assert np.max(np.abs(h(t["delta"]) - d_ref)) <= 1e-5 * np.max(np.abs(d_ref))
    np.testing.assert_allclose(h(t["bias_out"]), b_ref, rtol=1e-5, atol=1e-5 * np.max(np.abs(d_ref)))

    # ---- forward: sampled token rows one by one
    Wt = orc.dequant_weight_h(q["codes_u"], group, q["step"], q["zero"])
    rng = np.random.default_rng(2024 + bits)
    rows = np.unique(np.concatenate([np.arange(130), np.arange(T - 130, T), rng.integers(0, T, 130)])).astype(np.int64)
    idx = torch.from_numpy(rows).to(DEV)
    progress(f"W{bits}: oracle forward on {rows.size} sampled rows")
    bias = h(t["bias_out"])
    ref, mag = orc.wonly_forward(h(X[idx]), Wt, bias)
    got = h(y[idx]).astype(np.float64)
    bound = K * 2.0 ** -24 * mag + 2.0 ** -11 * np.abs(ref) + 2.0 ** -24
    assert np.all(np.abs(got - ref) <= bound), float(np.max(np.abs(got - ref) / bound))

    # ---- forward: every token, random 0/1 combinations of its outputs (fp64 on the device; each
    # output carries at most the bound above, so the combination carries at most its sum)
    progress(f"W{bits}: output combinations over all {T} tokens")
    V = rng.integers(0, 2, (N, 3)).astype(np.float64)
    U = torch.from_numpy(Wt.astype(np.float64).T @ V).to(DEV)                 # [K, 3]
    Uabs = torch.from_numpy(np.abs(Wt.astype(np.float64)).T @ V).to(DEV)
    Vd = torch.from_numpy(V).to(DEV)
    bv = torch.from_numpy(bias.astype(np.float64) @ V).to(DEV)
    worst = 0.0
    for r0 in range(0, T, 16384):
        xs = X[r0:r0 + 16384].to(torch.float64)
        ys = y[r0:r0 + 16384].to(torch.float64)
        lhs = ys @ Vd
        rhs = xs @ U + bv
        slack = (K * 2.0 ** -24 + 2.0 ** -11) * (xs.abs() @ Uabs + bv.abs()) + 2.0 ** -11 * (ys.abs() @ Vd) + 1e-6
        worst = max(worst, float(((lhs - rhs).abs() / slack).max()))
    assert worst <= 1.0, worst
