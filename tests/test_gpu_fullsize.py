"""Parity at the full size and in the launch configuration bench.py times: linears of the
OPT-6.7B-shaped block (q_proj: T = 262144 calibration tokens, 4096 x 4096, fp16) and of the
LLaMA-7B-shaped block (down_proj: 4096 x 11008, heavy-tailed activations, three ragged column
chunks in the activation quantizer, 172 K-panels in the GEMM) and of the LLaMA-65B-shaped block
(gate_proj: 22016 x 8192, 86 output-tile columns, 23 GB of int32 output; down_proj: 8192 x 22016, 11.5 GB of
activations, 344 K-panels: both distinct inputs of the configuration the benchmark's default line runs) run through the whole
path on the GPU with the same driver the benchmark uses.

The streaming stages are checked against the oracle over the FULL input (statistics, and the
activation quantizer's codes through its exact column / row sums); the int32 GEMM output on
sampled rows the oracle computes one by one, plus properties that hold at any size (Freivalds
products, the column-sum identity).  No teacher forcing is needed for the integer stages:
they are checked against the oracle fed the GPU's own fp32 scales.
"""
import numpy as np
import pytest
from conftest import from_panels

torch = pytest.importorskip("torch")

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def progress(msg):
    print(f"[gpu-fullsize] {msg}", flush=True)


@pytest.fixture(scope="module", params=[(2, 0), (3, 6), (5, 4), (5, 6)],
                ids=["opt6.7b-q_proj", "llama7b-down_proj", "llama65b-gate_proj", "llama65b-down_proj"])
def run(request):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2311_01305_amd import binding, pipeline, synth
    binding.load_library()
    cfg, li = request.param
    wl = synth.WORKLOADS[cfg]
    lin = wl.linears[li]
    seed = synth.layer_seed(cfg, li)
    progress(f"generating {lin.name} X[{wl.T} x {lin.K}] on the device")
    X = synth.make_act_torch(seed, wl.T, lin.K, wl, DEV)
    W = synth.make_weight_torch(seed, lin.N, lin.K, wl.dtype, DEV)
    b_np = synth.make_bias_np(seed, lin.N, wl.has_bias)
    b = None if b_np is None else torch.from_numpy(b_np).to(DEV)
    buf = pipeline.LayerBuffers(wl.T, lin.K, lin.N, torch.float16, want_out_i32=True, want_out_deq=False, device=DEV)
    progress("running the whole path")
    t = pipeline.calibrate_layer(X, W, b, buf, fused_weight_pass=True)  # the call sequence bench.py times
    torch.cuda.synchronize()
    return dict(wl=wl, lin=lin, X=X, W=W, b=b, t=t)


def h(x):
    return x.cpu().numpy()


def test_fullsize_statistics_and_scales(run, orc):
    t, wl, lin = run["t"], run["wl"], run["lin"]
    progress("oracle statistics over the full X (host)")
    Xh = h(run["X"])
    sx = orc.col_stats(Xh)
    assert np.array_equal(h(t["xmin"]), sx["cmin"]) and np.array_equal(h(t["xmax"]), sx["cmax"])
    # library special case: numpy's reductions on the same bits
    assert np.array_equal(sx["cmin"], Xh.min(axis=0).astype(np.float32))
    mean_abs = np.abs(Xh[::64].astype(np.float64)).mean(axis=0)
    assert np.all(np.abs(h(t["xsum"]) - sx["csum"]) / wl.T <= 1e-6 * mean_abs + 1e-12)
    assert int(h(t["count"])[0]) == wl.T
    sw = orc.col_stats(h(run["W"]), want_sum=False)
    assert np.array_equal(h(t["wmin"]), sw["cmin"]) and np.array_equal(h(t["wmax"]), sw["cmax"])
    r_x, R_x, p_x = orc.ranges(sx["cmin"], sx["cmax"])
    r_w, R_w, p_w = orc.ranges(sw["cmin"], sw["cmax"])
    assert np.array_equal(h(t["r_x"]), r_x) and h(t["R_x"])[0] == R_x and h(t["R_w"])[0] == R_w
    np.testing.assert_allclose(h(t["p_x"]), p_x, rtol=1e-6)
    s, inv_s, st = orc.scales(r_x, r_w)
    np.testing.assert_allclose(h(t["s"]), s, rtol=1e-5)
    np.testing.assert_allclose(h(t["inv_s"]), inv_s, rtol=1e-5)
    lo, hi, mu = orc.xhat_stats(sx["cmin"], sx["cmax"], sx["csum"], sx["count"], h(t["inv_s"]))
    assert h(t["xhat_range"]).tolist() == [float(lo), float(hi)]
    np.testing.assert_allclose(h(t["mu_xhat"]), mu, rtol=1e-5, atol=1e-9)
    step, zero, _ = orc.qparams(lo, hi, 8)
    assert h(t["act_step"])[0] == step and int(h(t["act_zero"])[0]) == zero
    assert int(h(t["status"])[0]) == 0
    run["Xh"] = Xh


def test_fullsize_weight_quantizer(run, orc):
    t, lin = run["t"], run["lin"]
    progress("weight fold + quantizer, all rows")
    Wh = orc.fold_weight(h(run["W"]), h(t["s"]))
    assert np.array_equal(h(t["W_hat"]).view(np.uint16), Wh.view(np.uint16))
    q = orc.quant_weight(Wh, 8, 0)
    assert np.array_equal(h(t["step_w"]), q["step"]) and np.array_equal(h(t["zero_w"]), q["zero"])
    assert np.array_equal(from_panels(h(t["codes"]), lin.N, lin.K), orc.pack_codes(q["codes_u"], 8))
    assert np.array_equal(h(t["rowsum_w"]), q["rowsum_w"])
    run["q"] = q


def test_fullsize_activation_quantizer(run, orc):
    t, wl = run["t"], run["wl"]
    Xh = run.get("Xh")
    if Xh is None:
        Xh = h(run["X"])
    progress("oracle activation quantizer over the full X (host)")
    a = orc.quant_act(Xh, h(t["inv_s"]), h(t["act_step"])[0], int(h(t["act_zero"])[0]))
    # every row sum and every column sum exact, and the codes themselves on a sample of rows
    assert np.array_equal(h(t["rowsum_x"]), a["rowsum_x"])
    assert np.array_equal(h(t["colsum_xq"]), a["colsum_xq"])
    rows = sample_rows(wl.T)
    assert np.array_equal(h(xq_rows_dev(t["xq"], wl.T, Xh.shape[1], torch.from_numpy(rows).to(DEV))), a["xq"][rows])
    assert a["xq"].min() == -128 and a["xq"].max() == 127
    run["a_rows"] = (rows, a["xq"][rows].copy())
    run["colsum_xq"] = a["colsum_xq"]


def xq_rows_dev(xq, T, K, idx):
    """Rows idx (a tensor of indices or a slice) of the K-panel buffer xq as a row-major [len, K] tensor."""
    assert K % 64 == 0
    v = xq.view(K // 64, T, 64)[:, idx, :]
    return v.permute(1, 0, 2).reshape(-1, K)


def sample_rows(T):
    rng = np.random.default_rng(12345)
    return np.unique(np.concatenate([np.arange(256), np.arange(T - 256, T), rng.integers(0, T, 256),
                                     np.arange(T // 2 - 3, T // 2 + 3)])).astype(np.int64)


def test_fullsize_gemm(run, orc):
    t, wl, lin = run["t"], run["wl"], run["lin"]
    wq = from_panels(h(t["codes"]), lin.N, lin.K)
    rows = sample_rows(wl.T)
    idx = torch.from_numpy(rows).to(DEV)
    progress(f"oracle GEMM on {rows.size} sampled rows")
    xq_rows = h(xq_rows_dev(t["xq"], wl.T, lin.K, idx))
    ref = orc.gemm_i8(xq_rows, wq)
    assert np.array_equal(h(t["out_i32"][idx]), ref)
    # Freivalds: acc v = xq (wq^T v) for random 0/1 vectors, exact in fp64 (all values < 2^53)
    progress("Freivalds products over the full output")
    rng = np.random.default_rng(7)
    V = rng.integers(0, 2, (lin.N, 4)).astype(np.float64)
    U = wq.astype(np.float64).T @ V
    Vd, Ud = torch.from_numpy(V).to(DEV), torch.from_numpy(U).to(DEV)
    for r0 in range(0, wl.T, 32768):
        lhs = t["out_i32"][r0:r0 + 32768].to(torch.float64) @ Vd
        rhs = xq_rows_dev(t["xq"], wl.T, lin.K, slice(r0, r0 + 32768)).to(torch.float64) @ Ud
        assert torch.equal(lhs, rhs), f"Freivalds mismatch in rows {r0}.."
    # sum over tokens of the accumulator = wq . (column sums of xq): exact integers
    colsum_xq = run.get("colsum_xq")
    if colsum_xq is None:
        colsum_xq = h(t["colsum_xq"])
    assert np.array_equal(h(t["colsum_acc"]), orc.colsum_acc_from_colsum_xq(wq, colsum_xq))


def test_fullsize_bias_correction(run, orc):
    t, wl, lin = run["t"], run["wl"], run["lin"]
    progress("bias correction")
    d_ref, b_ref = orc.bias_w8a8(h(t["W_hat"]), h(t["mu_xhat"]), wl.T, h(t["colsum_acc"]), h(t["colsum_xq"]),
                                 h(t["rowsum_w"]), h(t["act_step"])[0], int(h(t["act_zero"])[0]), h(t["step_w"]),
                                 h(t["zero_w"]), None if run["b"] is None else h(run["b"]))
    assert np.max(np.abs(h(t["delta"]) - d_ref)) <= 1e-5 * np.max(np.abs(d_ref))
    np.testing.assert_allclose(h(t["bias_out"]), b_ref, rtol=1e-5, atol=1e-5 * np.max(np.abs(d_ref)))
