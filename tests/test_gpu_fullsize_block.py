"""The whole LLaMA-7B-shaped decoder block at full size (T = 262144 calibration tokens, fp16, W8A8 with
bias correction) with its real data flow -- the linears that read the same activation share one
statistics pass, one equalization scale from their merged weight ranges and one activation
quantization (Sec. 3.1: equalization sits at the entrance of the attention block and of the MLP):
q/k/v, o, gate/up, down = 7 linears on 4 distinct inputs, in the launch configuration bench.py times
(`pipeline.calibrate_group`).

Statistics, scales, weight codes and the activation quantizer's sums are checked against the oracle over
the FULL inputs; activation codes and int32 GEMM outputs on sampled rows the oracle computes one by one,
plus properties that hold at any size (Freivalds products over the whole output, the column-sum identity);
the bias correction to 1e-5 of its norm."""
import numpy as np
import pytest
from conftest import from_panels

torch = pytest.importorskip("torch")

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
CFG = 3
GROUPS = (("q_proj", "k_proj", "v_proj"), ("o_proj",), ("gate_proj", "up_proj"), ("down_proj",))


def progress(msg):
    print(f"[gpu-fullsize-block] {msg}", flush=True)


def h(x):
    return x.cpu().numpy()


@pytest.fixture(scope="module", params=range(len(GROUPS)), ids=["qkv", "o", "gate_up", "down"])
def run(request):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2311_01305_amd import binding, pipeline, synth
    binding.load_library()
    wl = synth.WORKLOADS[CFG]
    names = GROUPS[request.param]
    members = [(j, l) for j, l in enumerate(wl.linears) if l.name in names]
    li, lin = members[0]
    progress(f"group {names}: generating X[{wl.T} x {lin.K}] on the device")
    X = synth.make_act_torch(synth.layer_seed(CFG, li), wl.T, lin.K, wl, DEV)
    Ws = [synth.make_weight_torch(synth.layer_seed(CFG, j), l.N, l.K, wl.dtype, DEV) for j, l in members]
    gb = pipeline.GroupBuffers(wl.T, lin.K, tuple(l.N for _, l in members), torch.float16, want_out_i32=True, device=DEV)
    progress("running the group")
    pipeline.calibrate_group(X, Ws, [None] * len(Ws), gb)
    torch.cuda.synchronize()
    yield dict(wl=wl, K=lin.K, lins=[l for _, l in members], X=X, Ws=Ws, gb=gb)
    del X, Ws, gb
    torch.cuda.empty_cache()


def test_block_statistics_and_shared_scale(run, orc):
    t, wl, K = run["gb"].t, run["wl"], run["K"]
    progress("oracle statistics over the full X (host) and the merged weight ranges")
    Xh = h(run["X"])
    sx = orc.col_stats(Xh)
    assert np.array_equal(h(t["xmin"]), sx["cmin"]) and np.array_equal(h(t["xmax"]), sx["cmax"])
    mean_abs = np.abs(Xh[::64].astype(np.float64)).mean(axis=0)
    assert np.all(np.abs(h(t["xsum"]) - sx["csum"]) / wl.T <= 1e-6 * mean_abs + 1e-12)
    sw = None
    for W in run["Ws"]:
        sw = orc.col_stats(h(W), prev=sw, want_sum=False)
    assert np.array_equal(h(t["wmin"]), sw["cmin"]) and np.array_equal(h(t["wmax"]), sw["cmax"])
    r_x, R_x, p_x = orc.ranges(sx["cmin"], sx["cmax"])
    r_w, R_w, p_w = orc.ranges(sw["cmin"], sw["cmax"])
    assert np.array_equal(h(t["r_x"]), r_x) and np.array_equal(h(t["r_w"]), r_w)
    assert h(t["R_x"])[0] == R_x and h(t["R_w"])[0] == R_w
    np.testing.assert_allclose(h(t["p_x"]), p_x, rtol=1e-6)
    np.testing.assert_allclose(h(t["p_w"]), p_w, rtol=1e-6)
    s, inv_s, _ = orc.scales(r_x, r_w)
    np.testing.assert_allclose(h(t["s"]), s, rtol=1e-5)
    np.testing.assert_allclose(h(t["inv_s"]), inv_s, rtol=1e-5)
    lo, hi, mu = orc.xhat_stats(sx["cmin"], sx["cmax"], sx["csum"], sx["count"], h(t["inv_s"]))
    assert h(t["xhat_range"]).tolist() == [float(lo), float(hi)]
    np.testing.assert_allclose(h(t["mu_xhat"]), mu, rtol=1e-5, atol=1e-9)
    step, zero, _ = orc.qparams(lo, hi, 8)
    assert h(t["act_step"])[0] == step and int(h(t["act_zero"])[0]) == zero
    assert int(h(t["status"])[0]) == 0
    run["Xh"] = Xh


def xq_rows_dev(xq, T, K, idx):
    """Rows idx (a tensor of indices or a slice) of the K-panel buffer xq as a row-major [len, K] tensor."""
    assert K % 64 == 0
    return xq.view(K // 64, T, 64)[:, idx, :].permute(1, 0, 2).reshape(-1, K)


def sample_rows(T):
    rng = np.random.default_rng(4321)
    return np.unique(np.concatenate([np.arange(128), np.arange(T - 128, T), rng.integers(0, T, 128),
                                     np.arange(T // 2 - 3, T // 2 + 3)])).astype(np.int64)


def test_block_shared_activation_quantizer(run, orc):
    t, wl, K = run["gb"].t, run["wl"], run["K"]
    Xh = run.pop("Xh", None)
    if Xh is None:
        Xh = h(run["X"])
    progress("oracle activation quantizer over the full X (host)")
    a = orc.quant_act(Xh, h(t["inv_s"]), h(t["act_step"])[0], int(h(t["act_zero"])[0]))
    assert np.array_equal(h(t["rowsum_x"]), a["rowsum_x"]) and np.array_equal(h(t["colsum_xq"]), a["colsum_xq"])
    rows = sample_rows(wl.T)
    assert np.array_equal(h(xq_rows_dev(t["xq"], wl.T, K, torch.from_numpy(rows).to(DEV))), a["xq"][rows])
    assert a["status"] == 0 and a["xq"].min() == -128 and a["xq"].max() == 127


def test_block_members_weights_gemm_and_bias(run, orc):
    gb, wl, K = run["gb"], run["wl"], run["K"]
    t = gb.t
    gs = h(t["s"])
    rows = sample_rows(wl.T)
    idx = torch.from_numpy(rows).to(DEV)
    xq_rows = h(xq_rows_dev(t["xq"], wl.T, K, idx))
    colsum_xq = h(t["colsum_xq"])
    rng = np.random.default_rng(11)
    for lin, W, p in zip(run["lins"], run["Ws"], gb.per):
        progress(f"{lin.name}: fold + weight quantizer (all rows), GEMM ({rows.size} sampled rows, Freivalds), bias")
        Wh = orc.fold_weight(h(W), gs)
        assert np.array_equal(h(p["W_hat"]).view(np.uint16), Wh.view(np.uint16)), lin.name
        q = orc.quant_weight(Wh, 8, 0)
        wq = orc.pack_codes(q["codes_u"], 8)
        assert np.array_equal(h(p["step_w"]), q["step"]) and np.array_equal(h(p["zero_w"]), q["zero"]), lin.name
        assert np.array_equal(from_panels(h(p["codes"]), lin.N, K), wq), lin.name
        assert np.array_equal(h(p["rowsum_w"]), q["rowsum_w"]), lin.name
        assert np.array_equal(h(p["out_i32"][idx]), orc.gemm_i8(xq_rows, wq)), lin.name
        # Freivalds: acc v = xq (wq^T v) for random 0/1 vectors, exact in fp64 (all values < 2^53)
        V = rng.integers(0, 2, (lin.N, 3)).astype(np.float64)
        Vd, Ud = torch.from_numpy(V).to(DEV), torch.from_numpy(wq.astype(np.float64).T @ V).to(DEV)
        for r0 in range(0, wl.T, 32768):
            lhs = p["out_i32"][r0:r0 + 32768].to(torch.float64) @ Vd
            rhs = xq_rows_dev(t["xq"], wl.T, K, slice(r0, r0 + 32768)).to(torch.float64) @ Ud
            assert torch.equal(lhs, rhs), f"{lin.name}: Freivalds mismatch in rows {r0}.."
        # sum over tokens of the accumulator = wq . (column sums of xq): exact integers
        assert np.array_equal(h(p["colsum_acc"]), orc.colsum_acc_from_colsum_xq(wq, colsum_xq)), lin.name
        d_ref, b_ref = orc.bias_w8a8(Wh, h(t["mu_xhat"]), wl.T, h(p["colsum_acc"]), colsum_xq, q["rowsum_w"],
                                     h(t["act_step"])[0], int(h(t["act_zero"])[0]), q["step"], q["zero"], None)
        assert np.max(np.abs(h(p["delta"]) - d_ref)) <= 1e-5 * np.max(np.abs(d_ref)), lin.name
        np.testing.assert_allclose(h(p["bias_out"]), b_ref, rtol=1e-5, atol=1e-5 * np.max(np.abs(d_ref)))
