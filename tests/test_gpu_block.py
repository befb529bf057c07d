"""A LLaMA-shaped decoder block (7 linears, 4 distinct inputs) through the GPU path with the
layers that share an input (q/k/v, gate/up) sharing one statistics pass, one equalization
scale (from their merged weight ranges) and one activation quantization, against the same
composition of oracle functions."""
import numpy as np
import pytest
from conftest import from_panels

torch = pytest.importorskip("torch")

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def h(x):
    torch.cuda.synchronize()
    return x.cpu().numpy()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def test_block_with_shared_inputs(orc):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2311_01305_amd import binding, pipeline, synth
    binding.load_library()
    H, F, T = 512, 1408, 1536  # hidden, FFN (11 x 128), tokens
    wl = synth.scaled(synth.WORKLOADS[3], T, [])
    groups = [("attn_in", H, [("q_proj", H), ("k_proj", H), ("v_proj", H)]), ("attn_out", H, [("o_proj", H)]),
              ("mlp_in", H, [("gate_proj", F), ("up_proj", F)]), ("mlp_mid", F, [("down_proj", H)])]
    seed = 3000
    for gname, K, lins in groups:
        print(f"[gpu-block] group {gname}: K={K}, {[n for n, _ in lins]}", flush=True)
        seed += 10
        X = synth.make_act_np(seed, T, K, wl)
        Ws = [synth.make_weight_np(seed + 1 + i, N, K, wl.dtype) for i, (_, N) in enumerate(lins)]
        gb = pipeline.GroupBuffers(T, K, tuple(N for _, N in lins), torch.float16, want_out_i32=True, device=DEV)
        pipeline.calibrate_group(dev(X), [dev(W) for W in Ws], [None] * len(Ws), gb)
        t = gb.t
        # oracle: one pass over X, weight statistics merged over the group
        sx = orc.col_stats(X)
        sw = None
        for W in Ws:
            sw = orc.col_stats(W, prev=sw, want_sum=False)
        assert np.array_equal(h(t["xmin"]), sx["cmin"]) and np.array_equal(h(t["xmax"]), sx["cmax"])
        assert np.array_equal(h(t["wmin"]), sw["cmin"]) and np.array_equal(h(t["wmax"]), sw["cmax"])
        assert np.array_equal(sw["cmin"], np.min([W.astype(np.float32).min(axis=0) for W in Ws], axis=0))
        r_x, _, _ = orc.ranges(sx["cmin"], sx["cmax"])
        r_w, R_w, _ = orc.ranges(sw["cmin"], sw["cmax"])
        assert np.array_equal(h(t["r_w"]), r_w) and h(t["R_w"])[0] == R_w
        s, inv_s, _ = orc.scales(r_x, r_w)
        np.testing.assert_allclose(h(t["s"]), s, rtol=1e-5)
        gs, gi = h(t["s"]), h(t["inv_s"])
        lo, hi, mu = orc.xhat_stats(sx["cmin"], sx["cmax"], sx["csum"], sx["count"], gi)
        step, zero, _ = orc.qparams(lo, hi, 8)
        assert h(t["act_step"])[0] == step and int(h(t["act_zero"])[0]) == zero
        a = orc.quant_act(X, gi, step, zero)
        assert np.array_equal(from_panels(h(t["xq"]), T, K), a["xq"]) and np.array_equal(h(t["colsum_xq"]), a["colsum_xq"])
        for W, p, (name, N) in zip(Ws, gb.per, lins):
            Wh = orc.fold_weight(W, gs)
            assert np.array_equal(h(p["W_hat"]).view(np.uint16), Wh.view(np.uint16)), name
            q = orc.quant_weight(Wh, 8, 0)
            wq = orc.pack_codes(q["codes_u"], 8)
            assert np.array_equal(from_panels(h(p["codes"]), N, K), wq), name
            acc = orc.gemm_i8(a["xq"], wq)
            assert np.array_equal(h(p["out_i32"]), acc), name
            csa = acc.astype(np.int64).sum(axis=0)
            assert np.array_equal(h(p["colsum_acc"]), csa), name
            d_ref, b_ref = orc.bias_w8a8(Wh, h(t["mu_xhat"]), T, csa, a["colsum_xq"], q["rowsum_w"], step, zero,
                                         q["step"], q["zero"], None)
            assert np.max(np.abs(h(p["delta"]) - d_ref)) <= 1e-5 * np.max(np.abs(d_ref)), name
            # the shared scale still leaves every layer's FP product unchanged (Eq. 3)
            Xh = orc.fold_act(X[:64], gi).astype(np.float64)
            y0 = X[:64].astype(np.float64) @ W.astype(np.float64).T
            y1 = Xh @ Wh.astype(np.float64).T
            assert np.max(np.abs(y1 - y0)) <= 3e-3 * np.max(np.abs(y0))
        assert int(h(t["status"])[0]) == 0
