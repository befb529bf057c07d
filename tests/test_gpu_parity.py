"""Parity of the HIP path (through the C ABI) with the CPU oracle, stage by stage with
teacher forcing: each GPU stage is fed the oracle's outputs of the previous stage.

Bars: min / max / ranges exact; codes, zero points, row / column sums and int32 GEMM
outputs bit-exact given identical fp32 scales; scales and bias corrections <= 1e-5 relative.
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


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def dtc(B, a):
    return B.AWEQ_F16 if a.dtype in (np.float16, torch.float16) else B.AWEQ_F32


def e(*shape, dtype):
    return torch.empty(shape, dtype=dtype, device=DEV)


def qa_ws(B, T, K):
    """Workspace of the activation quantizer, filled with garbage: its contents must not matter."""
    n = max(16, B.aweq_workspace_size(B.OP_QUANT_ACT, T, K))
    return torch.full((n,), 0x5A, dtype=torch.uint8, device=DEV)


def progress(msg):
    print(f"[gpu-parity] {msg}", flush=True)


# ------------------------------------------------------------------------------ stage 1


def gpu_stats(B, M_t, rows, K, ld, prev=None, want_sum=True, finalize=True):
    dt = dtc(B, M_t)
    if prev is None:
        cmin, cmax = e(K, dtype=torch.float32), e(K, dtype=torch.float32)
        csum = e(K, dtype=torch.float64) if want_sum else None
        count = torch.zeros(1, dtype=torch.int64, device=DEV)
        acc = 0
    else:
        cmin, cmax, csum, count = prev
        acc = 1
    r, R, p = e(K, dtype=torch.float32), e(1, dtype=torch.float32), e(K, dtype=torch.float32)
    ws = e(max(16, B.aweq_workspace_size(B.OP_CALIB_STATS, rows, K)), dtype=torch.uint8)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    B.aweq_calib_stats(M_t, dt, rows, K, ld, cmin, cmax, csum, count, acc, int(finalize), r, R, p, ws, status)
    return dict(cmin=cmin, cmax=cmax, csum=csum, count=count, r=r, R=R, p=p, status=status)


@pytest.mark.parametrize("dtype,rows,K", [
    (np.float16, 1000, 520),     # ragged rows, two column chunks with a ragged tail
    (np.float16, 37, 8),         # fewer rows than one row batch
    (np.float16, 4099, 1536),    # several slices, several chunks
    (np.float32, 2048, 512),     # config-1 shape
    (np.float32, 777, 264),
    (np.float16, 1, 64),
])
def test_stats_parity(B, orc, dtype, rows, K):
    progress(f"stats {dtype.__name__} rows={rows} K={K}")
    rng = np.random.default_rng(rows * 31 + K)
    M = (rng.standard_normal((rows, K)) * 3).astype(dtype)
    M[:, K // 3] *= 50
    g = gpu_stats(B, dev(M), rows, K, K)
    o = orc.col_stats(M)
    assert np.array_equal(host(g["cmin"]), o["cmin"]) and np.array_equal(host(g["cmax"]), o["cmax"])
    scale = np.abs(M.astype(np.float64)).mean(axis=0) * rows
    assert np.all(np.abs(host(g["csum"]) - o["csum"]) <= 1e-6 * scale + 1e-12)
    assert int(host(g["count"])[0]) == rows and int(host(g["status"])[0]) == 0
    r, R, p = orc.ranges(o["cmin"], o["cmax"])
    assert np.array_equal(host(g["r"]), r) and host(g["R"])[0] == R
    np.testing.assert_allclose(host(g["p"]), p, rtol=1e-6)


def test_stats_pitch_accumulate_and_flags(B, orc):
    progress("stats pitch/accumulate/nonfinite")
    rng = np.random.default_rng(5)
    rows, K, ld = 300, 128, 160
    buf = rng.standard_normal((rows, ld)).astype(np.float16)
    M = buf[:, :K]
    t = dev(buf)
    g = gpu_stats(B, t, rows, K, ld)
    o = orc.col_stats(np.ascontiguousarray(M))
    assert np.array_equal(host(g["cmin"]), o["cmin"]) and np.array_equal(host(g["cmax"]), o["cmax"])
    # two batches merged == one pass (min of mins, max of maxes, counts add)
    a = gpu_stats(B, dev(buf[:100]), 100, K, ld, finalize=False)
    b = gpu_stats(B, dev(buf[100:]), 200, K, ld, prev=(a["cmin"], a["cmax"], a["csum"], a["count"]))
    assert np.array_equal(host(b["cmin"]), o["cmin"]) and np.array_equal(host(b["cmax"]), o["cmax"])
    assert int(host(b["count"])[0]) == rows
    np.testing.assert_allclose(host(b["csum"]), o["csum"], rtol=1e-6, atol=1e-4)
    # weights: no sums asked
    w = gpu_stats(B, t, rows, K, ld, want_sum=False)
    assert np.array_equal(host(w["cmax"]), o["cmax"])
    bad = M.copy()
    bad[17, 5] = np.inf
    assert int(host(gpu_stats(B, dev(np.ascontiguousarray(bad)), rows, K, K)["status"])[0]) & B.ST_NONFINITE
    # determinism: run twice, identical bits (fixed reduction order)
    g2 = gpu_stats(B, t, rows, K, ld)
    assert np.array_equal(host(g["csum"]).view(np.int64), host(g2["csum"]).view(np.int64))


# ------------------------------------------------------------------------------ stage 2


def make_layer(rng, dtype, T, K, N, outliers=(3,), factor=40.0):
    X = rng.standard_normal((T, K)).astype(np.float32) + rng.uniform(-0.3, 0.3, K).astype(np.float32)
    for c in outliers:
        X[:, c % K] *= factor
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    return X.astype(dtype), W.astype(dtype)


def oracle_front(orc, X, W, enable_awe=True):
    sx, sw = orc.col_stats(X), orc.col_stats(W, want_sum=False)
    r_x, _, _ = orc.ranges(sx["cmin"], sx["cmax"])
    r_w, _, _ = orc.ranges(sw["cmin"], sw["cmax"])
    s, inv_s, st = orc.scales(r_x, r_w, enable_awe)
    return sx, sw, s, inv_s, st


def gpu_equalize(B, sx, sw, W, enable_awe=True, prev_scale=None):
    N, K = W.shape
    s, inv_s, mu = e(K, dtype=torch.float32), e(K, dtype=torch.float32), e(K, dtype=torch.float32)
    W_t = dev(W)
    W_hat = torch.empty_like(W_t)
    rng_t, step, zero = e(2, dtype=torch.float32), e(1, dtype=torch.float32), e(1, dtype=torch.int32)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    B.aweq_equalize(dev(sx["cmin"]), dev(sx["cmax"]), dev(sx["csum"]), sx["count"], dev(sw["cmin"]), dev(sw["cmax"]),
                    K, int(enable_awe), s, inv_s, W_t, W_hat, dtc(B, W), N, K, K, prev_scale, rng_t, mu, step, zero, status)
    return dict(s=s, inv_s=inv_s, W_hat=W_hat, xhat_range=rng_t, mu_xhat=mu, act_step=step, act_zero=zero, status=status)


@pytest.mark.parametrize("dtype,T,K,N", [(np.float16, 200, 520, 33), (np.float32, 128, 512, 64), (np.float16, 64, 4104, 5)])
def test_equalize_parity(B, orc, dtype, T, K, N):
    progress(f"equalize {dtype.__name__} T={T} K={K} N={N}")
    rng = np.random.default_rng(K + N)
    X, W = make_layer(rng, dtype, T, K, N, outliers=(3, 100))
    sx, sw, s, inv_s, st = oracle_front(orc, X, W)
    prev = dev(np.arange(1, K + 1, dtype=np.float32))
    g = gpu_equalize(B, sx, sw, W, prev_scale=prev)
    gs, gi = host(g["s"]), host(g["inv_s"])
    np.testing.assert_allclose(gs, s, rtol=1e-6)
    np.testing.assert_allclose(gi, inv_s, rtol=1e-6)
    assert int(host(g["status"])[0]) == st
    # given the scales the GPU produced, everything downstream is exact
    assert np.array_equal(gi, np.float32(1.0) / gs)
    assert np.array_equal(host(g["W_hat"]).view(np.uint16 if dtype == np.float16 else np.uint32),
                          orc.fold_weight(W, gs).view(np.uint16 if dtype == np.float16 else np.uint32))
    lo, hi, mu = orc.xhat_stats(sx["cmin"], sx["cmax"], sx["csum"], sx["count"], gi)
    assert host(g["xhat_range"]).tolist() == [float(lo), float(hi)]
    np.testing.assert_allclose(host(g["mu_xhat"]), mu, rtol=1e-6, atol=1e-30)
    step, zero, _ = orc.qparams(lo, hi, 8)
    assert host(g["act_step"])[0] == step and int(host(g["act_zero"])[0]) == zero
    np.testing.assert_allclose(host(prev), np.arange(1, K + 1, dtype=np.float32) * gi, rtol=1e-7)


def test_equalize_switch_and_guards(B, orc):
    progress("equalize AWE off / guards")
    rng = np.random.default_rng(9)
    X, W = make_layer(rng, np.float16, 64, 64, 16)
    X[:, 7] = 0.25   # constant activation channel: r_x = 0 -> s = 1
    W[:, 9] = 0.0    # dead weight channel: r_w = 0 -> s = 1
    sx, sw, s, inv_s, st = oracle_front(orc, X, W)
    g = gpu_equalize(B, sx, sw, W)
    gs = host(g["s"])
    assert gs[7] == 1.0 and gs[9] == 1.0 and int(host(g["status"])[0]) & B.ST_SCALEGUARD and st & orc.ST_SCALEGUARD
    np.testing.assert_allclose(gs, s, rtol=1e-6)
    off = gpu_equalize(B, sx, sw, W, enable_awe=False)
    assert np.all(host(off["s"]) == 1.0) and np.all(host(off["inv_s"]) == 1.0)
    assert np.array_equal(host(off["W_hat"]).view(np.uint16), W.view(np.uint16))


# ------------------------------------------------------------------------------ stage 3


def gpu_quant_weight(B, Wh, bits, group, want_rowsum=True):
    N, K = Wh.shape
    ng = 1 if group < 0 else (N if group == 0 else N * (K // group))
    panel = bits == 8 and group <= 0  # the GEMM's weight operand: K-panel layout
    codes = torch.full((B.aweq_panel_bytes(N, K) if panel else N * K * bits // 8,), 0x5a, dtype=torch.uint8, device=DEV)
    step, zero = e(ng, dtype=torch.float32), e(ng, dtype=torch.int32)
    rowsum = e(N, dtype=torch.int32) if (bits == 8 and group <= 0 and want_rowsum) else None
    ws = e(64, dtype=torch.uint8)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    B.aweq_quant_weight(dev(Wh), dtc(B, Wh), N, K, K, bits, group, codes, step, zero, rowsum, ws, status)
    return dict(codes=codes, step=step, zero=zero, rowsum_w=rowsum, status=status)


@pytest.mark.parametrize("dtype,N,K,bits,group", [
    (np.float16, 37, 4096, 8, 0),
    (np.float16, 5, 11008, 8, 0),     # row longer than one pass of the block, ragged
    (np.float16, 3, 24576, 8, 0),     # the longest row the block holds
    (np.float32, 64, 512, 8, 0),      # config-1
    (np.float16, 19, 4096, 4, 128),
    (np.float16, 19, 4096, 3, 128),
    (np.float16, 7, 11008, 4, 128),   # 86 groups per row, ragged last block
    (np.float16, 7, 11008, 3, 128),
    (np.float32, 9, 1024, 4, 128),
    (np.float32, 9, 1024, 3, 32),
    (np.float16, 6, 512, 4, 8),       # one-lane groups
    (np.float16, 6, 1024, 3, 512),    # whole-wavefront groups
    (np.float16, 11, 2048, 4, 0),     # per-row 4-bit
    (np.float16, 11, 2048, 3, 0),
    (np.float16, 21, 1024, 8, -1),    # per-tensor
    (np.float16, 21, 1024, 4, -1),
    (np.float16, 4, 256, 8, 64),      # grouped int8 (no row sums)
])
def test_quant_weight_parity(B, orc, dtype, N, K, bits, group):
    progress(f"quant_weight {dtype.__name__} N={N} K={K} b={bits} g={group}")
    rng = np.random.default_rng(N * 7 + K + bits + group)
    Wh = (rng.standard_normal((N, K)) * 0.02 * rng.uniform(0.2, 5.0, (1, K))).astype(dtype)
    if N > 2:
        Wh[1, : min(K, 256)] = 0  # an all-zero group / partly constant row
    o = orc.quant_weight(Wh, bits, group)
    g = gpu_quant_weight(B, Wh, bits, group)
    assert np.array_equal(host(g["step"]), o["step"].reshape(-1))
    assert np.array_equal(host(g["zero"]), o["zero"].reshape(-1))
    packed = orc.pack_codes(o["codes_u"], bits).view(np.uint8).reshape(-1)
    got = host(g["codes"])
    if bits == 8 and group <= 0:
        got = from_panels(got, N, K).reshape(-1)
    assert np.array_equal(got, packed)
    if g["rowsum_w"] is not None:
        assert np.array_equal(host(g["rowsum_w"]), o["rowsum_w"])
    assert int(host(g["status"])[0]) == o["status"]


def test_quant_weight_degenerate_and_half_ties(B, orc):
    progress("quant_weight degenerate / ties")
    # values sitting exactly on rounding ties (the b = 3 worked example, tiled)
    base = np.array([-1, -0.75, -0.25, 0, 0.25, 0.75, 1.3, 2.5], np.float16)
    Wh = np.tile(base, (4, 16))
    o = orc.quant_weight(Wh, 3, 0)
    g = gpu_quant_weight(B, Wh, 3, 0)
    assert np.array_equal(host(g["codes"]), orc.pack_codes(o["codes_u"], 3).reshape(-1))
    assert o["codes_u"][0, :8].tolist() == [0, 0, 2, 2, 2, 4, 5, 7]
    z = np.zeros((3, 128), np.float16)
    g = gpu_quant_weight(B, z, 8, 0)
    assert np.all(host(g["step"]) == 1.0) and np.all(host(g["zero"]) == 0)
    assert np.all(from_panels(host(g["codes"]), 3, 128).view(np.int8) == -128) and int(host(g["status"])[0]) & B.ST_DEGENERATE


@pytest.mark.parametrize("dtype,N,K,bits", [(np.float16, 37, 4096, 8), (np.float16, 5, 11008, 8), (np.float32, 64, 520, 8),
                                             (np.float16, 11, 2048, 4), (np.float16, 11, 2048, 3)])
def test_fold_quant_weight_equals_two_calls(B, orc, dtype, N, K, bits):
    """The fused fold + per-row quantizer against the oracle's fold followed by its quantizer."""
    progress(f"fold+quant {dtype.__name__} N={N} K={K} b={bits}")
    rng = np.random.default_rng(N + K + bits)
    W = (rng.standard_normal((N, K)) * 0.02).astype(dtype)
    s = rng.uniform(0.2, 5.0, K).astype(np.float32)
    Wh = orc.fold_weight(W, s)
    o = orc.quant_weight(Wh, bits, 0)
    panel = bits == 8
    codes = torch.full((B.aweq_panel_bytes(N, K) if panel else N * K * bits // 8,), 0x5a, dtype=torch.uint8, device=DEV)
    step, zero = e(N, dtype=torch.float32), e(N, dtype=torch.int32)
    rowsum = e(N, dtype=torch.int32) if bits == 8 else None
    W_hat = torch.zeros((N, K), dtype=torch.float16 if dtype == np.float16 else torch.float32, device=DEV)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    B.aweq_fold_quant_weight(dev(W), dtc(B, W), N, K, K, dev(s), W_hat, K, bits, codes, step, zero, rowsum, status)
    assert np.array_equal(host(W_hat).view(np.uint8), Wh.view(np.uint8))
    assert np.array_equal(host(step), o["step"]) and np.array_equal(host(zero), o["zero"])
    got = host(codes)
    if panel:
        got = from_panels(got, N, K).reshape(-1)
        assert np.array_equal(host(rowsum), o["rowsum_w"])
    assert np.array_equal(got, orc.pack_codes(o["codes_u"], bits).view(np.uint8).reshape(-1))
    assert int(host(status)[0]) == o["status"]
    # in place: W_hat aliasing W
    Wd = dev(W)
    B.aweq_fold_quant_weight(Wd, dtc(B, W), N, K, K, dev(s), Wd, K, bits, codes, step, zero, rowsum, status)
    assert np.array_equal(host(Wd).view(np.uint8), Wh.view(np.uint8)) and np.array_equal(host(zero), o["zero"])


def double_rounding_pairs(rng, count, want_up):
    """(w binary16, s binary32) pairs whose product rounds differently in one step (exact -> binary16)
    than in the two steps of the fold (exact -> binary32 -> binary16); want_up: single > double."""
    out = []
    while len(out) < count:
        w = rng.uniform(0.5, 1.0, 400000).astype(np.float16)
        s = rng.uniform(16.0, 32.0, w.size).astype(np.float32)
        two = (w.astype(np.float32) * s).astype(np.float16)
        one = (w.astype(np.float64) * s.astype(np.float64)).astype(np.float16)
        pick = np.nonzero((one > two) if want_up else (one < two))[0]
        out += [(w[i], s[i]) for i in pick]
    return out[:count]


def test_fold_rounds_twice_at_the_row_extremes(B, orc):
    """Eq. 3's fold is an fp32 product rounded to the weight's type.  Each row here has its
    maximum (even rows) or minimum (odd rows) on an element where rounding the exact product
    once gives the neighbouring binary16 value: Step, Z and the codes must follow the
    twice-rounded W_hat that is stored."""
    progress("fold double rounding at the row extremes (fused fold + quantizer)")
    rng = np.random.default_rng(99)
    N, K = 16, 1024
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    s = rng.uniform(0.5, 2.0, K).astype(np.float32)
    up, down = double_rounding_pairs(rng, N // 2, True), double_rounding_pairs(rng, N // 2, False)
    for n in range(N):
        w, sv = (up if n % 2 == 0 else down)[n // 2]
        col = 8 * n + 3
        s[col] = sv
        W[:, col] = 0
        W[n, col] = w if n % 2 == 0 else -w          # negated: the minimum, with single < double
    Wh = orc.fold_weight(W, s)
    one = (W.astype(np.float64) * s.astype(np.float64)).astype(np.float16)
    assert np.count_nonzero(one != Wh) >= N and all(Wh[n].argmax() == 8 * n + 3 for n in range(0, N, 2))
    o = orc.quant_weight(Wh, 8, 0)
    codes = torch.full((B.aweq_panel_bytes(N, K),), 0x5a, dtype=torch.uint8, device=DEV)
    step, zero, rowsum = e(N, dtype=torch.float32), e(N, dtype=torch.int32), e(N, dtype=torch.int32)
    W_hat = torch.zeros((N, K), dtype=torch.float16, device=DEV)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    B.aweq_fold_quant_weight(dev(W), B.AWEQ_F16, N, K, K, dev(s), W_hat, K, 8, codes, step, zero, rowsum, status)
    assert np.array_equal(host(W_hat).view(np.uint16), Wh.view(np.uint16))
    assert np.array_equal(host(step), o["step"]) and np.array_equal(host(zero), o["zero"])
    assert np.array_equal(from_panels(host(codes), N, K).reshape(-1), orc.pack_codes(o["codes_u"], 8).view(np.uint8).reshape(-1))
    assert np.array_equal(host(rowsum), o["rowsum_w"])


# ------------------------------------------------------------------------------ stage 4a


def gpu_quant_act(B, X, inv_s, step, zero):
    T, K = X.shape
    xq = torch.full((B.aweq_panel_bytes(T, K),), 0x5a, dtype=torch.int8, device=DEV)
    rs, cs = e(T, dtype=torch.int32), e(K, dtype=torch.int64)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    B.aweq_quant_act(dev(X), dtc(B, X), T, K, K, dev(inv_s), dev(np.array([step], np.float32)),
                     dev(np.array([zero], np.int32)), xq, rs, cs, qa_ws(B, T, K), status)
    return dict(xq=xq, rowsum_x=rs, colsum_xq=cs, status=status)


def check_quant_act(B, orc, X, inv_s, step, zero):
    o = orc.quant_act(X, inv_s, step, zero)
    g = gpu_quant_act(B, X, inv_s, step, zero)
    assert np.array_equal(from_panels(host(g["xq"]), *X.shape), o["xq"])
    assert np.array_equal(host(g["rowsum_x"]), o["rowsum_x"])
    assert np.array_equal(host(g["colsum_xq"]), o["colsum_xq"])
    assert int(host(g["status"])[0]) == o["status"]
    return o


@pytest.mark.parametrize("dtype,T,K", [
    (np.float16, 1000, 4096),    # one column chunk, several row slices, ragged last batch
    (np.float16, 515, 11008),    # three column chunks (row sums via atomics), ragged
    (np.float16, 130, 520),
    (np.float32, 2048, 512),     # config-1: binary32 input takes the true division
    (np.float16, 3, 8),
])
def test_quant_act_parity(B, orc, dtype, T, K):
    progress(f"quant_act {dtype.__name__} T={T} K={K}")
    rng = np.random.default_rng(T + K)
    X, W = make_layer(rng, dtype, T, K, 16, outliers=(3, 77), factor=30.0)
    sx, sw, s, inv_s, _ = oracle_front(orc, X, W)
    lo, hi, mu = orc.xhat_stats(sx["cmin"], sx["cmax"], sx["csum"], sx["count"], inv_s)
    step, zero, _ = orc.qparams(lo, hi, 8)
    o = check_quant_act(B, orc, X, inv_s, step, zero)
    assert o["xq"].min() == -128 and o["xq"].max() == 127


def test_quant_act_sums_are_deterministic_and_ignore_the_workspace_contents(B, orc):
    """The sums go through per-slice partial buffers folded in a fixed order: two runs give the same bits
    whatever the workspace held before (no atomics, nothing to clear), for one and for several column chunks."""
    progress("quant_act determinism / workspace contents")
    rng = np.random.default_rng(314)
    for T, K in ((700, 512), (1300, 1544)):
        X = (rng.standard_normal((T, K)) * 2).astype(np.float16)
        inv_s = rng.uniform(0.3, 3.0, K).astype(np.float32)
        outs = []
        for fill in (0x00, 0xFF, 0x5A):
            xq = torch.empty(B.aweq_panel_bytes(T, K), dtype=torch.int8, device=DEV)
            rs, cs = e(T, dtype=torch.int32), e(K, dtype=torch.int64)
            ws = torch.full((B.aweq_workspace_size(B.OP_QUANT_ACT, T, K),), fill, dtype=torch.uint8, device=DEV)
            B.aweq_quant_act(dev(X), B.AWEQ_F16, T, K, K, dev(inv_s), dev(np.array([0.031], np.float32)),
                             dev(np.array([131], np.int32)), xq, rs, cs, ws, None)
            outs.append((host(xq).copy(), host(rs).copy(), host(cs).copy()))
        for o in outs[1:]:
            assert all(np.array_equal(a, b) for a, b in zip(o, outs[0]))
        ref = orc.quant_act(X, inv_s, np.float32(0.031), 131)
        assert np.array_equal(outs[0][1], ref["rowsum_x"]) and np.array_equal(outs[0][2], ref["colsum_xq"])


def test_quant_act_quotient_paths(B, orc):
    """The division-free quotient must equal the true division: many Step values (random
    significands, including ones near a power of two and the all-ones guard), values on and
    next to rounding ties, out-of-range values, a large zero point."""
    progress("quant_act quotient paths")
    rng = np.random.default_rng(77)
    T, K = 256, 512
    X = (rng.standard_normal((T, K)) * 2).astype(np.float16)
    inv_s = rng.uniform(0.05, 4.0, K).astype(np.float32)
    steps = [np.float32(0.5), np.float32(0.037), np.float32(1.0) / np.float32(3.0),
             np.nextafter(np.float32(0.125), np.float32(0)),               # significand all ones: guarded
             np.float32(np.uint32(0x3c7fffe0).view(np.float32)),           # just below the guard
             np.nextafter(np.float32(0.25), np.float32(1)), np.float32(1e-3), np.float32(7.3e-5)]
    steps += list((rng.uniform(1.0, 2.0, 12) * 2.0 ** rng.integers(-9, 0, 12)).astype(np.float32))
    for sp in steps:
        # put a band of values exactly on / next to ties of this Step
        Xt = X.copy()
        m = rng.integers(-120, 120, K).astype(np.float32) + np.float32(0.5)
        tie = (m * sp / inv_s)
        Xt[0] = tie.astype(np.float16)
        Xt[1] = np.nextafter(Xt[0], np.float16(np.inf))
        Xt[2] = np.nextafter(Xt[0], np.float16(-np.inf))
        check_quant_act(B, orc, Xt, inv_s, sp, int(rng.integers(100, 156)))
    # zero point beyond 2^23 and a huge Step take the generic path
    check_quant_act(B, orc, X, inv_s, np.float32(0.01), 1 << 24)
    check_quant_act(B, orc, X, inv_s, np.float32(2.0 ** 70), 128)
    # values far outside the calibrated range saturate at both ends
    Xo = X.copy()
    Xo[5] = 60000
    Xo[6] = -60000
    o = check_quant_act(B, orc, Xo, inv_s, np.float32(0.02), 128)
    assert o["xq"][5].max() == 127 and o["xq"][6].min() == -128


def test_quant_act_screened_near_ties(B, orc):
    """The screened quotient decides from one FMA unless a value is close to a rounding tie; then
    the unit is redone exactly.  Here every column has its inv_s tuned so that x inv_s / Step lands
    within a few binary32 ulps of a tie (both sides and exactly on it), for small, negative, large
    and too-large zero points."""
    progress("quant_act screened quotient next to ties")
    rng = np.random.default_rng(4242)
    T, K = 40, 1024
    mult = np.array([1, 3, 5, -1, -3], np.float64)
    for sp, zero in ((0.037, 128), (0.5, 0), (1.0 / 3.0, 255), (0.0123, -300), (0.21, 4000), (0.21, 4097),
                     (7.3e-3, 77), (1.9990234375, 130)):
        sp = np.float32(sp)
        xk = (rng.integers(8, 129, K) / 16.0)                      # few significand bits: 3 x, 5 x exact in binary16
        m = rng.integers(-zero - 2, 258 - zero, K).astype(np.float64)
        target = (m + 0.5) * np.float64(sp) / xk
        inv_s = target.astype(np.float32)
        for _ in range(3):                                         # 0 .. 3 ulps to either side
            up = rng.random(K) < 0.5
            moved = np.where(up, np.nextafter(inv_s, np.float32(np.inf)), np.nextafter(inv_s, np.float32(-np.inf)))
            inv_s = np.where(rng.random(K) < 0.6, moved, inv_s).astype(np.float32)
        inv_s = np.where(np.abs(inv_s) > 1e-6, inv_s, np.float32(1.0)).astype(np.float32)
        X = (rng.standard_normal((T, K)) * 2).astype(np.float16)
        for r, c in enumerate(mult):
            X[r] = (xk * c).astype(np.float16)
            assert np.array_equal(X[r].astype(np.float64), xk * c)
        check_quant_act(B, orc, X, inv_s, sp, zero)


def test_panel_converters(B):
    progress("K-panel pack / unpack")
    rng = np.random.default_rng(5)
    for rows, K, ld in ((300, 200, 208), (64, 64, 64), (5, 8, 8), (1000, 1040, 1040)):
        m = rng.integers(-128, 128, (rows, ld), dtype=np.int8)
        panels = torch.full((B.aweq_panel_bytes(rows, K),), 0x5a, dtype=torch.int8, device=DEV)
        B.aweq_pack_panels_i8(dev(m), rows, K, ld, panels)
        assert np.array_equal(host(panels), to_panels(m[:, :K]))
        back = torch.full((rows, ld), 0x5a, dtype=torch.int8, device=DEV)
        B.aweq_unpack_panels_i8(panels, rows, K, back, ld)
        assert np.array_equal(host(back)[:, :K], m[:, :K]) and np.all(host(back)[:, K:] == 0x5a)


# ------------------------------------------------------------------------------ stage 4b


def gpu_gemm(B, xq, wq, want_i32=True, deq=None, colsum=True):
    T, K = xq.shape
    N = wq.shape[0]
    out = torch.full((T, N), -7, dtype=torch.int32, device=DEV) if want_i32 else None
    cs = e(N, dtype=torch.int64) if colsum else None
    out_deq, args = None, [None] * 6
    out_dt = B.AWEQ_F32
    if deq is not None:
        out_dt = B.AWEQ_F16 if deq["dtype"] == np.float16 else B.AWEQ_F32
        out_deq = torch.zeros((T, N), dtype=torch.float16 if deq["dtype"] == np.float16 else torch.float32, device=DEV)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    B.aweq_w8a8_gemm(dev(to_panels(xq)), B.AWEQ_I8, T, K, K, None,
                     dev(np.array([deq["step_x"]], np.float32)) if deq else None,
                     dev(np.array([deq["zero_x"]], np.int32)) if deq else None,
                     None, dev(deq["rowsum_x"]) if deq else None, None, dev(to_panels(wq)), N,
                     dev(deq["step_w"]) if deq else None, dev(deq["zero_w"]) if deq else None,
                     int(deq.get("w_group", 0)) if deq else 0, dev(deq["rowsum_w"]) if deq else None, dev(deq["bias"]) if deq and deq["bias"] is not None else None,
                     out, out_deq, out_dt, N, cs, None, status)
    return out, out_deq, cs


@pytest.mark.parametrize("T,N,K", [
    (256, 256, 64),      # exactly one tile, one panel
    (300, 200, 192),     # ragged in both directions, three panels (the ring's prologue only)
    (260, 256, 128),     # two panels
    (512, 512, 512),     # config-1 weight shape
    (1000, 700, 1040),   # K % 64 = 16: zero-filled last panel
    (2048, 1024, 4096),
    (1, 1, 16),          # generic kernel (N % 4 != 0), one partial panel
    (4, 4, 8),           # LDS-DMA kernel, one partial panel
    (700, 2100, 128),    # more than one patch along N
    (1000, 700, 1024),   # ragged in both directions
    (515, 1028, 384),    # six panels, ragged
    (256, 256, 256),     # four panels: one pass of the steady-state loop
    (300, 260, 328),     # K % 64 = 8
    (300, 202, 256),     # N % 4 != 0: falls back to the generic kernel
    (300, 203, 200),     # generic kernel, zero-filled last panel
    (5157, 4100, 512),   # 21 x 17 = 357 tiles on 256 persistent workgroups: second tiles, ragged edges on
                         # both sides, the relaxed wait after interior tiles and the full wait after edge tiles
    (5157, 4100, 320),   # the same with five panels (never relaxed)
    (700, 2304, 4608),   # K >= 2 N with nine tile columns: the 4 x 8 patch shape, ragged on both sides
])
def test_gemm_parity(B, orc, T, N, K):
    progress(f"gemm T={T} N={N} K={K}")
    rng = np.random.default_rng(T + N + K)
    xq = rng.integers(-128, 128, (T, K), dtype=np.int8)
    wq = rng.integers(-128, 128, (N, K), dtype=np.int8)
    xq[0], wq[0] = -128, -128  # extreme accumulator
    out, _, cs = gpu_gemm(B, xq, wq)
    ref = orc.gemm_i8(xq, wq)
    assert np.array_equal(host(out), ref)
    assert np.array_equal(host(cs), ref.astype(np.int64).sum(axis=0))
    # column sums alone (no output written)
    _, _, cs2 = gpu_gemm(B, xq, wq, want_i32=False)
    assert np.array_equal(host(cs2), host(cs))


def test_gemm_largest_contraction_and_extreme_accumulators(B, orc):
    """K = 32768 is the largest contraction the int32 accumulator is guaranteed for: all-(-128) rows
    give 128 * 128 * 32768 = 2^29, mixed signs give -(127 * 128 * 32768); column sums stay exact."""
    progress("gemm K=32768, extreme accumulators")
    rng = np.random.default_rng(8)
    T, N, K = 260, 256, 32768
    xq = rng.integers(-128, 128, (T, K), dtype=np.int8)
    wq = rng.integers(-128, 128, (N, K), dtype=np.int8)
    xq[0], xq[1], wq[0], wq[1] = -128, 127, -128, 127
    out, _, cs = gpu_gemm(B, xq, wq)
    ref = orc.gemm_i8(xq, wq)
    assert ref[0, 0] == 2 ** 29 and ref[1, 0] == -127 * 128 * 32768 and ref[1, 1] == 127 * 127 * 32768
    assert np.array_equal(host(out), ref)
    assert np.array_equal(host(cs), ref.astype(np.int64).sum(axis=0))


@pytest.mark.parametrize("K,N", [(320, 260), (328, 260), (328, 262)])   # ..., zero-filled last panel, generic kernel
@pytest.mark.parametrize("T", [300, 70000])   # one tile per workgroup / two tiles on some (persistent loop)
@pytest.mark.parametrize("odt", [np.float32, np.float16])
def test_gemm_dequant_epilogue(B, orc, odt, K, N, T):
    progress(f"gemm dequant epilogue {odt.__name__} K={K} N={N} T={T}")
    rng = np.random.default_rng(3)
    xq = rng.integers(-128, 128, (T, K), dtype=np.int8)
    wq = rng.integers(-128, 128, (N, K), dtype=np.int8)
    deq = dict(dtype=odt, step_x=0.0123, zero_x=141, step_w=rng.uniform(1e-4, 1e-3, N).astype(np.float32),
               zero_w=rng.integers(90, 170, N).astype(np.int32), bias=rng.standard_normal(N).astype(np.float32),
               rowsum_x=xq.astype(np.int64).sum(axis=1).astype(np.int32), rowsum_w=wq.astype(np.int64).sum(axis=1).astype(np.int32))
    out, out_deq, cs = gpu_gemm(B, xq, wq, deq=deq)
    acc = orc.gemm_i8(xq, wq)
    assert np.array_equal(host(out), acc)            # the raw accumulator written next to the de-quantised output
    assert np.array_equal(host(cs), acc.astype(np.int64).sum(axis=0))
    ref = orc.w8a8_output_direct(xq, wq, deq["step_x"], deq["zero_x"], deq["step_w"], deq["zero_w"], deq["bias"])
    got = host(out_deq).astype(np.float64)
    if odt == np.float32:
        assert np.max(np.abs(got - ref)) <= 1e-6 * np.max(np.abs(ref))
        assert np.array_equal(host(out_deq), ref.astype(np.float32))  # fp64 product rounded once
    else:
        ulp = np.maximum(np.abs(ref), 2.0 ** -14) * 2.0 ** -10
        assert np.all(np.abs(got - ref) <= ulp)


@pytest.mark.parametrize("N", [260, 262])   # the tiled kernel / the generic kernel
def test_gemm_dequant_zero_points_outside_the_code_range(B, orc, N):
    """A slice whose range does not contain 0 has its zero point outside [0, 255] (Eq. 2 does not clamp
    it).  The epilogue must still de-quantise exactly while the integer part fits 32 bits, and says so
    in the status word."""
    progress(f"gemm dequant epilogue, zero points outside [0, 255], N={N}")
    rng = np.random.default_rng(12)
    T, K = 300, 320
    xq = rng.integers(-128, 128, (T, K), dtype=np.int8)
    wq = rng.integers(-128, 128, (N, K), dtype=np.int8)
    zero_w = rng.integers(90, 170, N).astype(np.int32)
    zero_w[[0, 5, 70, 130, N - 1]] = [-40, 300, 1000, -3000, 256]
    deq = dict(dtype=np.float32, step_x=0.0123, zero_x=141, step_w=rng.uniform(1e-4, 1e-3, N).astype(np.float32),
               zero_w=zero_w, bias=rng.standard_normal(N).astype(np.float32),
               rowsum_x=xq.astype(np.int64).sum(axis=1).astype(np.int32), rowsum_w=wq.astype(np.int64).sum(axis=1).astype(np.int32))
    ref = orc.w8a8_output_direct(xq, wq, deq["step_x"], deq["zero_x"], deq["step_w"], deq["zero_w"], deq["bias"])
    for odt in (np.float32, np.float16):
        deq["dtype"] = odt
        T_, K_ = xq.shape
        out_deq = torch.zeros((T_, N), dtype=torch.float16 if odt == np.float16 else torch.float32, device=DEV)
        cs = e(N, dtype=torch.int64)
        status = torch.zeros(1, dtype=torch.int32, device=DEV)
        B.aweq_w8a8_gemm(dev(to_panels(xq)), B.AWEQ_I8, T_, K_, K_, None, dev(np.array([deq["step_x"]], np.float32)),
                         dev(np.array([deq["zero_x"]], np.int32)), None, dev(deq["rowsum_x"]), None, dev(to_panels(wq)), N,
                         dev(deq["step_w"]), dev(deq["zero_w"]), 0, dev(deq["rowsum_w"]), dev(deq["bias"]), None, out_deq,
                         B.AWEQ_F16 if odt == np.float16 else B.AWEQ_F32, N, cs, None, status)
        got = host(out_deq)
        if odt == np.float32:
            assert np.array_equal(got, ref.astype(np.float32))
        else:
            assert np.all(np.abs(got.astype(np.float64) - ref) <= np.maximum(np.abs(ref), 2.0 ** -14) * 2.0 ** -10)
        assert np.array_equal(host(cs), orc.gemm_i8(xq, wq).astype(np.int64).sum(axis=0))
        assert int(host(status)[0]) == B.ST_ZEROPOINT


def test_gemm_column_sums_do_not_depend_on_zero_points(B, orc):
    """colsum_acc is the sum of the accumulator itself.  With an all-positive weight row, a large
    contraction and a zero point far outside [0, 255] the corrected integer of the de-quantisation no
    longer fits 32 bits (the status bit says so); the column sums must still be exact, and equal with
    and without a de-quantised output, in the tiled and in the generic kernel."""
    progress("gemm column sums under wrapping zero points")
    rng = np.random.default_rng(99)
    T, K = 300, 8192
    for N in (260, 262):
        xq = rng.integers(-128, 128, (T, K), dtype=np.int8)
        wq = rng.integers(-128, 128, (N, K), dtype=np.int8)
        wq[3] = 127
        xq[:8] = 127
        zero_w = rng.integers(100, 160, N).astype(np.int32)
        zero_w[3], zero_w[7] = 128 - 4000000, 128 + 3000000      # |Z'w rowsum_x| up to 4e6 * 127 * 8192 >> 2^31
        deq = dict(dtype=np.float32, step_x=0.01, zero_x=133, step_w=rng.uniform(1e-4, 1e-3, N).astype(np.float32),
                   zero_w=zero_w, bias=None, rowsum_x=xq.astype(np.int64).sum(axis=1).astype(np.int32),
                   rowsum_w=wq.astype(np.int64).sum(axis=1).astype(np.int32))
        ref = orc.gemm_i8(xq, wq).astype(np.int64).sum(axis=0)
        for odt in (np.float32, np.float16):
            deq["dtype"] = odt
            _, _, cs_deq = gpu_gemm(B, xq, wq, want_i32=False, deq=deq)
            assert np.array_equal(host(cs_deq), ref), (N, odt)
        _, _, cs_plain = gpu_gemm(B, xq, wq, want_i32=False)
        assert np.array_equal(host(cs_plain), ref)


def test_gemm_dequant_per_tensor_weight_scale(B, orc):
    """w_group = -1: one (Step, Z) for the whole weight (the paper's per-tensor setting, Sec. 3), read from
    index 0 by the epilogue; equal to the per-channel call with that pair repeated."""
    progress("gemm dequant epilogue, per-tensor weight scale")
    rng = np.random.default_rng(17)
    T, K = 300, 320
    for N in (260, 262):
        xq = rng.integers(-128, 128, (T, K), dtype=np.int8)
        wq = rng.integers(-128, 128, (N, K), dtype=np.int8)
        common = dict(dtype=np.float32, step_x=0.0123, zero_x=141, bias=rng.standard_normal(N).astype(np.float32),
                      rowsum_x=xq.astype(np.int64).sum(axis=1).astype(np.int32), rowsum_w=wq.astype(np.int64).sum(axis=1).astype(np.int32))
        one = dict(common, step_w=np.array([3.7e-4], np.float32), zero_w=np.array([119], np.int32), w_group=-1)
        rep = dict(common, step_w=np.full(N, 3.7e-4, np.float32), zero_w=np.full(N, 119, np.int32))
        ref = orc.w8a8_output_direct(xq, wq, 0.0123, 141, rep["step_w"], rep["zero_w"], common["bias"])
        _, got, _ = gpu_gemm(B, xq, wq, want_i32=False, deq=one)
        assert np.array_equal(host(got), ref.astype(np.float32))
        _, got_rep, _ = gpu_gemm(B, xq, wq, want_i32=False, deq=rep)
        assert np.array_equal(host(got_rep), host(got))


def test_gemm_with_activation_quantizer_in_front(B, orc):
    """aweq_w8a8_gemm with FP input runs stage 4a itself."""
    progress("gemm with fused call of stage 4a")
    rng = np.random.default_rng(21)
    T, K, N = 520, 1024, 300
    X, W = make_layer(rng, np.float16, T, K, N)
    sx, sw, s, inv_s, _ = oracle_front(orc, X, W)
    lo, hi, mu = orc.xhat_stats(sx["cmin"], sx["cmax"], sx["csum"], sx["count"], inv_s)
    step, zero, _ = orc.qparams(lo, hi, 8)
    q = orc.quant_weight(orc.fold_weight(W, s), 8, 0)
    wq = orc.pack_codes(q["codes_u"], 8)
    a = orc.quant_act(X, inv_s, step, zero)
    xq, rs, csx = e(B.aweq_panel_bytes(T, K), dtype=torch.int8), e(T, dtype=torch.int32), e(K, dtype=torch.int64)
    out, csa = e(T, N, dtype=torch.int32), e(N, dtype=torch.int64)
    B.aweq_w8a8_gemm(dev(X), B.AWEQ_F16, T, K, K, dev(inv_s), dev(np.array([step], np.float32)),
                     dev(np.array([zero], np.int32)), xq, rs, csx, dev(to_panels(wq)), N, None, None, 0, None, None, out, None,
                     B.AWEQ_F16, N, csa, qa_ws(B, T, K), None)
    assert np.array_equal(from_panels(host(xq), T, K), a["xq"]) and np.array_equal(host(rs), a["rowsum_x"])
    ref = orc.gemm_i8(a["xq"], wq)
    assert np.array_equal(host(out), ref)
    assert np.array_equal(host(csa), orc.colsum_acc_from_colsum_xq(wq, a["colsum_xq"]))


# ------------------------------------------------------------------------------ stage 5


def front_for_bias(orc, dtype, T, K, N, seed):
    rng = np.random.default_rng(seed)
    X, W = make_layer(rng, dtype, T, K, N, outliers=(3, 50))
    sx, sw, s, inv_s, _ = oracle_front(orc, X, W)
    Wh = orc.fold_weight(W, s)
    lo, hi, mu = orc.xhat_stats(sx["cmin"], sx["cmax"], sx["csum"], sx["count"], inv_s)
    return X, Wh, inv_s, lo, hi, mu, rng


@pytest.mark.parametrize("dtype,T,K,N,bias", [(np.float16, 300, 1024, 70, True), (np.float32, 128, 512, 40, False),
                                              (np.float16, 64, 11008, 9, True)])
def test_bias_w8a8_parity(B, orc, dtype, T, K, N, bias):
    progress(f"bias w8a8 {dtype.__name__} T={T} K={K} N={N}")
    X, Wh, inv_s, lo, hi, mu, rng = front_for_bias(orc, dtype, T, K, N, 31)
    step, zero, _ = orc.qparams(lo, hi, 8)
    a = orc.quant_act(X, inv_s, step, zero)
    q = orc.quant_weight(Wh, 8, 0)
    wq = orc.pack_codes(q["codes_u"], 8)
    csa = orc.colsum_acc_from_colsum_xq(wq, a["colsum_xq"])
    b_in = rng.standard_normal(N).astype(np.float32) if bias else None
    d_ref, b_ref = orc.bias_w8a8(Wh, mu, T, csa, a["colsum_xq"], q["rowsum_w"], step, zero, q["step"], q["zero"], b_in)
    delta, bout = e(N, dtype=torch.float32), e(N, dtype=torch.float32)

    def run(enable):
        B.aweq_bias_correct(B.BIAS_W8A8, dev(Wh), dtc(B, Wh), N, K, K, dev(mu), T, dev(csa), dev(a["colsum_xq"]),
                            dev(q["rowsum_w"]), dev(np.array([step], np.float32)), dev(np.array([zero], np.int32)),
                            None, 8, 0, dev(q["step"]), dev(q["zero"]), dev(b_in) if bias else None, delta, bout,
                            enable)
    run(1)
    assert np.max(np.abs(host(delta) - d_ref)) <= 1e-5 * np.max(np.abs(d_ref))
    np.testing.assert_allclose(host(bout), b_ref, rtol=1e-5, atol=1e-5 * np.max(np.abs(d_ref)))
    run(0)
    assert np.array_equal(host(bout), b_in if bias else np.zeros(N, np.float32))
    assert np.max(np.abs(host(delta) - d_ref)) <= 1e-5 * np.max(np.abs(d_ref))


@pytest.mark.parametrize("dtype,K,N,bits,group", [(np.float16, 1024, 50, 4, 128), (np.float16, 1024, 50, 3, 128),
                                                  (np.float16, 11008, 6, 4, 128), (np.float32, 512, 20, 8, 0),
                                                  (np.float16, 512, 20, 3, 0), (np.float16, 512, 20, 4, -1)])
def test_bias_weight_only_parity(B, orc, dtype, K, N, bits, group):
    progress(f"bias weight-only {dtype.__name__} K={K} N={N} b={bits} g={group}")
    X, Wh, inv_s, lo, hi, mu, rng = front_for_bias(orc, dtype, 96, K, N, 41)
    q = orc.quant_weight(Wh, bits, group)
    packed = orc.pack_codes(q["codes_u"], bits).view(np.uint8).reshape(-1)
    b_in = rng.standard_normal(N).astype(np.float32)
    d_ref, b_ref = orc.bias_wonly(Wh, mu, q["codes_u"], group, q["step"], q["zero"], b_in)
    delta, bout = e(N, dtype=torch.float32), e(N, dtype=torch.float32)
    B.aweq_bias_correct(B.BIAS_WEIGHT_ONLY, dev(Wh), dtc(B, Wh), N, K, K, dev(mu), 96, None, None, None, None, None,
                        dev(to_panels(packed.view(np.int8).reshape(N, K)) if bits == 8 and group <= 0 else packed), bits, group, dev(q["step"].reshape(-1)), dev(q["zero"].reshape(-1)), dev(b_in),
                        delta, bout, 1)
    assert np.max(np.abs(host(delta) - d_ref)) <= 1e-5 * np.max(np.abs(d_ref))
    np.testing.assert_allclose(host(bout), b_ref, rtol=1e-5, atol=1e-5 * np.max(np.abs(d_ref)))


# --------------------------------------------------------------------------- end to end


@pytest.mark.parametrize("cfg,T,shapes", [
    (1, 2048, [("fc", 512, 512)]),                                        # config 1 at full size
    (2, 1536, [("q_proj", 384, 512), ("fc1", 1024, 512), ("fc2", 512, 1024)]),
    (3, 1536, [("q_proj", 512, 512), ("gate_proj", 1376, 512), ("down_proj", 512, 1376)]),
])
def test_end_to_end_unforced(B, orc, cfg, T, shapes):
    """The whole path on the GPU with no teacher forcing, against the whole path in the oracle:
    ranges exact, scales to 1e-5, codes equal except where a last-ulp difference of s moved a
    value across a rounding boundary (then off by one), bias correction to 1e-5 of its norm."""
    from paper_2311_01305_amd import pipeline, synth
    wl = synth.WORKLOADS[cfg]
    tdt = torch.float16 if wl.dtype == "f16" else torch.float32
    for li, (name, N, K) in enumerate(shapes):
        progress(f"end-to-end cfg{cfg} {name} N={N} K={K}")
        seed = synth.layer_seed(cfg, li)
        W = synth.make_weight_np(seed, N, K, wl.dtype)
        X = synth.make_act_np(seed, T, K, wl)
        b = synth.make_bias_np(seed, N, wl.has_bias)
        buf = pipeline.LayerBuffers(T, K, N, tdt, want_out_i32=True, want_out_deq=True)
        t = pipeline.calibrate_layer(dev(X), dev(W), dev(b) if b is not None else None, buf)
        sx, sw, s, inv_s, _ = oracle_front(orc, X, W)
        assert np.array_equal(host(t["xmin"]), sx["cmin"]) and np.array_equal(host(t["xmax"]), sx["cmax"])
        assert np.array_equal(host(t["wmin"]), sw["cmin"]) and np.array_equal(host(t["wmax"]), sw["cmax"])
        np.testing.assert_allclose(host(t["s"]), s, rtol=1e-5)
        Wh = orc.fold_weight(W, s)
        lo, hi, mu = orc.xhat_stats(sx["cmin"], sx["cmax"], sx["csum"], sx["count"], inv_s)
        step, zero, _ = orc.qparams(lo, hi, 8)
        np.testing.assert_allclose(host(t["act_step"])[0], step, rtol=1e-5)
        q = orc.quant_weight(Wh, 8, 0)
        codes = from_panels(host(t["codes"]), N, K).astype(np.int32)
        ref_codes = orc.pack_codes(q["codes_u"], 8).astype(np.int32)
        diff = np.abs(codes - ref_codes)
        assert diff.max() <= 1 and np.mean(diff != 0) < 1e-3
        a = orc.quant_act(X, inv_s, step, zero)
        gxq = from_panels(host(t["xq"]), T, K)
        dxq = np.abs(gxq.astype(np.int32) - a["xq"].astype(np.int32))
        assert dxq.max() <= 1 and np.mean(dxq != 0) < 1e-3
        # the GPU's own chain is self-consistent: its GEMM output is exact for its own codes
        acc = orc.gemm_i8(gxq, from_panels(host(t["codes"]), N, K))
        assert np.array_equal(host(t["out_i32"]), acc)
        wq = orc.pack_codes(q["codes_u"], 8)
        d_ref, b_ref = orc.bias_w8a8(Wh, mu, T, orc.colsum_acc_from_colsum_xq(wq, a["colsum_xq"]), a["colsum_xq"],
                                     q["rowsum_w"], step, zero, q["step"], q["zero"], b)
        # post-condition on the GPU's own outputs: corrected mean output error vanishes
        Xh = orc.fold_act(X, host(t["inv_s"])).astype(np.float64)
        y_fp = Xh @ host(t["W_hat"]).astype(np.float64).T
        y_q = orc.w8a8_output_direct(gxq, from_panels(host(t["codes"]), N, K), host(t["act_step"])[0],
                                     int(host(t["act_zero"])[0]), host(t["step_w"]), host(t["zero_w"]), None)
        resid = (y_q + host(t["delta"]).astype(np.float64) - y_fp).mean(axis=0)
        assert np.max(np.abs(resid)) <= 2e-5 * np.max(np.abs(d_ref)) + 1e-6 * np.max(np.abs(y_fp.mean(axis=0)))
        assert int(host(t["status"])[0]) == 0


@pytest.mark.parametrize("dtype,T,K,N,has_bias", [(np.float16, 700, 1032, 260, True), (np.float32, 300, 512, 64, False)])
def test_calibration_without_the_forward(B, orc, dtype, T, K, N, has_bias):
    """Bias correction needs only the sum over tokens of the accumulator, and that is the weight
    codes times the column sums of the activation codes (exact integers): the layer calibrated with
    the GEMM skipped and a sums-only activation quantizer must give bit-identical delta and bias."""
    from paper_2311_01305_amd import pipeline
    progress(f"calibration without the forward {dtype.__name__} T={T} K={K} N={N}")
    rng = np.random.default_rng(T + K)
    X, W = make_layer(rng, dtype, T, K, N, outliers=(3, 60))
    b = (rng.standard_normal(N) * 0.02).astype(np.float32) if has_bias else None
    tdt = torch.float16 if dtype == np.float16 else torch.float32
    res = []
    for forward in (True, False):
        buf = pipeline.LayerBuffers(T, K, N, tdt, want_out_i32=forward, want_out_deq=False)
        t = pipeline.calibrate_layer(dev(X), dev(W), dev(b) if b is not None else None, buf, forward=forward)
        res.append({k: host(t[k]) for k in ("delta", "bias_out", "colsum_xq", "rowsum_w", "codes", "mu_xhat", "act_step",
                                            "act_zero", "step_w", "zero_w", "W_hat", "status")})
    full, lean = res
    for k in ("delta", "bias_out", "colsum_xq"):
        assert np.array_equal(full[k].view(np.uint8), lean[k].view(np.uint8)), k
    assert int(lean["status"][0]) == int(full["status"][0])
    # and against the oracle's identity route
    wq = from_panels(lean["codes"], N, K)
    ca = orc.colsum_acc_from_colsum_xq(wq, lean["colsum_xq"])
    d_ref, b_ref = orc.bias_w8a8(lean["W_hat"], lean["mu_xhat"], T, ca, lean["colsum_xq"], lean["rowsum_w"], lean["act_step"][0],
                                 int(lean["act_zero"][0]), lean["step_w"], lean["zero_w"], b)
    assert np.max(np.abs(lean["delta"] - d_ref)) <= 1e-5 * np.max(np.abs(d_ref))
    np.testing.assert_allclose(lean["bias_out"], b_ref, rtol=1e-5, atol=1e-5 * np.max(np.abs(d_ref)))
    # the sums-only activation quantizer alone
    rs, cs = e(T, dtype=torch.int32), e(K, dtype=torch.int64)
    B.aweq_quant_act(dev(X), dtc(B, X), T, K, K, dev(host(t["inv_s"])), t["act_step"], t["act_zero"], None, rs, cs, qa_ws(B, T, K))
    a = orc.quant_act(X, host(t["inv_s"]), lean["act_step"][0], int(lean["act_zero"][0]))
    assert np.array_equal(host(rs), a["rowsum_x"]) and np.array_equal(host(cs), a["colsum_xq"])
