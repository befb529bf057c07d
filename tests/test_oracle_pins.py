"""Pins for the CPU oracle: hand-worked examples, closed forms, invariants, brute force
and special cases that reduce to library routines.  No GPU."""
from fractions import Fraction

import numpy as np
import pytest

from conftest import read_golden

# ---------------------------------------------------------------- binary16 conversion


def test_h2f_exhaustive_vs_numpy(orc):
    bits = np.arange(65536, dtype=np.uint16)
    ours = orc.h2f(bits)
    ref = bits.view(np.float16).astype(np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(ours), nan)
    assert np.array_equal(ours[~nan].view(np.uint32), ref[~nan].view(np.uint32))


def test_f2h_vs_numpy_random_and_boundaries(orc):
    rng = np.random.default_rng(1)
    # every half value, the midpoints between neighbours, and values just off the midpoints
    h = np.arange(0x7c00, dtype=np.uint16).view(np.float16).astype(np.float64)
    mid = (h[:-1] + h[1:]) / 2
    cand = np.concatenate([h, mid, np.nextafter(mid.astype(np.float32), np.float32(np.inf)).astype(np.float64),
                           np.nextafter(mid.astype(np.float32), np.float32(-np.inf)).astype(np.float64),
                           [65504.0, 65519.99, 65520.0, 65536.0, 1e30, 2.0 ** -25, 2.0 ** -24, 3e-8, 0.0],
                           rng.standard_normal(200000) * 10.0 ** rng.uniform(-9, 5, 200000)])
    cand = np.concatenate([cand, -cand]).astype(np.float32)
    ours = orc.f2h(cand)
    with np.errstate(over="ignore"):
        ref = cand.astype(np.float16).view(np.uint16)
    assert np.array_equal(ours, ref)


# ---------------------------------------------------------------------- stage 1: statistics


def test_stats_golden(orc):
    g = read_golden("stats_3x3.txt")
    for dt in (np.float32, np.float16):
        M = np.array(g["m"], dt).reshape(3, 3)
        st = orc.col_stats(M)
        assert st["cmin"].tolist() == g["cmin"]
        assert st["cmax"].tolist() == g["cmax"]
        assert st["csum"].tolist() == g["csum"]
        assert st["count"] == 3 and st["status"] == 0
        r, R, p = orc.ranges(st["cmin"], st["cmax"])
        assert r.tolist() == g["r"]
        assert float(R) == g["R"][0]
        np.testing.assert_allclose(p, np.array(g["p"]), rtol=1e-7)


@pytest.mark.parametrize("dt", [np.float32, np.float16])
def test_stats_reduce_to_numpy_and_permutation_invariance(orc, dt):
    rng = np.random.default_rng(2)
    M = (rng.standard_normal((257, 71)) * 3).astype(dt)
    st = orc.col_stats(M)
    assert np.array_equal(st["cmin"], M.min(axis=0).astype(np.float32))
    assert np.array_equal(st["cmax"], M.max(axis=0).astype(np.float32))
    np.testing.assert_allclose(st["csum"], M.astype(np.float64).sum(axis=0), rtol=1e-13, atol=1e-12)
    perm = rng.permutation(M.shape[0])
    st2 = orc.col_stats(M[perm])
    assert np.array_equal(st["cmin"], st2["cmin"]) and np.array_equal(st["cmax"], st2["cmax"])
    # a transposed-operand mistake would swap the two axes
    assert st["cmin"].shape == (71,)


def test_stats_accumulate_equals_one_pass(orc):
    rng = np.random.default_rng(3)
    M = rng.standard_normal((100, 16)).astype(np.float32)
    full = orc.col_stats(M)
    part = orc.col_stats(M[:37])
    part = orc.col_stats(M[37:], prev=part)
    assert np.array_equal(full["cmin"], part["cmin"]) and np.array_equal(full["cmax"], part["cmax"])
    assert part["count"] == 100
    np.testing.assert_allclose(full["csum"], part["csum"], rtol=1e-14, atol=1e-13)


def test_stats_flags_nonfinite(orc):
    M = np.ones((4, 4), np.float32)
    M[2, 1] = np.inf
    assert orc.col_stats(M)["status"] & orc.ST_NONFINITE


def test_p_bounds_and_max(orc):
    rng = np.random.default_rng(4)
    cmin = -np.abs(rng.standard_normal(50)).astype(np.float32)
    cmax = np.abs(rng.standard_normal(50)).astype(np.float32)
    r, R, p = orc.ranges(cmin, cmax)
    assert np.all(p >= 0) and np.all(p <= 1)
    assert float(R) == float(np.float32(cmax.max()) - np.float32(cmin.min()))
    # p reaches 1 exactly when one channel holds both global extremes
    cmin[7], cmax[7] = -10.0, 10.0
    r, R, p = orc.ranges(cmin, cmax)
    assert p[7] == 1.0 and np.count_nonzero(p == 1.0) == 1


# -------------------------------------------------------------------- stage 2: equalization


def test_scale_golden(orc):
    g = read_golden("equalization_scale.txt")
    r_x, r_w = np.array(g["r_x"], np.float32), np.array(g["r_w"], np.float32)
    s, inv_s, st = orc.scales(r_x, r_w)
    assert s.tolist() == g["s"] and st == 0
    assert (r_x / s).tolist() == g["equalised_range"]
    assert (s * r_w).tolist() == g["equalised_range"]
    obj = lambda sv: float(np.max(r_x / sv) * np.max(sv * r_w))
    assert obj(np.ones(3, np.float32)) == g["objective_before"][0]
    assert obj(s) == g["objective_after"][0]
    assert np.array_equal(inv_s, np.float32(1.0) / s)


def test_scale_closed_forms(orc):
    rng = np.random.default_rng(5)
    K = 64
    r_x = rng.uniform(0.1, 300.0, K).astype(np.float32)
    r_w = rng.uniform(0.01, 2.0, K).astype(np.float32)
    s, inv_s, st = orc.scales(r_x, r_w)
    assert st == 0
    # equalised ranges coincide channel by channel (assumption before Eq. 10)
    np.testing.assert_allclose(r_x.astype(np.float64) / s, s.astype(np.float64) * r_w, rtol=3e-7)
    # fp64 closed form s = sqrt(r_x / r_w)
    np.testing.assert_allclose(s, np.sqrt(r_x.astype(np.float64) / r_w.astype(np.float64)), rtol=1e-7)
    # Eq. 8: the objective attains its lower bound max_i r_x r_w
    obj = np.max(r_x.astype(np.float64) / s) * np.max(s.astype(np.float64) * r_w)
    np.testing.assert_allclose(obj, np.max(r_x.astype(np.float64) * r_w), rtol=1e-6)
    # r_x = r_w  =>  s = 1 ; scaling X by c scales s by sqrt(c)
    s1, _, _ = orc.scales(r_w, r_w)
    assert np.all(s1 == 1.0)
    s4, _, _ = orc.scales(r_x * np.float32(4.0), r_w)
    np.testing.assert_allclose(s4, 2.0 * s, rtol=2e-7)
    # AWE off
    s0, i0, _ = orc.scales(r_x, r_w, enable_awe=False)
    assert np.all(s0 == 1.0) and np.all(i0 == 1.0)


def test_scale_never_beaten_by_brute_force(orc):
    rng = np.random.default_rng(6)
    for K in (2, 3, 5, 8):
        r_x = rng.uniform(0.5, 50.0, K).astype(np.float32)
        r_w = rng.uniform(0.05, 2.0, K).astype(np.float32)
        s, _, _ = orc.scales(r_x, r_w)
        best = np.max(r_x / s) * np.max(s * r_w)
        trial = np.exp(rng.uniform(-4, 4, (20000, K)))
        objs = np.max(r_x[None] / trial, axis=1) * np.max(trial * r_w[None], axis=1)
        assert objs.min() >= best * (1 - 1e-6)


def test_scale_guards(orc):
    r_x = np.array([0.0, 1.0, 1e12, 1e-12 + 1e-5, 2.0], np.float32)
    r_w = np.array([1.0, 0.0, 1e-4, 1e4, 2.0], np.float32)
    s, inv_s, st = orc.scales(r_x, r_w)
    assert st & orc.ST_SCALEGUARD
    assert s[0] == 1.0 and s[1] == 1.0  # degenerate channel ranges
    assert s[2] == np.float32(1e4) and s[3] == np.float32(1e-4)  # clamped
    assert s[4] == 1.0


def test_absmax_scale_golden_and_closed_forms(orc):
    """The abs-max variant of the difficulty (the definition the method replaces): channel quantity
    max |.| instead of max - min, same closed form."""
    g = read_golden("absmax_scale.txt")
    f = lambda k: np.array(g[k], np.float32)
    m_x, m_w = orc.channel_absmax(f("x_min"), f("x_max")), orc.channel_absmax(f("w_min"), f("w_max"))
    assert m_x.tolist() == g["m_x"] and m_w.tolist() == g["m_w"]
    s, inv_s, st = orc.scales(m_x, m_w)
    assert s.tolist() == g["s"] and st == 0
    assert (m_x / s).tolist() == g["equalised_absmax"] and (s * m_w).tolist() == g["equalised_absmax"]
    # brute force on data: m = max |x| over the rows of each column; a dropped abs or a min/max swap fails
    rng = np.random.default_rng(77)
    X = (rng.standard_normal((200, 24)) * rng.uniform(0.1, 30, 24) + rng.uniform(-5, 5, 24)).astype(np.float16)
    sx = orc.col_stats(X)
    m = orc.channel_absmax(sx["cmin"], sx["cmax"])
    assert np.array_equal(m, np.abs(X.astype(np.float32)).max(axis=0))
    # a channel that is symmetric about zero has m = r / 2, so both definitions give the same scale there
    r_x, _, _ = orc.ranges(np.float32([-4, -2]), np.float32([4, 2]))
    r_w, _, _ = orc.ranges(np.float32([-0.5, -1]), np.float32([0.5, 1]))
    sr, _, _ = orc.scales(r_x, r_w)
    sm, _, _ = orc.scales(orc.channel_absmax(np.float32([-4, -2]), np.float32([4, 2])),
                          orc.channel_absmax(np.float32([-0.5, -1]), np.float32([0.5, 1])))
    assert np.array_equal(sr, sm)
    # and they differ for a shifted channel: range 2 around 10 has m = 11
    assert orc.channel_absmax(np.float32([9]), np.float32([11]))[0] == 11.0


def test_fold_rounds_in_two_steps(orc):
    """The folded binary16 weight is the fp32 product rounded to binary16 (Sec. 3.1, Eq. 3, with
    the model stored as FP16, Sec. 2): two roundings.  Special case that reduces to a library
    routine: numpy's float32 multiply followed by its float16 cast.  The inputs are pairs found
    by search for which rounding the exact product once gives the other binary16 neighbour, so
    the pin tells the two readings apart."""
    # a searched pair where the two routes differ, so that the pin can tell them apart
    rng = np.random.default_rng(5)
    wv = rng.uniform(0.5, 1.0, 200000).astype(np.float16)
    sv = rng.uniform(16.0, 32.0, wv.size).astype(np.float32)
    two = (wv.astype(np.float32) * sv).astype(np.float16)
    one = (wv.astype(np.float64) * sv.astype(np.float64)).astype(np.float16)
    d = np.nonzero(one != two)[0]
    assert d.size > 0
    got = np.array([orc.fold_weight(np.array([[wv[i]]], np.float16), np.array([sv[i]], np.float32))[0, 0] for i in d[:20]])
    assert np.array_equal(got.view(np.uint16), two[d[:20]].view(np.uint16))
    assert not np.array_equal(got.view(np.uint16), one[d[:20]].view(np.uint16))


@pytest.mark.parametrize("dt,tol", [(np.float32, 2e-6), (np.float16, 2e-3)])
def test_fold_leaves_product_unchanged(orc, dt, tol):
    """Eq. 3: (X diag(s)^-1)(diag(s) W) = X W."""
    rng = np.random.default_rng(7)
    T, K, N = 33, 48, 17
    X = rng.standard_normal((T, K)).astype(dt)
    X[:, 5] *= 40
    W = (rng.standard_normal((N, K)) * 0.02).astype(dt)
    sx, sw = orc.col_stats(X), orc.col_stats(W, want_sum=False)
    r_x, _, _ = orc.ranges(sx["cmin"], sx["cmax"])
    r_w, _, _ = orc.ranges(sw["cmin"], sw["cmax"])
    s, inv_s, _ = orc.scales(r_x, r_w)
    Wh = orc.fold_weight(W, s)
    Xh = orc.fold_act(X, inv_s)
    assert Wh.dtype == dt and Xh.dtype == np.float32
    y0 = X.astype(np.float64) @ W.astype(np.float64).T
    y1 = Xh.astype(np.float64) @ Wh.astype(np.float64).T
    assert np.max(np.abs(y1 - y0)) <= tol * np.max(np.abs(y0))
    # the fold multiplies column k (not row n): scaling pattern check on a rank-1 probe
    ones = np.ones((3, K), dt)
    assert np.array_equal(orc.fold_weight(ones, s)[1].astype(np.float32), s.astype(dt).astype(np.float32))
    # equalised channel ranges are equal (what Eq. 10 is built to achieve)
    rxh = Xh.max(axis=0) - Xh.min(axis=0)
    rwh = Wh.astype(np.float32).max(axis=0) - Wh.astype(np.float32).min(axis=0)
    np.testing.assert_allclose(rxh, rwh, rtol=5e-3 if dt == np.float16 else 1e-5)


def test_xhat_stats_equal_brute_force(orc):
    rng = np.random.default_rng(8)
    X = rng.standard_normal((200, 24)).astype(np.float16)
    X[:, 3] *= 30
    inv_s = rng.uniform(0.05, 3.0, 24).astype(np.float32)
    st = orc.col_stats(X)
    lo, hi, mu = orc.xhat_stats(st["cmin"], st["cmax"], st["csum"], st["count"], inv_s)
    Xh = orc.fold_act(X, inv_s)
    assert lo == Xh.min() and hi == Xh.max()  # exact: rounding is monotone
    np.testing.assert_allclose(mu, Xh.astype(np.float64).mean(axis=0), rtol=2e-6, atol=1e-7)


# ------------------------------------------------------------------------ stage 3: quantizer


@pytest.mark.parametrize("name", ["quantizer_b3.txt", "quantizer_b8.txt"])
def test_quantizer_golden(orc, name):
    g = read_golden(name)
    x = np.array(g["x"], np.float32)
    bits = int(g["bits"][0])
    step, zero, st = orc.qparams(x.min(), x.max(), bits)
    assert float(step) == g["step"][0] and zero == int(g["zero"][0]) and st == 0
    u, st = orc.quant_values(x, step, zero, bits)
    assert u.tolist() == [int(v) for v in g["codes"]] and st == 0
    assert orc.dequant_values(u, step, zero).tolist() == g["dequant"]
    if "outside_x" in g:
        u2, _ = orc.quant_values(np.array(g["outside_x"], np.float32), step, zero, bits)
        assert u2.tolist() == [int(v) for v in g["outside_codes"]]
    # the same numbers through the weight quantizer (one row) and the storage format
    q = orc.quant_weight(x[None, :].copy(), bits, 0) if x.size % 8 == 0 else None
    if q is not None:
        assert q["codes_u"][0].tolist() == [int(v) for v in g["codes"]]
        assert float(q["step"][0]) == g["step"][0] and int(q["zero"][0]) == int(g["zero"][0])
    if "stored" in g:
        packed = orc.pack_codes(u.astype(np.uint8)[None, :], 8)
        assert packed[0].tolist() == [int(v) for v in g["stored"]]


def test_quantizer_big_quotients_golden(orc):
    """Quotients at and beyond 2^24 and 2^30 (Eq. 1 with a Step / Z that do not come from the data):
    the flag is raised from |round(x / Step)| >= 2^24 on, the rounded quotient saturates at +-2^30
    before Z is added, the sum is an exact integer sum, then the clamp."""
    g = read_golden("quantizer_bigquot.txt")
    step, bits = np.float32(g["step"][0]), int(g["bits"][0])
    for case in "abcd":
        zero = int(g[case + "_zero"][0])
        x = np.array(g[case + "_x"], np.float32)
        u, st = orc.quant_values(x, step, zero, bits)
        assert u.tolist() == [int(v) for v in g[case + "_codes"]], case
        if case + "_flag" in g:
            for xi, fl in zip(x, g[case + "_flag"]):
                _, st1 = orc.quant_values(np.array([xi], np.float32), step, zero, bits)
                assert bool(st1 & orc.ST_BIGQUOT) == bool(fl), (case, xi)
    # the same through the activation quantizer (its status word and sums), binary32 input
    X = np.array([[16777216.0, 3.0, -2.0, 0.0, 1.0, 2.0, 4.0, 5.0]], np.float32)
    a = orc.quant_act(X, np.ones(8, np.float32), 1.0, 100 - 2 ** 24)
    assert a["status"] & orc.ST_BIGQUOT and a["xq"][0, 0] == 100 - 128 and np.all(a["xq"][0, 1:] == -128)
    a = orc.quant_act(X / np.float32(2), np.ones(8, np.float32), 1.0, 100 - 2 ** 24)
    assert not a["status"] & orc.ST_BIGQUOT
    # a Step whose quotient only just reaches 2^24 after the rounding of the division still flags:
    # x / Step = 2^24 - 0.5 rounds (ties to even) to 2^24 in binary32
    u, st = orc.quant_values(np.array([16777215.5 * 3.0], np.float64).astype(np.float32), np.float32(3.0), 0, 8)
    assert st & orc.ST_BIGQUOT


@pytest.mark.parametrize("bits", [8, 4, 3])
def test_quantizer_invariants(orc, bits):
    rng = np.random.default_rng(9 + bits)
    for trial in range(20):
        x = (rng.standard_normal(512) * 10.0 ** rng.uniform(-3, 2)).astype(np.float32) + np.float32(rng.uniform(-1, 1))
        step, zero, st = orc.qparams(x.min(), x.max(), bits)
        u, st2 = orc.quant_values(x, step, zero, bits)
        assert st == 0 and st2 == 0
        assert u.min() >= 0 and u.max() <= 2 ** bits - 1
        assert u[np.argmin(x)] == 0  # lo -> code 0
        xd = orc.dequant_values(u, step, zero)
        # |x - dequant| <= Step/2 inside the range, in exact rational arithmetic (+ fp32 rounding slack)
        S = Fraction(float(step))
        worst = max(abs(Fraction(float(a)) - Fraction(int(c) - zero) * S) for a, c in zip(x[:64], u[:64]))
        assert worst <= S / 2 * (1 + Fraction(1, 2 ** 18)) + abs(Fraction(float(x.max()))) * Fraction(1, 2 ** 22)
        assert np.max(np.abs(x - xd)) <= float(step) * 0.5 * (1 + 1e-5) + 1e-6 * np.abs(x).max()
        # power-of-two scaling: identical codes, Step scaled
        step2, zero2, _ = orc.qparams(x.min() * 8, x.max() * 8, bits)
        u2, _ = orc.quant_values(x * np.float32(8), step2, zero2, bits)
        assert step2 == step * 8 and zero2 == zero and np.array_equal(u, u2)
        # re-quantising the de-quantised values with the same (Step, Z) is the identity
        u3, _ = orc.quant_values(xd, step, zero, bits)
        assert np.array_equal(u3, u)


def test_quantizer_degenerate_slice(orc):
    step, zero, st = orc.qparams(0.3, 0.3, 4)
    assert step == 1.0 and zero == 0 and st & orc.ST_DEGENERATE
    u, _ = orc.quant_values(np.array([0.3], np.float32), step, zero, 4)
    assert u.tolist() == [0]
    z = orc.quant_weight(np.zeros((2, 16), np.float16), 8, 0)
    assert np.all(z["codes_u"] == 0) and np.all(z["step"] == 1.0) and np.all(z["zero"] == 0)
    assert z["status"] & orc.ST_DEGENERATE


def test_quantizer_loose_vs_library_fake_quant(orc):
    """A textbook affine quantizer from a library: conventions differ in the last ulp
    (reciprocal multiply, rounding), so only a loose agreement is asked."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(10)
    x = rng.standard_normal(100000).astype(np.float32)
    step, zero, _ = orc.qparams(x.min(), x.max(), 8)
    u, _ = orc.quant_values(x, step, zero, 8)
    xd = orc.dequant_values(u, step, zero)
    ref = torch.fake_quantize_per_tensor_affine(torch.from_numpy(x), float(step), int(zero), 0, 255).numpy()
    off = np.abs(ref - xd) / float(step)
    assert np.mean(off < 0.5) >= 0.9999 and off.max() <= 1.0 + 1e-3


@pytest.mark.parametrize("bits,group", [(8, 0), (4, 128), (3, 128), (4, 32), (8, -1), (4, 0)])
def test_quant_weight_matches_slicewise_brute_force(orc, bits, group):
    rng = np.random.default_rng(11)
    N, K = 6, 256
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    q = orc.quant_weight(W, bits, group)
    Wf = W.astype(np.float32)
    g = K if group == 0 else (group if group > 0 else None)
    if g is None:
        slices = [(slice(0, N), slice(0, K), 0)]
    else:
        slices = [(slice(n, n + 1), slice(j * g, (j + 1) * g), n * (K // g) + j) for n in range(N) for j in range(K // g)]
    step, zero = q["step"].reshape(-1), q["zero"].reshape(-1)
    for rs, cs, pi in slices:
        v = Wf[rs, cs].reshape(-1)
        sp, z, _ = orc.qparams(v.min(), v.max(), bits)
        assert sp == step[pi] and z == zero[pi]
        u, _ = orc.quant_values(v, sp, z, bits)
        assert np.array_equal(u, q["codes_u"][rs, cs].reshape(-1))
    if bits == 8:
        assert np.array_equal(q["rowsum_w"], (q["codes_u"].astype(np.int64) - 128).sum(axis=1))
    Wt = orc.dequant_weight(q["codes_u"], group, q["step"], q["zero"])
    rep = np.repeat(q["step"], g, axis=1) if group > 0 else (q["step"][:, None] if group == 0 else q["step"][0])
    assert np.all(np.abs(Wt - Wf) <= rep * 0.5 * (1 + 1e-5) + 1e-9)


def test_pack_formats(orc):
    # 3-bit: the eight codes 0..7 in order are the 24-bit word 0xFAC688, little-endian bytes
    c = np.arange(8, dtype=np.uint8)[None, :]
    assert orc.pack_codes(c, 3).reshape(-1).tolist() == [0x88, 0xC6, 0xFA]
    # 4-bit: even k in the low nibble
    assert orc.pack_codes(np.array([[1, 2, 15, 0, 7, 8, 3, 12]], np.uint8), 4).reshape(-1).tolist() == [0x21, 0x0F, 0x87, 0xC3]
    # 8-bit: code - 128 as int8
    assert orc.pack_codes(np.array([[0, 128, 255, 127, 1, 2, 3, 4]], np.uint8), 8).reshape(-1).tolist() == [-128, 0, 127, -1, -127, -126, -125, -124]
    rng = np.random.default_rng(12)
    for bits in (8, 4, 3):
        codes = rng.integers(0, 2 ** bits, (5, 64), dtype=np.uint8)
        # every code value at every position of the 8-code period
        for pos in range(8):
            codes[0, pos::8][: 2 ** bits] = np.arange(2 ** bits)[: codes[0, pos::8].size]
        packed = orc.pack_codes(codes, bits)
        assert packed.size == 5 * 64 * bits // 8
        assert np.array_equal(orc.unpack_codes(packed, 5, 64, bits), codes)


# -------------------------------------------------------------------------- stage 4: W8A8


def test_quant_act_matches_elementwise_and_sums(orc):
    rng = np.random.default_rng(13)
    T, K = 50, 40
    X = rng.standard_normal((T, K)).astype(np.float16)
    X[:, 11] *= 25
    inv_s = rng.uniform(0.1, 2.0, K).astype(np.float32)
    Xh = orc.fold_act(X, inv_s)
    step, zero, _ = orc.qparams(Xh.min(), Xh.max(), 8)
    a = orc.quant_act(X, inv_s, step, zero)
    u, _ = orc.quant_values(Xh.reshape(-1), step, zero, 8)
    assert np.array_equal(a["xq"].astype(np.int32).reshape(-1), u - 128)
    assert np.array_equal(a["rowsum_x"], a["xq"].astype(np.int64).sum(axis=1))
    assert np.array_equal(a["colsum_xq"], a["xq"].astype(np.int64).sum(axis=0))
    assert a["xq"].min() == -128 and a["xq"].max() == 127  # the tensor extremes hit both ends


def test_gemm_reduces_to_integer_matmul(orc):
    rng = np.random.default_rng(14)
    T, N, K = 19, 23, 64
    xq = rng.integers(-128, 128, (T, K), dtype=np.int8)
    wq = rng.integers(-128, 128, (N, K), dtype=np.int8)
    acc = orc.gemm_i8(xq, wq)
    assert np.array_equal(acc.astype(np.int64), xq.astype(np.int64) @ wq.astype(np.int64).T)
    # extreme operands: -128 * -128 * K
    acc = orc.gemm_i8(np.full((2, 64), -128, np.int8), np.full((3, 64), -128, np.int8))
    assert np.all(acc == 128 * 128 * 64)
    cs = xq.astype(np.int64).sum(axis=0)
    assert np.array_equal(orc.colsum_acc_from_colsum_xq(wq, cs), orc.gemm_i8(xq, wq).astype(np.int64).sum(axis=0))


def test_dequant_output_direct_equals_expanded(orc):
    rng = np.random.default_rng(15)
    T, N, K = 9, 7, 32
    xq = rng.integers(-128, 128, (T, K), dtype=np.int8)
    wq = rng.integers(-128, 128, (N, K), dtype=np.int8)
    step_w = rng.uniform(1e-4, 1e-3, N).astype(np.float32)
    zero_w = rng.integers(90, 170, N).astype(np.int32)
    bias = rng.standard_normal(N).astype(np.float32)
    acc = orc.gemm_i8(xq, wq)
    rs_x = xq.astype(np.int64).sum(axis=1).astype(np.int32)
    rs_w = wq.astype(np.int64).sum(axis=1).astype(np.int32)
    d = orc.w8a8_output_direct(xq, wq, 0.037, 141, step_w, zero_w, bias)
    e, integer = orc.w8a8_output_expanded(acc, rs_x, rs_w, K, 0.037, 141, step_w, zero_w, bias)
    assert np.array_equal(d, e)
    ref_int = (xq.astype(np.int64) - 13)[:, None, :] * (wq.astype(np.int64)[None] - (zero_w.astype(np.int64) - 128)[None, :, None])
    assert np.array_equal(integer, ref_int.sum(axis=2))
    # real-valued meaning: y~ = x~ . w~ + b with the de-quantised operands
    xd = (xq.astype(np.float64) - 13) * np.float64(np.float32(0.037))
    wd = (wq.astype(np.float64) - (zero_w - 128)[:, None]) * step_w.astype(np.float64)[:, None]
    np.testing.assert_allclose(d, xd @ wd.T + bias, rtol=1e-12, atol=1e-12)


# ------------------------------------------------------------------ stage 5: bias correction


def test_bias_weight_only_golden(orc):
    g = read_golden("bias_weight_only.txt")
    Wh = np.array(g["w_hat"], np.float32)[None, :]
    X = np.array(g["x"], np.float32).reshape(2, 4)
    # K = 4 here: quantise the row through the scalar quantizer
    step, zero, _ = orc.qparams(Wh.min(), Wh.max(), 3)
    u, _ = orc.quant_values(Wh.reshape(-1), step, zero, 3)
    assert u.tolist() == [int(v) for v in g["codes"]]
    codes = u.astype(np.uint8)[None, :]
    Wt = orc.dequant_weight(codes, 0, np.array([step], np.float32), np.array([zero], np.int32))
    ones = np.ones(4, np.float32)
    bias_in = np.array(g["bias_in"], np.float32)
    d_lit, b_lit = orc.bias_literal_wonly(X, ones, Wh, Wt, bias_in)
    mu = X.mean(axis=0).astype(np.float32)
    d_id, b_id = orc.bias_wonly(Wh, mu, codes, 0, np.array([step], np.float32), np.array([zero], np.int32), bias_in)
    assert abs(d_lit[0] - g["delta"][0]) < 1e-6 and abs(d_id[0] - g["delta"][0]) < 1e-6
    assert abs(b_lit[0] - g["bias_out"][0]) < 1e-6 and abs(b_id[0] - g["bias_out"][0]) < 1e-6


def test_bias_w8a8_golden(orc):
    g = read_golden("bias_w8a8.txt")
    X = np.array(g["x"], np.float32).reshape(2, 2)
    W = np.array(g["w"], np.float32)[None, :]
    inv_s = np.ones(2, np.float32)
    step_x, zero_x, _ = orc.qparams(X.min(), X.max(), 8)
    assert float(step_x) == g["step_x"][0] and zero_x == int(g["zero_x"][0])
    a = orc.quant_act(X, inv_s, step_x, zero_x)
    assert a["xq"].reshape(-1).tolist() == [int(v) for v in g["xq"]]
    step_w, zero_w, _ = orc.qparams(W.min(), W.max(), 8)
    assert float(step_w) == g["step_w"][0] and zero_w == int(g["zero_w"][0])
    u, _ = orc.quant_values(W.reshape(-1), step_w, zero_w, 8)
    wq = (u - 128).astype(np.int8)[None, :]
    assert wq.reshape(-1).tolist() == [int(v) for v in g["wq"]]
    acc = orc.gemm_i8(a["xq"], wq)
    assert acc.reshape(-1).tolist() == [int(v) for v in g["acc"]]
    sw, zw = np.array([step_w], np.float32), np.array([zero_w], np.int32)
    d_lit, _ = orc.bias_literal_w8a8(X, inv_s, W, a["xq"], wq, step_x, zero_x, sw, zw)
    assert abs(d_lit[0] - g["delta"][0]) < 1e-6
    mu = X.astype(np.float64).mean(axis=0).astype(np.float32)
    d_id, _ = orc.bias_w8a8(W, mu, 2, acc.astype(np.int64).sum(axis=0), a["colsum_xq"], wq.astype(np.int32).sum(axis=1),
                            step_x, zero_x, sw, zw)
    assert abs(d_id[0] - g["delta"][0]) < 1e-6


def _small_layer(orc, dt, seed, T=96, K=64, N=24):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((T, K)).astype(dt) + np.array(rng.uniform(-0.5, 0.5, K), dt)
    X[:, 9] *= 30
    W = (rng.standard_normal((N, K)) * 0.02).astype(dt)
    sx, sw = orc.col_stats(X), orc.col_stats(W, want_sum=False)
    r_x, _, _ = orc.ranges(sx["cmin"], sx["cmax"])
    r_w, _, _ = orc.ranges(sw["cmin"], sw["cmax"])
    s, inv_s, _ = orc.scales(r_x, r_w)
    Wh = orc.fold_weight(W, s)
    lo, hi, mu = orc.xhat_stats(sx["cmin"], sx["cmax"], sx["csum"], sx["count"], inv_s)
    return X, W, Wh, s, inv_s, lo, hi, mu, T, K, N


@pytest.mark.parametrize("dt", [np.float32, np.float16])
def test_bias_w8a8_identity_equals_literal_and_postcondition(orc, dt):
    X, W, Wh, s, inv_s, lo, hi, mu, T, K, N = _small_layer(orc, dt, 16)
    step_x, zero_x, _ = orc.qparams(lo, hi, 8)
    a = orc.quant_act(X, inv_s, step_x, zero_x)
    q = orc.quant_weight(Wh, 8, 0)
    wq = orc.pack_codes(q["codes_u"], 8)
    acc = orc.gemm_i8(a["xq"], wq)
    bias = np.random.default_rng(1).standard_normal(N).astype(np.float32)
    d_lit, b_lit = orc.bias_literal_w8a8(X, inv_s, Wh, a["xq"], wq, step_x, zero_x, q["step"], q["zero"], bias)
    d_id, b_id = orc.bias_w8a8(Wh, mu, T, acc.astype(np.int64).sum(axis=0), a["colsum_xq"], q["rowsum_w"],
                               step_x, zero_x, q["step"], q["zero"], bias)
    assert np.max(np.abs(d_id - d_lit)) <= 1e-5 * np.max(np.abs(d_lit))
    np.testing.assert_allclose(b_id, b_lit, rtol=1e-6, atol=1e-9)
    # post-condition (Sec. 3.3): with the corrected bias the mean output error vanishes
    Xh = orc.fold_act(X, inv_s).astype(np.float64)
    y_fp = Xh @ Wh.astype(np.float64).T + bias
    y_q = orc.w8a8_output_direct(a["xq"], wq, step_x, zero_x, q["step"], q["zero"], None) + b_lit.astype(np.float64)
    resid = (y_q - y_fp).mean(axis=0)
    assert np.max(np.abs(resid)) <= 1e-6 * np.max(np.abs(y_fp)) + 1e-7
    assert np.max(np.abs(d_lit)) > 100 * np.max(np.abs(resid))  # the correction is not vacuous
    # BC off leaves the bias alone
    _, b_off = orc.bias_w8a8(Wh, mu, T, acc.astype(np.int64).sum(axis=0), a["colsum_xq"], q["rowsum_w"],
                             step_x, zero_x, q["step"], q["zero"], bias, enable_bc=False)
    assert np.array_equal(b_off, bias)


@pytest.mark.parametrize("bits,group", [(4, 32), (3, 32), (8, 0)])
def test_bias_weight_only_identity_equals_literal(orc, bits, group):
    X, W, Wh, s, inv_s, lo, hi, mu, T, K, N = _small_layer(orc, np.float16, 17)
    q = orc.quant_weight(Wh, bits, group)
    Wt = orc.dequant_weight(q["codes_u"], group, q["step"], q["zero"])
    d_lit, b_lit = orc.bias_literal_wonly(X, inv_s, Wh, Wt)
    d_id, b_id = orc.bias_wonly(Wh, mu, q["codes_u"], group, q["step"], q["zero"])
    assert np.max(np.abs(d_id - d_lit)) <= 1e-5 * np.max(np.abs(d_lit))
    # Eq. 12-15 in numpy: delta = -(W~ - W_hat) E[x_hat]
    eps = Wt.astype(np.float64) - Wh.astype(np.float64)
    np.testing.assert_allclose(d_id, -(eps @ mu.astype(np.float64)), rtol=1e-10, atol=1e-15)
    # post-condition
    Xh = orc.fold_act(X, inv_s).astype(np.float64)
    resid = (Xh @ Wt.astype(np.float64).T + b_lit - Xh @ Wh.astype(np.float64).T).mean(axis=0)
    assert np.max(np.abs(resid)) <= 1e-5 * np.max(np.abs(d_lit))


def test_equalization_reduces_w8a8_error_with_outliers(orc):
    """The method's purpose (Sec. 2-3): with outlier channels, AWE lowers the W8A8 output error."""
    rng = np.random.default_rng(18)
    T, K, N = 128, 64, 32
    X = rng.standard_normal((T, K)).astype(np.float32)
    X[:, [3, 40]] *= 60
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    y = X.astype(np.float64) @ W.astype(np.float64).T
    errs = {}
    for awe in (False, True):
        sx, sw = orc.col_stats(X), orc.col_stats(W, want_sum=False)
        r_x, _, _ = orc.ranges(sx["cmin"], sx["cmax"])
        r_w, _, _ = orc.ranges(sw["cmin"], sw["cmax"])
        s, inv_s, _ = orc.scales(r_x, r_w, enable_awe=awe)
        Wh = orc.fold_weight(W, s)
        lo, hi, mu = orc.xhat_stats(sx["cmin"], sx["cmax"], sx["csum"], sx["count"], inv_s)
        step_x, zero_x, _ = orc.qparams(lo, hi, 8)
        a = orc.quant_act(X, inv_s, step_x, zero_x)
        q = orc.quant_weight(Wh, 8, 0)
        yq = orc.w8a8_output_direct(a["xq"], orc.pack_codes(q["codes_u"], 8), step_x, zero_x, q["step"], q["zero"])
        errs[awe] = np.sqrt(np.mean((yq - y) ** 2))
    assert errs[True] < 0.5 * errs[False]


# ------------------------------------------------------------- weight-only forward (binary16)


def test_dequant_weight_h_special_cases_and_bound(orc):
    """Pins of the binary16 W-tilde: (i) a Step that binary16 holds exactly reproduces the binary32
    Eq. 1 de-quantisation exactly; (ii) a hand-worked value; (iii) in general it is within one
    binary16 rounding of Step and one of the product of the binary32 one."""
    rng = np.random.default_rng(3)
    codes = rng.integers(0, 16, (5, 256)).astype(np.uint8)
    zero = rng.integers(0, 16, (5, 2)).astype(np.int32)
    step = np.array([[0.25, 0.0078125]] * 5, np.float32)         # exact in binary16
    wh = orc.dequant_weight_h(codes, 128, step, zero)
    w32 = orc.dequant_weight(codes, 128, step, zero)
    assert np.array_equal(wh.astype(np.float32), w32)
    # hand-worked: Step = 0.1 -> binary16 0.0999755859375; (13 - 6) * that = 0.6998291015625,
    # nearest binary16 values are 0.69970703125 and 0.7001953125 -> the first
    one = orc.dequant_weight_h(np.array([[13]], np.uint8), 0, np.array([0.1], np.float32), np.array([6], np.int32))
    assert float(one[0, 0]) == 0.69970703125
    step = rng.uniform(1e-3, 3e-2, (5, 2)).astype(np.float32)
    wh = orc.dequant_weight_h(codes, 128, step, zero).astype(np.float64)
    w32 = orc.dequant_weight(codes, 128, step, zero).astype(np.float64)
    assert np.all(np.abs(wh - w32) <= np.abs(w32) * (2.0 ** -11 + 2.0 ** -11 + 2.0 ** -20))
    # per-row (group 0) and per-tensor (group -1) parameter indexing
    s_row, z_row = rng.uniform(1e-3, 3e-2, 5).astype(np.float32), rng.integers(0, 16, 5).astype(np.int32)
    a = orc.dequant_weight_h(codes, 0, s_row, z_row)
    for n in range(5):
        b = orc.dequant_weight_h(codes[n:n + 1], -1, s_row[n:n + 1], z_row[n:n + 1])
        assert np.array_equal(a[n:n + 1].view(np.uint16), b.view(np.uint16))


def test_wonly_forward_reduces_to_matmul(orc):
    """With binary16 operands the forward is a plain matrix product: equal to numpy's fp64 matmul
    of the widened operands up to fp64 summation order, to a brute-force loop exactly, and the
    magnitude output is the product of the absolute values."""
    rng = np.random.default_rng(4)
    T, K, N = 7, 96, 5
    X = rng.standard_normal((T, K)).astype(np.float16)
    W = (rng.standard_normal((N, K)) * 0.05).astype(np.float16)
    b = rng.standard_normal(N).astype(np.float32)
    y, a = orc.wonly_forward(X, W, b)
    ref = X.astype(np.float64) @ W.astype(np.float64).T + b.astype(np.float64)
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-12)
    brute = np.zeros((T, N))
    for t in range(T):
        for n in range(N):
            acc = 0.0
            for k in range(K):
                acc += float(X[t, k]) * float(W[n, k])
            brute[t, n] = acc + float(b[n])
    assert np.array_equal(y, brute)
    np.testing.assert_allclose(a, np.abs(X.astype(np.float64)) @ np.abs(W.astype(np.float64)).T + np.abs(b), rtol=1e-13)
    y0, _ = orc.wonly_forward(X, W)
    np.testing.assert_allclose(y0 + b, y, rtol=0, atol=1e-12)
    # a transposed operand or a dropped bias would not survive this: one-hot probes
    E = np.zeros((1, K), np.float16); E[0, 17] = 1
    yk, _ = orc.wonly_forward(E, W)
    assert np.array_equal(yk[0], W[:, 17].astype(np.float64))
