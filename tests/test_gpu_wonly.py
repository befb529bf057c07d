"""Weight-only forward (W4 / W3 per group, binary16 activations) against the oracle.
The de-quantised weight is checked bit for bit through one-hot activations (a single non-zero
product per output, so no summation is involved); the full product within a bound derived from
fp32 accumulation: |y - ref| <= K * 2^-24 * sum_k |x w| (any summation order of exact fp32
products) plus one rounding of the output type."""
import numpy as np
import pytest

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
    print(f"[gpu-wonly] {msg}", flush=True)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def make_weights(orc, rng, N, K, bits, group, shift=0.0):
    W = (rng.standard_normal((N, K)) * 0.02 * rng.uniform(0.3, 3.0, (1, K)) + shift).astype(np.float16)
    q = orc.quant_weight(W, bits, group)
    packed = orc.pack_codes(q["codes_u"], bits).view(np.uint8).reshape(-1)
    return q, packed


def run(B, Xh, packed, q, bits, group, N, bias, odt):
    T, K = Xh.shape
    out = torch.full((T, N), 7.0, dtype=torch.float16 if odt == np.float16 else torch.float32, device=DEV)
    ws = torch.empty(B.aweq_workspace_size(B.OP_WONLY_GEMM, T, K, N), dtype=torch.uint8, device=DEV)
    B.aweq_wonly_gemm(dev(Xh), T, K, K, dev(packed), bits, group, dev(q["step"].reshape(-1)), dev(q["zero"].reshape(-1)),
                      N, dev(bias) if bias is not None else None, out, B.AWEQ_F16 if odt == np.float16 else B.AWEQ_F32, N, ws)
    return host(out)


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("N,K,group", [(260, 256, 128), (64, 128, 64), (68, 96 + 32, 32), (36, 512, 0), (40, 192, -1), (300, 1024, 512)])
def test_dequantised_weight_bit_exact_through_one_hot_rows(B, orc, bits, N, K, group):
    progress(f"one-hot W{bits} N={N} K={K} g={group}")
    rng = np.random.default_rng(bits * 1000 + N + K)
    q, packed = make_weights(orc, rng, N, K, bits, group)
    Wh = orc.dequant_weight_h(q["codes_u"], group, q["step"], q["zero"])
    X = np.eye(K, dtype=np.float16)                     # token k is the unit vector e_k
    got = run(B, X, packed, q, bits, group, N, None, np.float16)
    assert np.array_equal(got.view(np.uint16), np.ascontiguousarray(Wh.T).view(np.uint16))


def test_zero_point_outside_the_packed_path(B, orc):
    """A slice far from zero has |Z| > 1024 (and |u - Z| > 2048): the binary32 path, same definition."""
    progress("one-hot, large zero points")
    rng = np.random.default_rng(9)
    N, K = 32, 128
    for bits in (4, 3):
        q, packed = make_weights(orc, rng, N, K, bits, 64, shift=30.0)
        assert (np.abs(q["zero"]) > 1024).any() and (bits == 3 or np.abs(q["zero"]).max() > 2048)
        Wh = orc.dequant_weight_h(q["codes_u"], 64, q["step"], q["zero"])
        got = run(B, np.eye(K, dtype=np.float16), packed, q, bits, 64, N, None, np.float16)
        assert np.array_equal(got.view(np.uint16), np.ascontiguousarray(Wh.T).view(np.uint16))


@pytest.mark.parametrize("odt", [np.float16, np.float32])
@pytest.mark.parametrize("bits,T,N,K,group", [
    (4, 300, 260, 256, 128), (3, 300, 260, 256, 128),
    (4, 515, 1028, 384, 128), (3, 515, 1028, 384, 64),
    (4, 256, 256, 64, 0), (3, 1, 4, 64, -1),
    (4, 700, 2100, 128, 128),        # more than one patch along N
    (4, 1000, 512, 4096, 128), (3, 777, 300, 4096, 128),   # the K of the LLaMA-7B attention linears
    (4, 300, 2052, 4224, 128),       # K >= 2 N with nine tile columns: the 4 x 8 patch shape
])
def test_forward_parity(B, orc, odt, bits, T, N, K, group):
    progress(f"forward W{bits} {odt.__name__} T={T} N={N} K={K} g={group}")
    rng = np.random.default_rng(T + N + K + bits)
    q, packed = make_weights(orc, rng, N, K, bits, group)
    X = rng.standard_normal((T, K)).astype(np.float32)
    X[:, 5 % K] *= 40.0                                   # an outlier channel
    Xh = X.astype(np.float16)
    bias = rng.standard_normal(N).astype(np.float32)
    Wh = orc.dequant_weight_h(q["codes_u"], group, q["step"], q["zero"])
    ref, mag = orc.wonly_forward(Xh, Wh, bias)
    got = run(B, Xh, packed, q, bits, group, N, bias, odt).astype(np.float64)
    out_ulp = 2.0 ** -11 if odt == np.float16 else 2.0 ** -24
    bound = K * 2.0 ** -24 * mag + out_ulp * np.abs(ref) + 2.0 ** -24
    assert np.all(np.abs(got - ref) <= bound), float(np.max(np.abs(got - ref) / bound))
    # and it is a far tighter match than a wrong scale or a dropped group would give
    assert np.max(np.abs(got - ref)) <= 2e-3 * np.max(np.abs(ref))
    got_nb = run(B, Xh, packed, q, bits, group, N, None, odt).astype(np.float64)
    assert np.max(np.abs(got_nb + bias - got)) <= 4 * out_ulp * np.max(np.abs(ref)) + 1e-6
