"""The statistics entry point that allocates nothing (its per-slice partial rows live in a device
array inside the library) against the ordinary entry point with a caller's workspace: the same
kernels in the same launch shape, so every output must agree bit for bit -- on two calls in a row,
the second on a smaller input (the array keeps the first call's contents), and with the oracle."""
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


def _outputs(K):
    e = lambda n, dt: torch.empty(n, dtype=dt, device=DEV)
    return dict(cmin=e(K, torch.float32), cmax=e(K, torch.float32), csum=e(K, torch.float64),
                count=torch.zeros(1, dtype=torch.int64, device=DEV), r=e(K, torch.float32), R=e(1, torch.float32),
                p=e(K, torch.float32), status=torch.zeros(1, dtype=torch.int32, device=DEV))


def _run(B, M, static, prev=None):
    rows, K = M.shape
    dt = B.AWEQ_F16 if M.dtype == torch.float16 else B.AWEQ_F32
    o = prev if prev is not None else _outputs(K)
    acc = int(prev is not None)
    if static:
        B.aweq_calib_stats_static(M, dt, rows, K, M.stride(0), o["cmin"], o["cmax"], o["csum"], o["count"], acc, 1,
                                  o["r"], o["R"], o["p"], o["status"])
    else:
        ws = torch.empty(max(16, B.aweq_workspace_size(B.OP_CALIB_STATS, rows, K)), dtype=torch.uint8, device=DEV)
        B.aweq_calib_stats(M, dt, rows, K, M.stride(0), o["cmin"], o["cmax"], o["csum"], o["count"], acc, 1,
                           o["r"], o["R"], o["p"], ws, o["status"])
    torch.cuda.synchronize()
    return o


def _same(a, b):
    for k in a:
        x, y = a[k].cpu().numpy(), b[k].cpu().numpy()
        assert np.array_equal(x.view(np.uint8), y.view(np.uint8)), k


def test_static_scratch_entry_matches_workspace_entry(B, orc):
    rng = np.random.default_rng(2311)
    shapes = [(np.float16, 6000, 1544),   # first call: many slices, four column chunks with a ragged tail
              (np.float16, 517, 264),     # second call, smaller: stale partial rows of the first stay in the array
              (np.float32, 1031, 520),
              (np.float16, 1, 8)]
    for dtype, rows, K in shapes:
        print(f"[no-alloc] stats {dtype.__name__} rows={rows} K={K}", flush=True)
        assert B.aweq_workspace_size(B.OP_CALIB_STATS, rows, K) <= B.STATIC_SCRATCH_BYTES
        Mh = (rng.standard_normal((rows, K)) * 2).astype(dtype)
        Mh[:, K // 2] *= 30
        M = torch.from_numpy(Mh).to(DEV)
        a = _run(B, M, static=True)
        b = _run(B, M, static=False)
        _same(a, b)
        o = orc.col_stats(Mh)
        assert np.array_equal(a["cmin"].cpu().numpy(), o["cmin"]) and np.array_equal(a["cmax"].cpu().numpy(), o["cmax"])
        scale = np.abs(Mh.astype(np.float64)).mean(axis=0) * rows
        assert np.all(np.abs(a["csum"].cpu().numpy() - o["csum"]) <= 1e-6 * scale + 1e-12)
        assert int(a["count"].item()) == rows and int(a["status"].item()) == 0
    # a second batch merged into the first (accumulate = 1) through both entry points
    M1 = torch.from_numpy((rng.standard_normal((900, 520)) * 2).astype(np.float16)).to(DEV)
    M2 = torch.from_numpy((rng.standard_normal((300, 520)) * 5).astype(np.float16)).to(DEV)
    a = _run(B, M2, static=True, prev=_run(B, M1, static=True))
    b = _run(B, M2, static=False, prev=_run(B, M1, static=False))
    _same(a, b)
    assert int(a["count"].item()) == 1200


def test_static_scratch_entry_rejects_what_does_not_fit(B):
    P = 0x10000
    rows, K = 1 << 20, 1 << 21      # the partial rows of this shape need more than the built-in array
    assert B.aweq_workspace_size(B.OP_CALIB_STATS, rows, K) > B.STATIC_SCRATCH_BYTES
    with pytest.raises(B.AweqError) as ei:
        B.aweq_calib_stats_static(P, B.AWEQ_F16, rows, K, K, P, P, P, P, 0, 1, P, P, P, None, stream=0)
    assert ei.value.name == "AWEQ_ERR_WORKSPACE"
