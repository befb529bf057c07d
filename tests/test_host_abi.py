"""Host-side checks of the C-ABI library: it loads, exports every symbol the header
declares, sizes workspaces, and turns bad arguments into error codes before launching
anything (so none of this needs a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2311_01305_amd import binding
    binding.load_library()
    return binding


def header_functions():
    src = open(os.path.join(ROOT, "include", "aweq.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(aweq_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol(B):
    names = header_functions()
    assert set(names) == set(B.EXPORTS)
    lib = B.load_library()
    for n in names:
        assert getattr(lib, n) is not None
    # and the python binding has a function of the same name for each
    for n in names:
        assert callable(getattr(B, n))


def test_status_strings(B):
    assert B.aweq_status_string(0) == "AWEQ_OK"
    for code, name in [(-1, "NULL"), (-2, "SHAPE"), (-3, "DTYPE"), (-4, "BITS"), (-5, "GROUP"), (-6, "ALIGN"),
                       (-7, "WORKSPACE"), (-8, "LAUNCH")]:
        assert B.aweq_status_string(code) == "AWEQ_ERR_" + name


def test_workspace_sizes(B):
    # stats partials: (min, max fp32 + sum fp64) per column per row slice; bounded and monotone in K
    a = B.aweq_workspace_size(B.OP_CALIB_STATS, 262144, 4096)
    b = B.aweq_workspace_size(B.OP_CALIB_STATS, 262144, 16384)
    assert (a - 16) % (4096 * 16) == 0 and 0 < a <= 64 << 20 and 0 < b <= 64 << 20   # + the merge kernel's control words
    assert B.aweq_workspace_size(B.OP_CALIB_STATS, 8, 8) == 8 * 16 + 16
    assert B.aweq_workspace_size(B.OP_CALIB_STATS, 0, 8) == 0
    assert B.aweq_workspace_size(B.OP_QUANT_WEIGHT, 4096, 4096) >= 8
    for op in (B.OP_EQUALIZE, B.OP_BIAS_CORRECT):
        assert B.aweq_workspace_size(op, 4096, 4096, 4096) == 0
    # the fused GEMM's output statistics (a key pair and a 64-bit sum per output channel) or stage 4a's
    # partial sums, whichever is larger
    assert B.aweq_workspace_size(B.OP_W8A8_GEMM, 64, 64, 11008) == 11008 * 16
    assert B.aweq_workspace_size(B.OP_W8A8_GEMM, 262144, 4096, 4096) == B.aweq_workspace_size(B.OP_QUANT_ACT, 262144, 4096)


P = 0x10000  # a fake, 16-byte aligned, never dereferenced "device pointer"


def _code(fn, *a, **k):
    from paper_2311_01305_amd.binding import AweqError
    with pytest.raises(AweqError) as e:
        fn(*a, **k)
    return e.value.name


def test_calib_stats_argument_errors(B):
    ok = dict(M=P, dt=B.AWEQ_F16, rows=64, K=64, ld=64, cmin=P, cmax=P, csum=P, count=P, accumulate=0, finalize=1,
              r=P, R=P, p=P, ws=P, ws_bytes=1 << 20)
    call = lambda **kw: B.aweq_calib_stats(**{**ok, **kw})
    assert _code(call, M=None) == "AWEQ_ERR_NULL"
    assert _code(call, cmin=None) == "AWEQ_ERR_NULL"
    assert _code(call, r=None) == "AWEQ_ERR_NULL"
    assert _code(call, dt=B.AWEQ_I8) == "AWEQ_ERR_DTYPE"
    assert _code(call, rows=0) == "AWEQ_ERR_SHAPE"
    assert _code(call, K=60, ld=60) == "AWEQ_ERR_SHAPE"
    assert _code(call, ld=32) == "AWEQ_ERR_SHAPE"
    assert _code(call, M=P + 2) == "AWEQ_ERR_ALIGN"
    assert _code(call, ld=68) == "AWEQ_ERR_ALIGN"  # 136-byte pitch
    assert _code(call, ws=None) == "AWEQ_ERR_WORKSPACE"
    assert _code(call, ws_bytes=16) == "AWEQ_ERR_WORKSPACE"


def test_calib_stats_static_argument_errors(B):
    """The entry point without a workspace argument: the same host checks, and a size limit instead
    of a workspace check (found before anything touches the GPU)."""
    ok = dict(M=P, dt=B.AWEQ_F16, rows=64, K=64, ld=64, cmin=P, cmax=P, csum=P, count=P, accumulate=0, finalize=1,
              r=P, R=P, p=P, stream=0)
    call = lambda **kw: B.aweq_calib_stats_static(**{**ok, **kw})
    assert _code(call, M=None) == "AWEQ_ERR_NULL"
    assert _code(call, R=None) == "AWEQ_ERR_NULL"
    assert _code(call, dt=B.AWEQ_I8) == "AWEQ_ERR_DTYPE"
    assert _code(call, K=60, ld=60) == "AWEQ_ERR_SHAPE"
    assert _code(call, M=P + 2) == "AWEQ_ERR_ALIGN"
    big = 1 << 21
    assert B.aweq_workspace_size(B.OP_CALIB_STATS, big, big) > B.STATIC_SCRATCH_BYTES
    assert _code(call, rows=big, K=big, ld=big) == "AWEQ_ERR_WORKSPACE"
    # every configuration of the benchmark fits
    for K in (4096, 8192, 11008, 16384, 22016):
        assert B.aweq_workspace_size(B.OP_CALIB_STATS, 262144, K) <= B.STATIC_SCRATCH_BYTES


def test_equalize_argument_errors(B):
    ok = dict(xmin=P, xmax=P, xsum=P, count=10, wmin=P, wmax=P, K=64, enable_awe=1, s=P, inv_s=P, W=P, W_hat=P,
              dt=B.AWEQ_F16, N=8, ldw=64, ldwh=64, prev_scale=None, xhat_range=P, mu_xhat=P, act_step=P, act_zero=P)
    call = lambda **kw: B.aweq_equalize(**{**ok, **kw})
    assert _code(call, s=None) == "AWEQ_ERR_NULL"
    assert _code(call, xsum=None) == "AWEQ_ERR_NULL"  # mu_xhat asked without sums
    assert _code(call, act_zero=None) == "AWEQ_ERR_NULL"
    assert _code(call, W_hat=None) == "AWEQ_ERR_NULL"
    assert _code(call, K=12) == "AWEQ_ERR_SHAPE"
    assert _code(call, count=0) == "AWEQ_ERR_SHAPE"
    assert _code(call, dt=B.AWEQ_I8) == "AWEQ_ERR_DTYPE"
    assert _code(call, W=P + 4) == "AWEQ_ERR_ALIGN"
    assert _code(call, ldwh=32) == "AWEQ_ERR_SHAPE"      # the folded weight has a pitch of its own
    assert _code(call, ldwh=68) == "AWEQ_ERR_ALIGN"


def test_quant_weight_argument_errors(B):
    ok = dict(W_hat=P, dt=B.AWEQ_F16, N=8, K=256, ldw=256, bits=4, group=128, codes=P, step=P, zero=P, rowsum_w=None,
              ws=None, ws_bytes=0)
    call = lambda **kw: B.aweq_quant_weight(**{**ok, **kw})
    assert _code(call, codes=None) == "AWEQ_ERR_NULL"
    assert _code(call, bits=5) == "AWEQ_ERR_BITS"
    assert _code(call, group=96) == "AWEQ_ERR_GROUP"     # not 8 * 2^m
    assert _code(call, group=512) == "AWEQ_ERR_GROUP"    # does not divide K
    assert _code(call, group=-2) == "AWEQ_ERR_GROUP"
    assert _code(call, rowsum_w=P, bits=8) == "AWEQ_ERR_GROUP"
    assert _code(call, bits=3, K=264, ldw=264, group=8) == "AWEQ_ERR_ALIGN"  # 3-bit rows need K % 32 == 0
    assert _code(call, group=-1) == "AWEQ_ERR_WORKSPACE"
    assert _code(call, group=0, K=24584, ldw=24584) == "AWEQ_ERR_SHAPE"  # row does not fit the block
    assert _code(call, dt=B.AWEQ_I8) == "AWEQ_ERR_DTYPE"


def test_gemm_and_quant_act_argument_errors(B):
    ok = dict(X=P, x_dt=B.AWEQ_F16, T=64, K=64, ldx=64, inv_s=P, act_step=P, act_zero=P, xq=P, rowsum_x=P,
              colsum_xq=P, wq=P, N=32, step_w=P, zero_w=P, w_group=0, rowsum_w=P, bias=None, out_i32=P, out_deq=None,
              out_dt=B.AWEQ_F16, ldo=32, colsum_acc=P, ws=P, ws_bytes=1 << 20)
    call = lambda **kw: B.aweq_w8a8_gemm(**{**ok, **kw})
    assert _code(call, w_group=128) == "AWEQ_ERR_GROUP"   # the int8 path has per-channel or per-tensor weight scales
    assert _code(call, ws=None, ws_bytes=0) == "AWEQ_ERR_WORKSPACE"   # stage 4a's column sums need it
    assert B.aweq_workspace_size(B.OP_W8A8_GEMM, 64, 64, 32) >= B.aweq_workspace_size(B.OP_QUANT_ACT, 64, 64) > 0
    assert _code(call, wq=None) == "AWEQ_ERR_NULL"
    assert _code(call, xq=None) == "AWEQ_ERR_NULL"        # float input needs the code buffer
    assert _code(call, inv_s=None) == "AWEQ_ERR_NULL"
    assert _code(call, K=20, ldx=20) == "AWEQ_ERR_SHAPE"
    assert _code(call, ldo=16) == "AWEQ_ERR_SHAPE"
    assert _code(call, x_dt=B.AWEQ_I8, ldx=128) == "AWEQ_ERR_SHAPE"
    assert _code(call, out_deq=P, out_dt=B.AWEQ_I8) == "AWEQ_ERR_DTYPE"
    assert _code(call, out_deq=P, rowsum_w=None) == "AWEQ_ERR_NULL"
    assert _code(call, K=65536, ldx=65536) == "AWEQ_ERR_SHAPE"
    qa = dict(X=P, dt=B.AWEQ_F16, T=8, K=64, ldx=64, inv_s=P, act_step=P, act_zero=P, xq=P, rowsum_x=None, colsum_xq=None)
    qcall = lambda **kw: B.aweq_quant_act(**{**qa, **kw})
    assert _code(qcall, colsum_xq=P) == "AWEQ_ERR_WORKSPACE"          # column sums go through per-slice partials
    assert _code(qcall, colsum_xq=P, ws=P, ws_bytes=8) == "AWEQ_ERR_WORKSPACE"
    assert _code(qcall, K=1024, ldx=1024, rowsum_x=P) == "AWEQ_ERR_WORKSPACE"   # row sums over several column chunks
    # per-slice int32 column sums plus per-chunk int32 row sums; no row-sum partials for one chunk
    assert B.aweq_workspace_size(B.OP_QUANT_ACT, 262144, 4096) == 1024 * 4096 * 4 + 8 * 262144 * 4
    assert B.aweq_workspace_size(B.OP_QUANT_ACT, 64, 512) == 64 // 32 * 512 * 4
    assert _code(qcall, act_step=None) == "AWEQ_ERR_NULL"
    assert _code(qcall, xq=None) == "AWEQ_ERR_NULL"           # no codes and no sums asked for: nothing to do
    assert _code(qcall, dt=B.AWEQ_I8) == "AWEQ_ERR_DTYPE"
    assert _code(qcall, X=P + 8) == "AWEQ_ERR_ALIGN"


def test_bias_correct_argument_errors(B):
    ok = dict(mode=B.BIAS_W8A8, W_hat=P, dt=B.AWEQ_F16, N=8, K=64, ldw=64, mu_xhat=P, count=16, colsum_acc=P,
              colsum_xq=P, rowsum_w=P, act_step=P, act_zero=P, codes=None, bits=8, group=0, step_w=P, zero_w=P,
              bias_in=None, delta=P, bias_out=P, enable_bc=1)
    call = lambda **kw: B.aweq_bias_correct(**{**ok, **kw})
    assert _code(call, colsum_acc=None) == "AWEQ_ERR_NULL"          # neither the GEMM's sums nor the codes to form them from
    assert _code(call, colsum_acc=None, codes=P, bits=4) == "AWEQ_ERR_BITS"
    assert _code(call, colsum_acc=None, codes=P, group=128) == "AWEQ_ERR_BITS"
    assert _code(call, group=128) == "AWEQ_ERR_GROUP"
    assert _code(call, count=0) == "AWEQ_ERR_SHAPE"
    assert _code(call, mode=7) == "AWEQ_ERR_SHAPE"
    assert _code(call, mode=B.BIAS_WEIGHT_ONLY) == "AWEQ_ERR_NULL"  # needs codes
    assert _code(call, mode=B.BIAS_WEIGHT_ONLY, codes=P, bits=2) == "AWEQ_ERR_BITS"
    assert _code(call, mode=B.BIAS_WEIGHT_ONLY, codes=P, bits=4, group=48) == "AWEQ_ERR_GROUP"


def test_product_does_not_import_the_oracle():
    """The HIP path and its binding must not reach into oracle/ (and vice versa)."""
    pkg = os.path.join(ROOT, "paper_2311_01305_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower() or f == "synth.py", f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2311_01305_amd" not in text and "libaweq" not in text, f


def test_panel_layout_helpers(B):
    """aweq_panel_bytes (host) and the argument checks of the converters."""
    assert B.aweq_panel_bytes(10, 64) == 640 and B.aweq_panel_bytes(10, 72) == 1280 and B.aweq_panel_bytes(3, 8) == 192
    assert B.aweq_panel_bytes(0, 64) == 0
    P = 0x10000
    for fn, args in ((B.aweq_pack_panels_i8, (P, 4, 64, 64, P)), (B.aweq_unpack_panels_i8, (P, 4, 64, P, 64))):
        ok = list(args)
        bad_k = list(ok); bad_k[2] = 12
        with pytest.raises(B.AweqError) as ei:
            fn(*bad_k, stream=0)
        assert ei.value.name == "AWEQ_ERR_SHAPE"
        null = list(ok); null[0] = None
        with pytest.raises(B.AweqError) as ei:
            fn(*null, stream=0)
        assert ei.value.name == "AWEQ_ERR_NULL"
    with pytest.raises(B.AweqError) as ei:
        B.aweq_pack_panels_i8(P + 4, 4, 64, 64, P, stream=0)
    assert ei.value.name == "AWEQ_ERR_ALIGN"
    # the numpy reference permutation the GPU tests use is its own inverse pair
    import numpy as np
    from conftest import from_panels, to_panels
    m = np.arange(5 * 72, dtype=np.int64).reshape(5, 72).astype(np.int8)
    p = to_panels(m)
    assert p.size == B.aweq_panel_bytes(5, 72) and np.array_equal(from_panels(p, 5, 72), m)
    assert p[64 * 5 + 8] == 0 and p[0:64].tolist() == m[0, :64].tolist() and p[64:128].tolist() == m[1, :64].tolist()


def test_wonly_gemm_argument_errors(B):
    P = 0x10000
    ok = dict(X_hat=P, T=64, K=128, ldx=128, codes=P, bits=4, group=128, step_w=P, zero_w=P, N=64, bias=None, out=P,
              out_dt=B.AWEQ_F16, ldo=64, ws=P, ws_bytes=64 * 128 * 2, stream=0)
    assert B.aweq_workspace_size(B.OP_WONLY_GEMM, 64, 128, 64) == 64 * 128 * 2
    call = lambda **kw: B.aweq_wonly_gemm(**{**ok, **kw})
    assert _code(call, ws=None, ws_bytes=0) == "AWEQ_ERR_WORKSPACE"
    assert _code(call, ws_bytes=100) == "AWEQ_ERR_WORKSPACE"
    assert _code(call, X_hat=None) == "AWEQ_ERR_NULL"
    assert _code(call, bits=8) == "AWEQ_ERR_BITS"
    assert _code(call, K=96, ldx=96) == "AWEQ_ERR_SHAPE"          # K % 64
    assert _code(call, group=16) == "AWEQ_ERR_GROUP"
    assert _code(call, group=96) == "AWEQ_ERR_GROUP"
    assert _code(call, N=62, ldo=62) == "AWEQ_ERR_SHAPE"          # N % 4
    assert _code(call, ldo=32) == "AWEQ_ERR_SHAPE"
    assert _code(call, out_dt=B.AWEQ_I8) == "AWEQ_ERR_DTYPE"
    assert _code(call, X_hat=P + 2) == "AWEQ_ERR_ALIGN"


def test_fold_quant_weight_argument_errors(B):
    P = 0x10000
    ok = dict(W=P, dt=B.AWEQ_F16, N=8, K=64, ldw=64, s=P, W_hat=P, ldwh=64, bits=8, codes=P, step=P, zero=P, rowsum_w=P, stream=0)
    call = lambda **kw: B.aweq_fold_quant_weight(**{**ok, **kw})
    assert _code(call, s=None) == "AWEQ_ERR_NULL"
    assert _code(call, bits=5) == "AWEQ_ERR_BITS"
    assert _code(call, bits=4) == "AWEQ_ERR_BITS"            # row sums are an int8 notion
    assert _code(call, K=24584, ldw=24584) == "AWEQ_ERR_SHAPE"
    assert _code(call, W=P + 8) == "AWEQ_ERR_ALIGN"
    assert _code(call, ldwh=56) == "AWEQ_ERR_SHAPE"


def test_fused_gemm_argument_errors(B):
    P = 0x10000
    ok = dict(xq=P, T=64, K=64, wq=P, N=64, act_step=P, act_zero=P, step_w=P, zero_w=P, rowsum_x=P, rowsum_w=P, bias=None,
              act=0, out_f16=P, ldo=64, colsum_acc=P, ycmin=P, ycmax=P, ycsum=P, ycount=P, accumulate=0, next_inv_s=P,
              next_step=P, next_zero=P, yq=P, rowsum_y=P, colsum_yq=P, ws=P, ws_bytes=64 * 16, stream=0)
    assert B.aweq_workspace_size(B.OP_W8A8_GEMM, 64, 64, 64) == 64 * 16
    call = lambda **kw: B.aweq_w8a8_gemm_fused(**{**ok, **kw})
    assert _code(call, colsum_acc=None) == "AWEQ_ERR_NULL"
    assert _code(call, ycmin=None, yq=None) == "AWEQ_ERR_NULL"      # at least one fused epilogue
    assert _code(call, ycmax=None) == "AWEQ_ERR_NULL"
    assert _code(call, next_step=None) == "AWEQ_ERR_NULL"
    assert _code(call, act=2) == "AWEQ_ERR_SHAPE"
    assert _code(call, N=62, ldo=62) == "AWEQ_ERR_SHAPE"            # the tiled kernel stores channel quads
    assert _code(call, ldo=32) == "AWEQ_ERR_SHAPE"
    assert _code(call, K=65536) == "AWEQ_ERR_SHAPE"
    assert _code(call, ws_bytes=100) == "AWEQ_ERR_WORKSPACE"
    assert _code(call, ws=None, ws_bytes=0) == "AWEQ_ERR_WORKSPACE"
    assert _code(call, next_inv_s=P + 4) == "AWEQ_ERR_ALIGN"
    assert _code(call, bias=P + 4) == "AWEQ_ERR_ALIGN"
