"""ctypes binding of libaweq.so: same names and argument order as include/aweq.h.

Argument marshalling only.  Tensor arguments are torch tensors living on the GPU (or None
for a nullable pointer); their data_ptr() is handed to the library, and the current torch
stream is passed unless `stream` is given.  PyTorch is used for device memory and streams
only.  Raw integer addresses are accepted in place of tensors (used by host-side tests).
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libaweq.so")
_lib = None

AWEQ_F32, AWEQ_F16, AWEQ_I8 = 0, 1, 2
OP_CALIB_STATS, OP_EQUALIZE, OP_QUANT_WEIGHT, OP_W8A8_GEMM, OP_BIAS_CORRECT, OP_WONLY_GEMM, OP_QUANT_ACT = 0, 1, 2, 3, 4, 5, 6
BIAS_W8A8, BIAS_WEIGHT_ONLY = 0, 1
SCALE_NONE, SCALE_RANGE, SCALE_ABSMAX = 0, 1, 2
ST_DEGENERATE, ST_NONFINITE, ST_BIGQUOT, ST_SCALEGUARD, ST_ZEROPOINT = 1, 2, 4, 8, 16

EXPORTS = ("aweq_workspace_size", "aweq_status_string", "aweq_calib_stats", "aweq_equalize",
           "aweq_quant_weight", "aweq_quant_act", "aweq_w8a8_gemm", "aweq_bias_correct",
           "aweq_panel_bytes", "aweq_pack_panels_i8", "aweq_unpack_panels_i8", "aweq_wonly_gemm", "aweq_fold_quant_weight", "aweq_w8a8_gemm_fused",
           "aweq_calib_stats_static")
STATIC_SCRATCH_BYTES = 16 << 20

_vp, _i64, _i32, _u64, _f32, _sz = C.c_void_p, C.c_int64, C.c_int, C.c_uint64, C.c_float, C.c_size_t


class AweqError(RuntimeError):
    def __init__(self, code, name):
        super().__init__(f"libaweq: {name} ({code})")
        self.code = code
        self.name = name


def load_library():
    """Load the in-tree libaweq.so; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    # torch brings its own HIP runtime; it has to be the one already in the process when
    # libaweq.so resolves its runtime symbols, or streams and kernels end up in two runtimes
    import torch  # noqa: F401
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2311_01305_amd.build` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(_LIB_PATH)
    lib.aweq_workspace_size.restype = _sz
    lib.aweq_workspace_size.argtypes = [_i32, _i64, _i64, _i64]
    lib.aweq_status_string.restype = C.c_char_p
    lib.aweq_status_string.argtypes = [_i32]
    lib.aweq_calib_stats.restype = _i32
    lib.aweq_calib_stats.argtypes = [_vp, _i32, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp,
                                     _vp, _sz, _vp, _vp]
    lib.aweq_calib_stats_static.restype = _i32
    lib.aweq_calib_stats_static.argtypes = [_vp, _i32, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp,
                                            _vp, _vp]
    lib.aweq_equalize.restype = _i32
    lib.aweq_equalize.argtypes = [_vp, _vp, _vp, _u64, _vp, _vp, _i64, _i32, _vp, _vp, _vp, _vp, _i32, _i64, _i64, _i64,
                                  _vp, _vp, _vp, _vp, _vp, _vp, _vp]
    lib.aweq_quant_weight.restype = _i32
    lib.aweq_quant_weight.argtypes = [_vp, _i32, _i64, _i64, _i64, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _sz, _vp, _vp]
    lib.aweq_quant_act.restype = _i32
    lib.aweq_quant_act.argtypes = [_vp, _i32, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp, _vp]
    lib.aweq_w8a8_gemm.restype = _i32
    lib.aweq_w8a8_gemm.argtypes = [_vp, _i32, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _vp, _vp, _i32,
                                   _vp, _vp, _vp, _vp, _i32, _i64, _vp, _vp, _sz, _vp, _vp]
    lib.aweq_w8a8_gemm_fused.restype = _i32
    lib.aweq_w8a8_gemm_fused.argtypes = [_vp, _i64, _i64, _vp, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _i64, _vp,
                                         _vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp, _vp]
    lib.aweq_bias_correct.restype = _i32
    lib.aweq_bias_correct.argtypes = [_i32, _vp, _i32, _i64, _i64, _i64, _vp, _u64, _vp, _vp, _vp, _vp, _vp, _vp,
                                      _i32, _i32, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp]
    lib.aweq_wonly_gemm.restype = _i32
    lib.aweq_wonly_gemm.argtypes = [_vp, _i64, _i64, _i64, _vp, _i32, _i32, _vp, _vp, _i64, _vp, _vp, _i32, _i64, _vp, _sz,
                                    _vp, _vp]
    lib.aweq_fold_quant_weight.restype = _i32
    lib.aweq_fold_quant_weight.argtypes = [_vp, _i32, _i64, _i64, _i64, _vp, _vp, _i64, _i32, _vp, _vp, _vp, _vp, _vp, _vp]
    lib.aweq_panel_bytes.restype = _sz
    lib.aweq_panel_bytes.argtypes = [_i64, _i64]
    lib.aweq_pack_panels_i8.restype = _i32
    lib.aweq_pack_panels_i8.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp]
    lib.aweq_unpack_panels_i8.restype = _i32
    lib.aweq_unpack_panels_i8.argtypes = [_vp, _i64, _i64, _vp, _i64, _vp]
    _lib = lib
    return lib


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _nbytes(t):
    if t is None:
        return 0
    return t.numel() * t.element_size()


def _stream(stream):
    if stream is not None:
        return stream if isinstance(stream, int) else stream.cuda_stream
    import torch
    return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None


def _check(code):
    if code != 0:
        raise AweqError(code, aweq_status_string(code))


def aweq_status_string(code):
    return load_library().aweq_status_string(int(code)).decode()


def aweq_workspace_size(op, rows, K, N=0):
    return int(load_library().aweq_workspace_size(int(op), int(rows), int(K), int(N)))


def aweq_calib_stats(M, dt, rows, K, ld, cmin, cmax, csum, count, accumulate, finalize, r, R, p, ws,
                     status=None, stream=None, ws_bytes=None):
    _check(load_library().aweq_calib_stats(
        _ptr(M), dt, rows, K, ld, _ptr(cmin), _ptr(cmax), _ptr(csum), _ptr(count), int(accumulate), int(finalize),
        _ptr(r), _ptr(R), _ptr(p), _ptr(ws), _nbytes(ws) if ws_bytes is None else ws_bytes, _ptr(status),
        _stream(stream)))


def aweq_calib_stats_static(M, dt, rows, K, ld, cmin, cmax, csum, count, accumulate, finalize, r, R, p,
                            status=None, stream=None):
    _check(load_library().aweq_calib_stats_static(
        _ptr(M), dt, rows, K, ld, _ptr(cmin), _ptr(cmax), _ptr(csum), _ptr(count), int(accumulate), int(finalize),
        _ptr(r), _ptr(R), _ptr(p), _ptr(status), _stream(stream)))


def aweq_equalize(xmin, xmax, xsum, count, wmin, wmax, K, enable_awe, s, inv_s, W, W_hat, dt, N, ldw, ldwh,
                  prev_scale, xhat_range, mu_xhat, act_step, act_zero, status=None, stream=None):
    _check(load_library().aweq_equalize(
        _ptr(xmin), _ptr(xmax), _ptr(xsum), int(count), _ptr(wmin), _ptr(wmax), K, int(enable_awe), _ptr(s),
        _ptr(inv_s), _ptr(W), _ptr(W_hat), dt, N, ldw, ldwh, _ptr(prev_scale), _ptr(xhat_range), _ptr(mu_xhat),
        _ptr(act_step), _ptr(act_zero), _ptr(status), _stream(stream)))


def aweq_quant_weight(W_hat, dt, N, K, ldw, bits, group, codes, step, zero, rowsum_w, ws=None,
                      status=None, stream=None, ws_bytes=None):
    _check(load_library().aweq_quant_weight(
        _ptr(W_hat), dt, N, K, ldw, int(bits), int(group), _ptr(codes), _ptr(step), _ptr(zero), _ptr(rowsum_w),
        _ptr(ws), _nbytes(ws) if ws_bytes is None else ws_bytes, _ptr(status), _stream(stream)))


def aweq_quant_act(X, dt, T, K, ldx, inv_s, act_step, act_zero, xq, rowsum_x, colsum_xq, ws=None, status=None, stream=None,
                   ws_bytes=None):
    _check(load_library().aweq_quant_act(
        _ptr(X), dt, T, K, ldx, _ptr(inv_s), _ptr(act_step), _ptr(act_zero), _ptr(xq), _ptr(rowsum_x),
        _ptr(colsum_xq), _ptr(ws), _nbytes(ws) if ws_bytes is None else ws_bytes, _ptr(status), _stream(stream)))


def aweq_w8a8_gemm(X, x_dt, T, K, ldx, inv_s, act_step, act_zero, xq, rowsum_x, colsum_xq, wq, N, step_w, zero_w, w_group,
                   rowsum_w, bias, out_i32, out_deq, out_dt, ldo, colsum_acc, ws=None, status=None, stream=None,
                   ws_bytes=None):
    _check(load_library().aweq_w8a8_gemm(
        _ptr(X), x_dt, T, K, ldx, _ptr(inv_s), _ptr(act_step), _ptr(act_zero), _ptr(xq), _ptr(rowsum_x),
        _ptr(colsum_xq), _ptr(wq), N, _ptr(step_w), _ptr(zero_w), int(w_group), _ptr(rowsum_w), _ptr(bias), _ptr(out_i32),
        _ptr(out_deq), out_dt, ldo, _ptr(colsum_acc), _ptr(ws), _nbytes(ws) if ws_bytes is None else ws_bytes,
        _ptr(status), _stream(stream)))


def aweq_bias_correct(mode, W_hat, dt, N, K, ldw, mu_xhat, count, colsum_acc, colsum_xq, rowsum_w, act_step,
                      act_zero, codes, bits, group, step_w, zero_w, bias_in, delta, bias_out, enable_bc,
                      status=None, stream=None):
    _check(load_library().aweq_bias_correct(
        int(mode), _ptr(W_hat), dt, N, K, ldw, _ptr(mu_xhat), int(count), _ptr(colsum_acc), _ptr(colsum_xq),
        _ptr(rowsum_w), _ptr(act_step), _ptr(act_zero), _ptr(codes), int(bits), int(group), _ptr(step_w),
        _ptr(zero_w), _ptr(bias_in), _ptr(delta), _ptr(bias_out), int(enable_bc), _ptr(status), _stream(stream)))


def aweq_panel_bytes(rows, K):
    return int(load_library().aweq_panel_bytes(int(rows), int(K)))


def aweq_pack_panels_i8(src, rows, K, ld, panels, stream=None):
    _check(load_library().aweq_pack_panels_i8(_ptr(src), rows, K, ld, _ptr(panels), _stream(stream)))


def aweq_unpack_panels_i8(panels, rows, K, dst, ld, stream=None):
    _check(load_library().aweq_unpack_panels_i8(_ptr(panels), rows, K, _ptr(dst), ld, _stream(stream)))


def aweq_w8a8_gemm_fused(xq, T, K, wq, N, act_step, act_zero, step_w, zero_w, rowsum_x, rowsum_w, bias, act, out_f16, ldo,
                         colsum_acc, ycmin=None, ycmax=None, ycsum=None, ycount=None, accumulate=0, next_inv_s=None,
                         next_step=None, next_zero=None, yq=None, rowsum_y=None, colsum_yq=None, ws=None, status=None,
                         stream=None, ws_bytes=None):
    _check(load_library().aweq_w8a8_gemm_fused(
        _ptr(xq), T, K, _ptr(wq), N, _ptr(act_step), _ptr(act_zero), _ptr(step_w), _ptr(zero_w), _ptr(rowsum_x),
        _ptr(rowsum_w), _ptr(bias), int(act), _ptr(out_f16), ldo, _ptr(colsum_acc), _ptr(ycmin), _ptr(ycmax), _ptr(ycsum),
        _ptr(ycount), int(accumulate), _ptr(next_inv_s), _ptr(next_step), _ptr(next_zero), _ptr(yq), _ptr(rowsum_y),
        _ptr(colsum_yq), _ptr(ws), (_nbytes(ws) if ws is not None else 0) if ws_bytes is None else ws_bytes, _ptr(status),
        _stream(stream)))


def aweq_wonly_gemm(X_hat, T, K, ldx, codes, bits, group, step_w, zero_w, N, bias, out, out_dt, ldo, ws,
                    status=None, stream=None, ws_bytes=None):
    _check(load_library().aweq_wonly_gemm(_ptr(X_hat), T, K, ldx, _ptr(codes), int(bits), int(group), _ptr(step_w),
                                          _ptr(zero_w), N, _ptr(bias), _ptr(out), out_dt, ldo, _ptr(ws),
                                          _nbytes(ws) if ws_bytes is None else ws_bytes, _ptr(status),
                                          _stream(stream)))


def aweq_fold_quant_weight(W, dt, N, K, ldw, s, W_hat, ldwh, bits, codes, step, zero, rowsum_w, status=None, stream=None):
    _check(load_library().aweq_fold_quant_weight(_ptr(W), dt, N, K, ldw, _ptr(s), _ptr(W_hat), ldwh, int(bits), _ptr(codes),
                                                 _ptr(step), _ptr(zero), _ptr(rowsum_w), _ptr(status), _stream(stream)))
