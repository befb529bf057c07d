"""numpy front-end of the CPU oracle (oracle/aweq_oracle.c).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may import this.  It marshals numpy arrays into the C
functions and returns numpy arrays; it contains no arithmetic of the method itself.

Matrices are row-major numpy arrays of dtype float32 or float16; the section / equation
each function follows is cited on the C side.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

ST_DEGENERATE, ST_NONFINITE, ST_BIGQUOT, ST_SCALEGUARD = 1, 2, 4, 8


def lib():
    global _LIB
    if _LIB is None:
        path = os.path.join(_HERE, "liboracle.so")
        src = os.path.join(_HERE, "aweq_oracle.c")
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(src):
            from oracle.build import build
            build()
        _LIB = C.CDLL(path)
        _LIB.orc_h2f.restype = C.c_float
        _LIB.orc_h2f.argtypes = [C.c_uint16]
        _LIB.orc_f2h.restype = C.c_uint16
        _LIB.orc_f2h.argtypes = [C.c_float]
        _LIB.orc_num_threads.restype = C.c_int
    return _LIB


def _dt(a):
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.float16:
        return 1
    raise TypeError(f"unsupported dtype {a.dtype}")


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _c(a, dtype=None):
    a = np.ascontiguousarray(a) if dtype is None else np.ascontiguousarray(a, dtype=dtype)
    return a


i64 = C.c_int64


def num_threads():
    return int(lib().orc_num_threads())


def h2f(h_bits):
    h = _c(h_bits, np.uint16)
    out = np.empty(h.shape, np.float32)
    lib().orc_h2f_array(_p(h), _p(out), i64(h.size))
    return out


def f2h(f):
    f = _c(f, np.float32)
    out = np.empty(f.shape, np.uint16)
    lib().orc_f2h_array(_p(f), _p(out), i64(f.size))
    return out


def col_stats(M, prev=None, want_sum=True):
    """-> dict(cmin, cmax, csum, count, status).  prev = an earlier result to continue from."""
    M = _c(M)
    rows, K = M.shape
    if prev is None:
        cmin = np.empty(K, np.float32)
        cmax = np.empty(K, np.float32)
        csum = np.zeros(K, np.float64) if want_sum else None
        count = C.c_uint64(0)
        acc = 0
    else:
        cmin, cmax = prev["cmin"].copy(), prev["cmax"].copy()
        csum = prev["csum"].copy() if (want_sum and prev["csum"] is not None) else None
        count = C.c_uint64(prev["count"])
        acc = 1
    st = C.c_uint32(0)
    lib().orc_col_stats(_p(M), _dt(M), i64(rows), i64(K), i64(K), _p(cmin), _p(cmax), _p(csum),
                        C.byref(count), acc, C.byref(st))
    return dict(cmin=cmin, cmax=cmax, csum=csum, count=int(count.value), status=int(st.value))


def ranges(cmin, cmax):
    """-> r[K], R, p[K]  (Eq. 4)."""
    cmin, cmax = _c(cmin, np.float32), _c(cmax, np.float32)
    K = cmin.size
    r = np.empty(K, np.float32)
    p = np.empty(K, np.float32)
    R = C.c_float(0)
    lib().orc_ranges(_p(cmin), _p(cmax), i64(K), _p(r), C.byref(R), _p(p))
    return r, np.float32(R.value), p


def scales(r_x, r_w, enable_awe=True):
    """-> s[K], inv_s[K], status  (Eq. 10)."""
    r_x, r_w = _c(r_x, np.float32), _c(r_w, np.float32)
    K = r_x.size
    s = np.empty(K, np.float32)
    inv_s = np.empty(K, np.float32)
    st = C.c_uint32(0)
    lib().orc_scales(_p(r_x), _p(r_w), i64(K), int(bool(enable_awe)), _p(s), _p(inv_s), C.byref(st))
    return s, inv_s, int(st.value)


def channel_absmax(cmin, cmax):
    """-> m[K] = max(|cmin|, |cmax|): the abs-max difficulty variant's channel quantity."""
    cmin, cmax = _c(cmin, np.float32), _c(cmax, np.float32)
    m = np.empty(cmin.size, np.float32)
    lib().orc_channel_absmax(_p(cmin), _p(cmax), i64(cmin.size), _p(m))
    return m


def fold_weight(W, s):
    W = _c(W)
    N, K = W.shape
    out = np.empty_like(W)
    lib().orc_fold_weight(_p(W), _dt(W), i64(N), i64(K), i64(K), _p(_c(s, np.float32)), _p(out), i64(K))
    return out


def fold_act(X, inv_s):
    X = _c(X)
    T, K = X.shape
    out = np.empty((T, K), np.float32)
    lib().orc_fold_act(_p(X), _dt(X), i64(T), i64(K), i64(K), _p(_c(inv_s, np.float32)), _p(out))
    return out


def xhat_stats(xmin, xmax, xsum, count, inv_s):
    """-> xhat_min, xhat_max, mu_xhat[K]."""
    xmin, xmax = _c(xmin, np.float32), _c(xmax, np.float32)
    xsum = _c(xsum, np.float64)
    inv_s = _c(inv_s, np.float32)
    K = xmin.size
    mu = np.empty(K, np.float32)
    lo, hi = C.c_float(0), C.c_float(0)
    lib().orc_xhat_stats(_p(xmin), _p(xmax), _p(xsum), C.c_uint64(count), _p(inv_s), i64(K),
                         C.byref(lo), C.byref(hi), _p(mu))
    return np.float32(lo.value), np.float32(hi.value), mu


def qparams(lo, hi, bits):
    """-> Step (float32), Z (int), status  (Eq. 2 and the zero point)."""
    step, zero, st = C.c_float(0), C.c_int32(0), C.c_uint32(0)
    lib().orc_qparams(C.c_float(lo), C.c_float(hi), int(bits), C.byref(step), C.byref(zero), C.byref(st))
    return np.float32(step.value), int(zero.value), int(st.value)


def quant_values(x, step, zero, bits):
    """Eq. 1 on a flat float32 array -> unsigned codes (int32), status."""
    x = _c(x, np.float32)
    u = np.empty(x.shape, np.int32)
    st = C.c_uint32(0)
    lib().orc_quant_values(_p(x), i64(x.size), C.c_float(step), C.c_int32(zero), int(bits), _p(u), C.byref(st))
    return u, int(st.value)


def dequant_values(u, step, zero):
    u = _c(u, np.int32)
    x = np.empty(u.shape, np.float32)
    lib().orc_dequant_values(_p(u), i64(u.size), C.c_float(step), C.c_int32(zero), _p(x))
    return x


def quant_weight(W_hat, bits, group):
    """-> dict(codes_u uint8[N,K], step, zero, rowsum_w (bits==8), status).

    group 0: per row; g>0: per g along K (step/zero shaped [N, K/g]); -1: per tensor."""
    W_hat = _c(W_hat)
    N, K = W_hat.shape
    if group > 0:
        assert K % group == 0
        shape = (N, K // group)
    elif group == 0:
        shape = (N,)
    else:
        shape = (1,)
    codes = np.empty((N, K), np.uint8)
    step = np.empty(shape, np.float32)
    zero = np.empty(shape, np.int32)
    rowsum = np.empty(N, np.int32) if bits == 8 else None
    st = C.c_uint32(0)
    lib().orc_quant_weight(_p(W_hat), _dt(W_hat), i64(N), i64(K), i64(K), int(bits), i64(group),
                           _p(codes), _p(step), _p(zero), _p(rowsum), C.byref(st))
    return dict(codes_u=codes, step=step, zero=zero, rowsum_w=rowsum, status=int(st.value))


def packed_size(N, K, bits):
    return N * K * bits // 8


def pack_codes(codes_u, bits):
    codes_u = _c(codes_u, np.uint8)
    N, K = codes_u.shape
    out = np.empty(packed_size(N, K, bits), np.uint8)
    lib().orc_pack_codes(_p(codes_u), i64(N), i64(K), int(bits), _p(out))
    if bits == 8:
        return out.view(np.int8).reshape(N, K)
    return out.reshape(N, -1)


def unpack_codes(packed, N, K, bits):
    packed = _c(packed).view(np.uint8).reshape(-1)
    out = np.empty((N, K), np.uint8)
    lib().orc_unpack_codes(_p(packed), i64(N), i64(K), int(bits), _p(out))
    return out


def dequant_weight(codes_u, group, step, zero):
    codes_u = _c(codes_u, np.uint8)
    N, K = codes_u.shape
    out = np.empty((N, K), np.float32)
    lib().orc_dequant_weight(_p(codes_u), i64(N), i64(K), i64(group), _p(_c(step, np.float32)),
                             _p(_c(zero, np.int32)), _p(out))
    return out


def dequant_weight_h(codes_u, group, step, zero):
    """-> binary16 W-tilde as the weight-only forward consumes it (Step rounded to binary16)."""
    codes_u = _c(codes_u, np.uint8)
    N, K = codes_u.shape
    out = np.empty((N, K), np.float16)
    lib().orc_dequant_weight_h(_p(codes_u), i64(N), i64(K), i64(group), _p(_c(step, np.float32)),
                               _p(_c(zero, np.int32)), _p(out))
    return out


def wonly_forward(X_hat_h, W_tilde_h, bias=None):
    """-> (y fp64 [T,N], abs_y fp64 [T,N]) for binary16 operands."""
    X_hat_h = _c(X_hat_h, np.float16)
    W_tilde_h = _c(W_tilde_h, np.float16)
    T, K = X_hat_h.shape
    N = W_tilde_h.shape[0]
    y = np.empty((T, N), np.float64)
    a = np.empty((T, N), np.float64)
    b = None if bias is None else _c(bias, np.float32)
    lib().orc_wonly_forward(_p(X_hat_h), i64(T), i64(K), i64(K), _p(W_tilde_h), i64(N),
                            _p(b) if b is not None else None, _p(y), _p(a))
    return y, a


def quant_act(X, inv_s, step_x, zero_x):
    """-> dict(xq int8[T,K], rowsum_x int32[T], colsum_xq int64[K], status)."""
    X = _c(X)
    T, K = X.shape
    xq = np.empty((T, K), np.int8)
    rs = np.empty(T, np.int32)
    cs = np.empty(K, np.int64)
    st = C.c_uint32(0)
    lib().orc_quant_act(_p(X), _dt(X), i64(T), i64(K), i64(K), _p(_c(inv_s, np.float32)),
                        C.c_float(step_x), C.c_int32(zero_x), _p(xq), _p(rs), _p(cs), C.byref(st))
    return dict(xq=xq, rowsum_x=rs, colsum_xq=cs, status=int(st.value))


def gemm_i8(xq, wq):
    xq, wq = _c(xq, np.int8), _c(wq, np.int8)
    T, K = xq.shape
    N = wq.shape[0]
    assert wq.shape[1] == K
    acc = np.empty((T, N), np.int32)
    lib().orc_gemm_i8(_p(xq), _p(wq), i64(T), i64(N), i64(K), _p(acc))
    return acc


def w8a8_output_direct(xq, wq, step_x, zero_x, step_w, zero_w, bias=None):
    xq, wq = _c(xq, np.int8), _c(wq, np.int8)
    T, K = xq.shape
    N = wq.shape[0]
    out = np.empty((T, N), np.float64)
    b = None if bias is None else _c(bias, np.float32)
    lib().orc_w8a8_output_direct(_p(xq), _p(wq), i64(T), i64(N), i64(K), C.c_float(step_x),
                                 C.c_int32(zero_x), _p(_c(step_w, np.float32)),
                                 _p(_c(zero_w, np.int32)), _p(b), _p(out))
    return out


def w8a8_output_expanded(acc, rowsum_x, rowsum_w, K, step_x, zero_x, step_w, zero_w, bias=None):
    acc = _c(acc, np.int32)
    T, N = acc.shape
    out = np.empty((T, N), np.float64)
    integer = np.empty((T, N), np.int64)
    b = None if bias is None else _c(bias, np.float32)
    lib().orc_w8a8_output_expanded(_p(acc), _p(_c(rowsum_x, np.int32)), _p(_c(rowsum_w, np.int32)),
                                   i64(T), i64(N), i64(K), C.c_float(step_x), C.c_int32(zero_x),
                                   _p(_c(step_w, np.float32)), _p(_c(zero_w, np.int32)), _p(b),
                                   _p(out), _p(integer))
    return out, integer


def bias_literal_w8a8(X, inv_s, W_hat, xq, wq, step_x, zero_x, step_w, zero_w, bias_in=None):
    """Eq. 11 token by token -> delta (float64[N]), bias_out (float32[N])."""
    X, W_hat = _c(X), _c(W_hat)
    assert X.dtype == W_hat.dtype
    T, K = X.shape
    N = W_hat.shape[0]
    delta = np.empty(N, np.float64)
    bout = np.empty(N, np.float32)
    b = None if bias_in is None else _c(bias_in, np.float32)
    lib().orc_bias_literal_w8a8(_p(X), _dt(X), i64(T), i64(K), i64(K), _p(_c(inv_s, np.float32)),
                                _p(W_hat), i64(N), i64(K), _p(_c(xq, np.int8)), _p(_c(wq, np.int8)),
                                C.c_float(step_x), C.c_int32(zero_x), _p(_c(step_w, np.float32)),
                                _p(_c(zero_w, np.int32)), _p(b), _p(delta), _p(bout))
    return delta, bout


def bias_literal_wonly(X, inv_s, W_hat, W_tilde, bias_in=None):
    X, W_hat = _c(X), _c(W_hat)
    assert X.dtype == W_hat.dtype
    T, K = X.shape
    N = W_hat.shape[0]
    delta = np.empty(N, np.float64)
    bout = np.empty(N, np.float32)
    b = None if bias_in is None else _c(bias_in, np.float32)
    lib().orc_bias_literal_wonly(_p(X), _dt(X), i64(T), i64(K), i64(K), _p(_c(inv_s, np.float32)),
                                 _p(W_hat), i64(N), i64(K), _p(_c(W_tilde, np.float32)), _p(b),
                                 _p(delta), _p(bout))
    return delta, bout


def bias_w8a8(W_hat, mu_xhat, count, colsum_acc, colsum_xq, rowsum_w, step_x, zero_x, step_w, zero_w,
              bias_in=None, enable_bc=True):
    W_hat = _c(W_hat)
    N, K = W_hat.shape
    delta = np.empty(N, np.float64)
    bout = np.empty(N, np.float32)
    b = None if bias_in is None else _c(bias_in, np.float32)
    lib().orc_bias_w8a8(_p(W_hat), _dt(W_hat), i64(N), i64(K), i64(K), _p(_c(mu_xhat, np.float32)),
                        C.c_uint64(count), _p(_c(colsum_acc, np.int64)), _p(_c(colsum_xq, np.int64)),
                        _p(_c(rowsum_w, np.int32)), C.c_float(step_x), C.c_int32(zero_x),
                        _p(_c(step_w, np.float32)), _p(_c(zero_w, np.int32)), _p(b),
                        int(bool(enable_bc)), _p(delta), _p(bout))
    return delta, bout


def bias_wonly(W_hat, mu_xhat, codes_u, group, step_w, zero_w, bias_in=None, enable_bc=True):
    W_hat = _c(W_hat)
    N, K = W_hat.shape
    delta = np.empty(N, np.float64)
    bout = np.empty(N, np.float32)
    b = None if bias_in is None else _c(bias_in, np.float32)
    lib().orc_bias_wonly(_p(W_hat), _dt(W_hat), i64(N), i64(K), i64(K), _p(_c(mu_xhat, np.float32)),
                         _p(_c(codes_u, np.uint8)), i64(group), _p(_c(step_w, np.float32)),
                         _p(_c(zero_w, np.int32)), _p(b), int(bool(enable_bc)), _p(delta), _p(bout))
    return delta, bout


def colsum_acc_from_colsum_xq(wq, colsum_xq):
    wq = _c(wq, np.int8)
    N, K = wq.shape
    out = np.empty(N, np.int64)
    lib().orc_colsum_acc_from_colsum_xq(_p(wq), i64(N), i64(K), _p(_c(colsum_xq, np.int64)), _p(out))
    return out
