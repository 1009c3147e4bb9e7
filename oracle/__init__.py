"""numpy front end of the CPU oracle (oracle/tweo_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
cpu_baseline leg of bench.py.  Nothing in the product package imports it and it
imports nothing from the product package.  bf16 tensors travel as uint16 bit
patterns, E4M3 tensors as uint8 codes.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tweo_oracle.c")
_LIB = os.path.join(_HERE, "libtweo_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc (plain scalar C, OpenMP over independent rows)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-std=c11",
           "-Wall", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ct))


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.orc_bf16_to_f32.restype = ctypes.c_float
        L.orc_bf16_to_f32.argtypes = [ctypes.c_uint16]
        L.orc_f32_to_bf16.restype = ctypes.c_uint16
        L.orc_f32_to_bf16.argtypes = [ctypes.c_float]
        L.orc_e4m3_decode.restype = ctypes.c_double
        L.orc_e4m3_decode.argtypes = [ctypes.c_uint8]
        L.orc_e4m3_encode.restype = ctypes.c_uint8
        L.orc_e4m3_encode.argtypes = [ctypes.c_float]
        L.orc_e5m2_decode.restype = ctypes.c_double
        L.orc_e5m2_decode.argtypes = [ctypes.c_uint8]
        L.orc_e5m2_encode.restype = ctypes.c_uint8
        L.orc_e5m2_encode.argtypes = [ctypes.c_float]
        L.orc_amax_bf16.restype = ctypes.c_float
        L.orc_penalty_sum.restype = ctypes.c_double
        L.orc_num_threads.restype = ctypes.c_int
        L.orc_f64_to_bf16.restype = ctypes.c_uint16
        L.orc_f64_to_bf16.argtypes = [ctypes.c_double]
        _lib = L
    return _lib


_u8, _u16, _i8, _i32, _i64 = (ctypes.c_uint8, ctypes.c_uint16, ctypes.c_int8, ctypes.c_int32,
                              ctypes.c_int64)
_f32, _f64 = ctypes.c_float, ctypes.c_double


def _c(a, dt):
    a = np.ascontiguousarray(a)
    assert a.dtype == dt, (a.dtype, dt)
    return a


def num_threads():
    return int(lib().orc_num_threads())


def bf16_to_f32(h):
    """uint16 patterns -> float32 (exact)."""
    h = np.asarray(h, dtype=np.uint16)
    if h.ndim == 0:
        return np.float32(lib().orc_bf16_to_f32(int(h)))
    return (h.astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_bf16_scalar(f):
    return int(lib().orc_f32_to_bf16(ctypes.c_float(float(f))))


def e4m3_decode(b):
    return float(lib().orc_e4m3_decode(int(b)))


def e4m3_encode(v):
    return int(lib().orc_e4m3_encode(ctypes.c_float(float(v))))


def e5m2_decode(b):
    return float(lib().orc_e5m2_decode(int(b)))


def e5m2_encode(v):
    return int(lib().orc_e5m2_encode(ctypes.c_float(float(v))))


def amax_bf16(x):
    x = _c(x, np.uint16)
    return np.float32(lib().orc_amax_bf16(_p(x, _u16), _i64(x.size)))


def scale_from_amax(amax):
    s, si = _f32(), _f32()
    lib().orc_scale_from_amax(_f32(float(amax)), ctypes.byref(s), ctypes.byref(si))
    return np.float32(s.value), np.float32(si.value)


def scale_from_amax_e5m2(amax):
    s, si = _f32(), _f32()
    lib().orc_scale_from_amax_e5m2(_f32(float(amax)), ctypes.byref(s), ctypes.byref(si))
    return np.float32(s.value), np.float32(si.value)


def quantize_e5m2(x, scale, transpose=True):
    x = _c(x, np.uint16)
    assert x.ndim == 2
    r, c = x.shape
    q = np.empty((r, c), np.uint8)
    qT = np.empty((c, r), np.uint8) if transpose else None
    lib().orc_quantize_e5m2(_p(x, _u16), _i64(r), _i64(c), _f32(float(scale)), _p(q, _u8),
                            _p(qT, _u8))
    return q, qT


def quantize_e4m3(x, scale, transpose=True):
    x = _c(x, np.uint16)
    assert x.ndim == 2
    r, c = x.shape
    q = np.empty((r, c), np.uint8)
    qT = np.empty((c, r), np.uint8) if transpose else None
    lib().orc_quantize_e4m3(_p(x, _u16), _i64(r), _i64(c), _f32(float(scale)), _p(q, _u8),
                            _p(qT, _u8))
    return q, qT


def _rows(rows, limit):
    if rows is None:
        return None, 0
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    assert rows.ndim == 1 and (rows >= 0).all() and (rows < limit).all()
    return rows, rows.size


def fp8_linear_fwd(xq, wq, sx_inv, sw_inv, residual=None, rows=None, want_abs=True):
    """Returns (y64, yabs, ybf16) for all rows m, or for the rows listed in `rows`."""
    xq, wq = _c(xq, np.uint8), _c(wq, np.uint8)
    M, K = xq.shape
    N, K2 = wq.shape
    assert K == K2
    if residual is not None:
        residual = _c(residual, np.uint16)
        assert residual.shape == (M, N)
    rows, nr = _rows(rows, M)
    R = nr if rows is not None else M
    y = np.empty((R, N), np.float64)
    ya = np.empty((R, N), np.float64) if want_abs else None
    yb = np.empty((R, N), np.uint16)
    lib().orc_fp8_linear_fwd(_p(xq, _u8), _p(wq, _u8), _p(residual, _u16), _i64(M), _i64(N),
                             _i64(K), _f32(float(sx_inv)), _f32(float(sw_inv)), _p(rows, _i64),
                             _i64(nr), _p(y, _f64), _p(ya, _f64), _p(yb, _u16))
    return y, ya, yb


def fp8_linear_dgrad(dyq, wq, sdy_inv, sw_inv, rows=None, want_abs=True, dy_e5m2=False):
    """dX rows (all m, or those in `rows`): (dx64, dxabs).  dy_e5m2: dyq holds E5M2 codes."""
    dyq, wq = _c(dyq, np.uint8), _c(wq, np.uint8)
    M, N = dyq.shape
    N2, K = wq.shape
    assert N == N2
    rows, nr = _rows(rows, M)
    R = nr if rows is not None else M
    dx = np.empty((R, K), np.float64)
    da = np.empty((R, K), np.float64) if want_abs else None
    lib().orc_fp8_linear_dgrad_fmt(_p(dyq, _u8), _p(wq, _u8), _i64(M), _i64(N), _i64(K),
                                   _f32(float(sdy_inv)), _f32(float(sw_inv)), _p(rows, _i64),
                                   _i64(nr), _p(dx, _f64), _p(da, _f64), ctypes.c_int(1 if dy_e5m2 else 0))
    return dx, da


def fp8_linear_wgrad(dyq, xq, sdy_inv, sx_inv, rows=None, want_abs=True, dy_e5m2=False):
    """dW rows (all n, or those in `rows`): (dw64, dwabs).  dy_e5m2: dyq holds E5M2 codes."""
    dyq, xq = _c(dyq, np.uint8), _c(xq, np.uint8)
    M, N = dyq.shape
    M2, K = xq.shape
    assert M == M2
    rows, nr = _rows(rows, N)
    R = nr if rows is not None else N
    dw = np.empty((R, K), np.float64)
    da = np.empty((R, K), np.float64) if want_abs else None
    lib().orc_fp8_linear_wgrad_fmt(_p(dyq, _u8), _p(xq, _u8), _i64(M), _i64(N), _i64(K),
                                   _f32(float(sdy_inv)), _f32(float(sx_inv)), _p(rows, _i64),
                                   _i64(nr), _p(dw, _f64), _p(da, _f64), ctypes.c_int(1 if dy_e5m2 else 0))
    return dw, da


def penalty_sum(a_bf16, tau=3.0, eps=1e-6, p=4):
    a = _c(a_bf16, np.uint16)
    return float(lib().orc_penalty_sum(_p(a, _u16), _i64(a.size), _f64(tau), _f64(eps),
                                       ctypes.c_int(p)))


def penalty_grad(a_bf16, tau=3.0, eps=1e-6, p=4, g=1.0):
    a = _c(a_bf16, np.uint16)
    out = np.empty(a.shape, np.float64)
    lib().orc_penalty_grad(_p(a, _u16), _i64(a.size), _f64(tau), _f64(eps), ctypes.c_int(p),
                           _f64(g), _p(out, _f64))
    return out


class DelayedScaling:
    """Per-tensor delayed scaling as the paper ran it (Sec. 4.3: amax history of length 16).

    The cast of step t uses 448 / max(amax of steps t-16 .. t-1); the paper names the history
    length, not the reduction over it (reading: the maximum).  An empty history takes the
    tensor's own amax (a current-scaling step).  Plain Python around the scalar routines."""

    LENGTH = 16

    def __init__(self, e5m2=False):
        self.history = []          # most recent last, at most LENGTH entries
        self.next_scale = np.float32(1.0)
        # the gradient tensors of the HYBRID recipe are cast to E5M2 (Sec. 4.3): same history, the
        # scale maps into +-57344 and the cast is the E5M2 one
        self._scale = scale_from_amax_e5m2 if e5m2 else scale_from_amax
        self._quantize = quantize_e5m2 if e5m2 else quantize_e4m3

    def _max(self):
        # maximum on the magnitude bit patterns, like amax itself (NaN above Inf above finite)
        bits = [int(np.float32(a).view(np.uint32)) for a in self.history]
        return np.uint32(max(bits)).view(np.float32) if bits else np.float32(0.0)

    def cast(self, x_bf16, transpose=True):
        """-> (q, qT, scale_used, scale_used_inv); appends this tensor's amax to the history."""
        a = np.float32(amax_bf16(x_bf16))
        if not self.history:                      # bootstrap
            self.history.append(a)
            used, used_inv = self._scale(self._max())
        else:
            used = self.next_scale
            used_inv = np.float32(1.0) / np.float32(used)
            self.history.append(a)
        self.history = self.history[-self.LENGTH:]
        self.next_scale = np.float32(self._scale(self._max())[0])
        qq, qqT = self._quantize(x_bf16, used, transpose=transpose)
        return qq, qqT, np.float32(used), np.float32(used_inv)


def penalty_grad_inject(dy_bf16, a_bf16, tau=3.0, eps=1e-6, p=4, g=1.0):
    """dy + d(penalty)/da rounded to bf16, and the unrounded fp64 sums."""
    dy, a = _c(dy_bf16, np.uint16), _c(a_bf16, np.uint16)
    assert dy.shape == a.shape
    out = np.empty(a.shape, np.uint16)
    exact = np.empty(a.shape, np.float64)
    lib().orc_penalty_grad_inject(_p(dy, _u16), _p(a, _u16), _i64(a.size), _f64(tau), _f64(eps),
                                  ctypes.c_int(p), _f64(g), _p(out, _u16), _p(exact, _f64))
    return out, exact


def quantize_i8(x, inv_step):
    x = _c(x, np.uint16)
    q = np.empty(x.shape, np.int8)
    lib().orc_quantize_i8(_p(x, _u16), _i64(x.size), _f32(float(inv_step)), _p(q, _i8))
    return q


def w8a8_linear(xq, wq, alpha, want_acc=False):
    xq, wq = _c(xq, np.int8), _c(wq, np.int8)
    M, K = xq.shape
    N, K2 = wq.shape
    assert K == K2
    y = np.empty((M, N), np.uint16)
    acc = np.empty((M, N), np.int32) if want_acc else None
    if M < 64 and not want_acc:
        lib().orc_w8a8_linear_small_m(_p(xq, _i8), _p(wq, _i8), _i64(M), _i64(N), _i64(K),
                                      _f32(float(alpha)), _p(y, _u16))
    else:
        lib().orc_w8a8_linear(_p(xq, _i8), _p(wq, _i8), _i64(M), _i64(N), _i64(K),
                              _f32(float(alpha)), _p(y, _u16), _p(acc, _i32))
    return (y, acc) if want_acc else y


def quantize_i8_rows(x, eps=0.0):
    """Row-granular AbsMax (Sec. 4.4, Eq. 4: per-token activations, per-channel weights)."""
    x = _c(x, np.uint16)
    rows, cols = x.shape
    q = np.empty((rows, cols), np.int8)
    step = np.empty(rows, np.float32)
    lib().orc_quantize_i8_rows(_p(x, _u16), _i64(rows), _i64(cols), _f32(float(eps)), _p(q, _i8),
                               _p(step, _f32))
    return q, step


def w8a8_linear_scaled(xq, wq, sx, sw):
    """y = bf16((fp32(acc) * sx[m]) * sw[n]); sx / sw of length 1 mean per-tensor steps."""
    xq, wq = _c(xq, np.int8), _c(wq, np.int8)
    M, K = xq.shape
    N, K2 = wq.shape
    assert K == K2
    sx = _c(np.atleast_1d(sx), np.float32)
    sw = _c(np.atleast_1d(sw), np.float32)
    assert sx.size in (1, M) and sw.size in (1, N)
    y = np.empty((M, N), np.uint16)
    lib().orc_w8a8_linear_scaled(_p(xq, _i8), _p(wq, _i8), _i64(M), _i64(N), _i64(K), _p(sx, _f32),
                                 _i64(0 if sx.size == 1 else 1), _p(sw, _f32),
                                 _i64(0 if sw.size == 1 else 1), _p(y, _u16))
    return y


def w8a8_linear_scaled_i8out(xq, wq, sx, sw, inv_step_out):
    """INT8 output for a quantised residual stream: clamp(rne(((fp32(acc)*sx[m])*sw[n]) * inv_step_out))."""
    xq, wq = _c(xq, np.int8), _c(wq, np.int8)
    M, K = xq.shape
    N, K2 = wq.shape
    assert K == K2
    sx = _c(np.atleast_1d(sx), np.float32)
    sw = _c(np.atleast_1d(sw), np.float32)
    assert sx.size in (1, M) and sw.size in (1, N)
    yq = np.empty((M, N), np.int8)
    lib().orc_w8a8_linear_scaled_i8out(_p(xq, _i8), _p(wq, _i8), _i64(M), _i64(N), _i64(K), _p(sx, _f32),
                                       _i64(0 if sx.size == 1 else 1), _p(sw, _f32),
                                       _i64(0 if sw.size == 1 else 1), _f32(float(inv_step_out)), _p(yq, _i8))
    return yq


def f64_to_bf16_scalar(v):
    return int(lib().orc_f64_to_bf16(ctypes.c_double(float(v))))


def residual_add_bf16(x, r):
    """h = bf16(x + r): the residual-stream update in front of a normalisation."""
    x, r = _c(x, np.uint16), _c(r, np.uint16)
    assert x.shape == r.shape
    h = np.empty(x.shape, np.uint16)
    lib().orc_residual_add_bf16(_p(x, _u16), _p(r, _u16), _i64(x.size), _p(h, _u16))
    return h


def layernorm(h, gamma, beta=None, eps=1e-5):
    """Row-wise LayerNorm in fp64 (Sec. 4.3: LayerNorm runs under FP8 too): (y64, y_bf16)."""
    h, gamma = _c(h, np.uint16), _c(gamma, np.uint16)
    rows, cols = h.shape
    assert gamma.shape == (cols,)
    if beta is not None:
        beta = _c(beta, np.uint16)
        assert beta.shape == (cols,)
    y64 = np.empty((rows, cols), np.float64)
    yb = np.empty((rows, cols), np.uint16)
    lib().orc_layernorm(_p(h, _u16), _p(gamma, _u16), _p(beta, _u16), _i64(rows), _i64(cols),
                        _f64(float(eps)), _p(y64, _f64), _p(yb, _u16))
    return y64, yb
