"""ctypes binding of libtweo_hip.so: same names as include/tweo.h, argument marshalling only.

Tensors are torch tensors on the GPU (torch provides device memory and streams,
nothing else); bf16 tensors have dtype torch.bfloat16, E4M3 code tensors
torch.uint8, INT8 tensors torch.int8.  Every call is enqueued on torch's current
stream.  A non-zero status raises TweoError; a missing library raises at load
time - there is no fallback path.
"""
import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libtweo_hip.so")

TWEO_OK, TWEO_ERR_INVALID_ARG, TWEO_ERR_UNSUPPORTED, TWEO_ERR_WORKSPACE, TWEO_ERR_HIP = range(5)
(TWEO_OP_FP8_LINEAR_FWD, TWEO_OP_FP8_LINEAR_BWD, TWEO_OP_W8A8_LINEAR, TWEO_OP_FP8_LINEAR_FWD_BF16,
 TWEO_OP_FP8_LINEAR_BWD_BF16, TWEO_OP_LAYERNORM_QUANTIZE) = range(6)

EXPORTS = ("tweo_workspace_bytes", "tweo_status_string", "tweo_amax", "tweo_quantize_e4m3",
           "tweo_fp8_linear_fwd", "tweo_fp8_linear_bwd", "tweo_quantize_i8", "tweo_w8a8_linear",
           "tweo_fp8_linear_fwd_bf16", "tweo_fp8_linear_bwd_bf16", "tweo_set_gemm_tile",
           "tweo_set_stream_k", "tweo_set_fused_cast", "tweo_fused_cast_timeouts", "tweo_amax_quantize_f8",
           "tweo_penalty_grad_inject", "tweo_delayed_state_bytes",
           "tweo_delayed_state_init", "tweo_quantize_e4m3_delayed", "tweo_profile_gemm_launches",
           "tweo_quantize_e5m2", "tweo_fp8_linear_bwd_hybrid", "tweo_fp8_linear_bwd_bf16_hybrid",
           "tweo_quantize_i8_rows", "tweo_w8a8_linear_scaled", "tweo_w8a8_linear_scaled_i8out",
           "tweo_quantize_e5m2_delayed", "tweo_fp8_linear_bwd_bf16_inject",
           "tweo_fp8_linear_fwd_static", "tweo_static_scratch_bytes",
           "tweo_layernorm_quantize_e4m3", "tweo_layernorm_quantize_e4m3_delayed",
           "tweo_fp8_linear_fwd_bf16_delayed", "tweo_fp8_linear_bwd_bf16_delayed")


class TweoError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: status %d (%s)" % (where, status, status_string(status)))


class PenaltyCfg(ctypes.Structure):
    _fields_ = [("tau", ctypes.c_float), ("eps", ctypes.c_float), ("p", ctypes.c_int)]


class Fp8Saved(ctypes.Structure):
    _fields_ = [("xq", ctypes.c_void_p), ("xqT", ctypes.c_void_p), ("wq", ctypes.c_void_p),
                ("wqT", ctypes.c_void_p), ("scalars", ctypes.c_void_p)]


_lib = None


def load():
    """Loads the HIP library (after torch, so that both share one HIP runtime)."""
    global _lib
    if _lib is not None:
        return _lib
    import torch  # noqa: F401  (loads libamdhip64 first)
    if not os.path.exists(LIB_PATH):
        raise ImportError("%s is missing: run `python -m paper_2511_23225_amd.build` "
                          "(or __graft_entry__.build()) first" % LIB_PATH)
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, f32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
    L.tweo_workspace_bytes.restype = sz
    L.tweo_workspace_bytes.argtypes = [ctypes.c_int, i64, i64, i64]
    L.tweo_status_string.restype = ctypes.c_char_p
    L.tweo_status_string.argtypes = [ctypes.c_int]
    L.tweo_amax.argtypes = [vp, i64, vp, vp]
    L.tweo_quantize_e4m3.argtypes = [vp, i64, i64, vp, vp, vp, vp, vp, vp]
    L.tweo_quantize_e5m2.argtypes = [vp, i64, i64, vp, vp, vp, vp, vp, vp]
    L.tweo_amax_quantize_f8.argtypes = [vp, i64, i64, ctypes.c_int, vp, vp, vp, vp, vp, vp, sz, vp]
    L.tweo_fp8_linear_fwd.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, vp,
                                      ctypes.POINTER(PenaltyCfg), vp, vp, sz, vp]
    L.tweo_fp8_linear_fwd_static.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, vp,
                                             ctypes.POINTER(PenaltyCfg), vp, vp]
    L.tweo_layernorm_quantize_e4m3.argtypes = [vp, vp, vp, vp, i64, i64, f32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.tweo_layernorm_quantize_e4m3_delayed.argtypes = [vp, vp, vp, vp, i64, i64, f32, vp, ctypes.c_int, vp, vp, vp,
                                                       vp, vp, sz, vp]
    L.tweo_fp8_linear_fwd_bf16_delayed.argtypes = [vp, vp, vp, i64, i64, i64, vp, ctypes.POINTER(PenaltyCfg), vp,
                                                   ctypes.POINTER(Fp8Saved), vp, vp, ctypes.c_int, vp, sz, vp]
    L.tweo_fp8_linear_bwd_bf16_delayed.argtypes = [vp, ctypes.POINTER(Fp8Saved), vp, ctypes.c_int, ctypes.c_int, i64,
                                                   i64, i64, vp, vp, vp, vp, vp, sz, vp]
    L.tweo_static_scratch_bytes.argtypes = []
    L.tweo_static_scratch_bytes.restype = ctypes.c_size_t
    L.tweo_fp8_linear_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, vp, vp, vp, sz, vp]
    L.tweo_fp8_linear_bwd_hybrid.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, vp, vp, vp, sz, vp]
    L.tweo_quantize_i8.argtypes = [vp, i64, f32, vp, vp]
    L.tweo_w8a8_linear.argtypes = [vp, vp, i64, i64, i64, f32, vp, vp, sz, vp]
    L.tweo_quantize_i8_rows.argtypes = [vp, i64, i64, f32, vp, vp, vp]
    L.tweo_w8a8_linear_scaled.argtypes = [vp, vp, i64, i64, i64, vp, ctypes.c_int, vp, ctypes.c_int, vp, vp]
    L.tweo_w8a8_linear_scaled_i8out.argtypes = [vp, vp, i64, i64, i64, vp, ctypes.c_int, vp, ctypes.c_int, f32, vp, vp]
    L.tweo_fp8_linear_fwd_bf16.argtypes = [vp, vp, vp, i64, i64, i64, vp, ctypes.POINTER(PenaltyCfg),
                                           vp, ctypes.POINTER(Fp8Saved), vp, sz, vp]
    L.tweo_fp8_linear_bwd_bf16.argtypes = [vp, ctypes.POINTER(Fp8Saved), i64, i64, i64, vp, vp, vp,
                                           vp, vp, sz, vp]
    L.tweo_fp8_linear_bwd_bf16_hybrid.argtypes = L.tweo_fp8_linear_bwd_bf16.argtypes
    L.tweo_fp8_linear_bwd_bf16_inject.argtypes = [vp, vp, ctypes.POINTER(PenaltyCfg), f32, ctypes.c_int,
                                                  ctypes.POINTER(Fp8Saved), i64, i64, i64, vp, vp, vp, vp, vp, sz, vp]
    L.tweo_set_gemm_tile.argtypes = [ctypes.c_int]
    L.tweo_set_stream_k.argtypes = [ctypes.c_int]
    L.tweo_set_fused_cast.argtypes = [ctypes.c_int]
    L.tweo_fused_cast_timeouts.argtypes = [ctypes.POINTER(ctypes.c_uint)]
    L.tweo_profile_gemm_launches.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int]
    L.tweo_delayed_state_bytes.argtypes = []
    L.tweo_delayed_state_bytes.restype = ctypes.c_size_t
    L.tweo_delayed_state_init.argtypes = [vp, vp]
    L.tweo_quantize_e4m3_delayed.argtypes = [vp, i64, i64, vp, ctypes.c_int, vp, vp, vp]
    L.tweo_quantize_e5m2_delayed.argtypes = [vp, i64, i64, vp, ctypes.c_int, vp, vp, vp]
    L.tweo_penalty_grad_inject.argtypes = [vp, vp, i64, ctypes.POINTER(PenaltyCfg), ctypes.c_float, vp, vp]
    for name in EXPORTS:
        if name not in ("tweo_workspace_bytes", "tweo_status_string", "tweo_delayed_state_bytes",
                        "tweo_static_scratch_bytes"):
            getattr(L, name).restype = ctypes.c_int
    _lib = L
    return L


def status_string(status):
    return load().tweo_status_string(int(status)).decode()


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status, where):
    if status != TWEO_OK:
        raise TweoError(status, where)


def _pen(pen):
    if pen is None:
        return None
    tau, eps, p = pen
    return ctypes.byref(PenaltyCfg(float(tau), float(eps), int(p)))


def _ws(workspace):
    if workspace is None:
        return None, 0
    return _ptr(workspace), workspace.numel() * workspace.element_size()


def tweo_workspace_bytes(op, M, N, K):
    return int(load().tweo_workspace_bytes(int(op), int(M), int(N), int(K)))


def tweo_set_gemm_tile(variant):
    _check(load().tweo_set_gemm_tile(int(variant)), "tweo_set_gemm_tile")


def tweo_set_stream_k(on):
    _check(load().tweo_set_stream_k(1 if on else 0), "tweo_set_stream_k")


def tweo_amax_quantize_f8(x_bf16, amax_out, q, qT, scale_out, scale_inv_out, workspace, e5m2=False):
    rows, cols = x_bf16.shape
    wp, wb = _ws(workspace)
    _check(load().tweo_amax_quantize_f8(_ptr(x_bf16), rows, cols, 1 if e5m2 else 0, _ptr(amax_out), _ptr(q), _ptr(qT),
                                        _ptr(scale_out), _ptr(scale_inv_out), wp, wb, _stream()),
           "tweo_amax_quantize_f8")


def tweo_set_fused_cast(on):
    _check(load().tweo_set_fused_cast(1 if on else 0), "tweo_set_fused_cast")


def tweo_fused_cast_timeouts():
    c = ctypes.c_uint(0)
    _check(load().tweo_fused_cast_timeouts(ctypes.byref(c)), "tweo_fused_cast_timeouts")
    return int(c.value)


def tweo_profile_gemm_launches(events):
    """events: flat list of hipEvent_t handles (ints), start/stop per upcoming GEMM kernel launch."""
    n = len(events)
    arr = (ctypes.c_void_p * max(n, 1))(*[ctypes.c_void_p(int(e)) for e in events])
    _check(load().tweo_profile_gemm_launches(arr, n // 2), "tweo_profile_gemm_launches")


def tweo_penalty_grad_inject(dy_bf16, a_bf16, pen, g, out_bf16):
    cfg = PenaltyCfg(float(pen[0]), float(pen[1]), int(pen[2]))
    _check(load().tweo_penalty_grad_inject(_ptr(dy_bf16), _ptr(a_bf16), dy_bf16.numel(), ctypes.byref(cfg),
                                           float(g), _ptr(out_bf16), _stream()), "tweo_penalty_grad_inject")


DELAYED_STATE_WORDS, DELAYED_NEXT_SCALE, DELAYED_USED_SCALE, DELAYED_USED_SCALE_INV = 32, 17, 21, 22


def tweo_delayed_state_bytes():
    return int(load().tweo_delayed_state_bytes())


def tweo_delayed_state_init(state):
    _check(load().tweo_delayed_state_init(_ptr(state), _stream()), "tweo_delayed_state_init")


def tweo_quantize_e4m3_delayed(x_bf16, state, q, qT=None, bootstrap=False):
    rows, cols = x_bf16.shape
    _check(load().tweo_quantize_e4m3_delayed(_ptr(x_bf16), rows, cols, _ptr(state), 1 if bootstrap else 0,
                                             _ptr(q), _ptr(qT), _stream()), "tweo_quantize_e4m3_delayed")


def tweo_quantize_e5m2_delayed(x_bf16, state, q, qT=None, bootstrap=False):
    rows, cols = x_bf16.shape
    _check(load().tweo_quantize_e5m2_delayed(_ptr(x_bf16), rows, cols, _ptr(state), 1 if bootstrap else 0,
                                             _ptr(q), _ptr(qT), _stream()), "tweo_quantize_e5m2_delayed")


def tweo_amax(x_bf16, amax_out):
    _check(load().tweo_amax(_ptr(x_bf16), x_bf16.numel(), _ptr(amax_out), _stream()), "tweo_amax")


def tweo_quantize_e4m3(x_bf16, amax, q, qT=None, scale_out=None, scale_inv_out=None):
    rows, cols = x_bf16.shape
    _check(load().tweo_quantize_e4m3(_ptr(x_bf16), rows, cols, _ptr(amax), _ptr(q), _ptr(qT),
                                     _ptr(scale_out), _ptr(scale_inv_out), _stream()),
           "tweo_quantize_e4m3")


def tweo_quantize_e5m2(x_bf16, amax, q, qT=None, scale_out=None, scale_inv_out=None):
    rows, cols = x_bf16.shape
    _check(load().tweo_quantize_e5m2(_ptr(x_bf16), rows, cols, _ptr(amax), _ptr(q), _ptr(qT),
                                     _ptr(scale_out), _ptr(scale_inv_out), _stream()),
           "tweo_quantize_e5m2")


def tweo_fp8_linear_fwd(xq, sx_inv, wq, sw_inv, y_bf16, residual_bf16=None, pen=None,
                        penalty_sum=None, workspace=None):
    M, K = xq.shape
    N = wq.shape[0]
    wp, wb = _ws(workspace)
    _check(load().tweo_fp8_linear_fwd(_ptr(xq), _ptr(sx_inv), _ptr(wq), _ptr(sw_inv),
                                      _ptr(residual_bf16), M, N, K, _ptr(y_bf16), _pen(pen),
                                      _ptr(penalty_sum), wp, wb, _stream()), "tweo_fp8_linear_fwd")


def tweo_layernorm_quantize_e4m3(x_bf16, gamma_bf16, q, workspace, beta_bf16=None, residual_bf16=None, eps=1e-5,
                                 h_out_bf16=None, y_out_bf16=None, amax_out=None, qT=None, scale_out=None,
                                 scale_inv_out=None):
    rows, cols = x_bf16.shape
    wp, wb = _ws(workspace)
    _check(load().tweo_layernorm_quantize_e4m3(_ptr(x_bf16), _ptr(residual_bf16), _ptr(gamma_bf16), _ptr(beta_bf16),
                                               rows, cols, float(eps), _ptr(h_out_bf16), _ptr(y_out_bf16),
                                               _ptr(amax_out), _ptr(q), _ptr(qT), _ptr(scale_out),
                                               _ptr(scale_inv_out), wp, wb, _stream()),
           "tweo_layernorm_quantize_e4m3")


def tweo_layernorm_quantize_e4m3_delayed(x_bf16, gamma_bf16, state, q, workspace, bootstrap=False, beta_bf16=None,
                                         residual_bf16=None, eps=1e-5, h_out_bf16=None, y_out_bf16=None, qT=None):
    rows, cols = x_bf16.shape
    wp, wb = _ws(workspace)
    _check(load().tweo_layernorm_quantize_e4m3_delayed(_ptr(x_bf16), _ptr(residual_bf16), _ptr(gamma_bf16),
                                                       _ptr(beta_bf16), rows, cols, float(eps), _ptr(state),
                                                       1 if bootstrap else 0, _ptr(h_out_bf16), _ptr(y_out_bf16),
                                                       _ptr(q), _ptr(qT), wp, wb, _stream()),
           "tweo_layernorm_quantize_e4m3_delayed")


def tweo_fp8_linear_fwd_bf16_delayed(x_bf16, w_bf16, y_bf16, saved, state_x, state_w, bootstrap=False,
                                     residual_bf16=None, pen=None, penalty_sum=None, workspace=None):
    M, K = x_bf16.shape
    N = w_bf16.shape[0]
    wp, wb = _ws(workspace)
    _check(load().tweo_fp8_linear_fwd_bf16_delayed(_ptr(x_bf16), _ptr(w_bf16), _ptr(residual_bf16), M, N, K,
                                                   _ptr(y_bf16), _pen(pen), _ptr(penalty_sum), ctypes.byref(saved),
                                                   _ptr(state_x), _ptr(state_w), 1 if bootstrap else 0, wp, wb,
                                                   _stream()), "tweo_fp8_linear_fwd_bf16_delayed")


def tweo_fp8_linear_bwd_bf16_delayed(dy_bf16, saved, state_dy, K, dyq, dyqT, dx_bf16=None, dw_bf16=None,
                                     workspace=None, bootstrap=False, dy_e5m2=False):
    M, N = dy_bf16.shape
    wp, wb = _ws(workspace)
    _check(load().tweo_fp8_linear_bwd_bf16_delayed(_ptr(dy_bf16), ctypes.byref(saved), _ptr(state_dy),
                                                   1 if bootstrap else 0, 1 if dy_e5m2 else 0, M, N, K, _ptr(dyq),
                                                   _ptr(dyqT), _ptr(dx_bf16), _ptr(dw_bf16), wp, wb, _stream()),
           "tweo_fp8_linear_bwd_bf16_delayed")


def tweo_static_scratch_bytes():
    return int(load().tweo_static_scratch_bytes())


def tweo_fp8_linear_fwd_static(xq, sx_inv, wq, sw_inv, y_bf16, residual_bf16=None, pen=None, penalty_sum=None):
    M, K = xq.shape
    N = wq.shape[0]
    _check(load().tweo_fp8_linear_fwd_static(_ptr(xq), _ptr(sx_inv), _ptr(wq), _ptr(sw_inv),
                                             _ptr(residual_bf16), M, N, K, _ptr(y_bf16), _pen(pen),
                                             _ptr(penalty_sum), _stream()), "tweo_fp8_linear_fwd_static")


def tweo_fp8_linear_bwd(dyq, dyqT, sdy_inv, wqT, sw_inv, xqT, sx_inv, M, N, K, dx_bf16=None,
                        dw_bf16=None, workspace=None):
    wp, wb = _ws(workspace)
    _check(load().tweo_fp8_linear_bwd(_ptr(dyq), _ptr(dyqT), _ptr(sdy_inv), _ptr(wqT), _ptr(sw_inv),
                                      _ptr(xqT), _ptr(sx_inv), M, N, K, _ptr(dx_bf16), _ptr(dw_bf16),
                                      wp, wb, _stream()), "tweo_fp8_linear_bwd")


def tweo_fp8_linear_bwd_hybrid(dyq, dyqT, sdy_inv, wqT, sw_inv, xqT, sx_inv, M, N, K, dx_bf16=None,
                               dw_bf16=None, workspace=None):
    wp, wb = _ws(workspace)
    _check(load().tweo_fp8_linear_bwd_hybrid(_ptr(dyq), _ptr(dyqT), _ptr(sdy_inv), _ptr(wqT), _ptr(sw_inv),
                                             _ptr(xqT), _ptr(sx_inv), M, N, K, _ptr(dx_bf16), _ptr(dw_bf16),
                                             wp, wb, _stream()), "tweo_fp8_linear_bwd_hybrid")


def tweo_quantize_i8(x_bf16, inv_step, out):
    _check(load().tweo_quantize_i8(_ptr(x_bf16), x_bf16.numel(), float(inv_step), _ptr(out),
                                   _stream()), "tweo_quantize_i8")


def tweo_w8a8_linear(xq, wq, alpha, y_bf16, workspace=None):
    M, K = xq.shape
    N = wq.shape[0]
    wp, wb = _ws(workspace)
    _check(load().tweo_w8a8_linear(_ptr(xq), _ptr(wq), M, N, K, float(alpha), _ptr(y_bf16), wp, wb,
                                   _stream()), "tweo_w8a8_linear")


def tweo_quantize_i8_rows(x_bf16, eps, q, step_out):
    rows, cols = x_bf16.shape
    _check(load().tweo_quantize_i8_rows(_ptr(x_bf16), rows, cols, float(eps), _ptr(q), _ptr(step_out),
                                        _stream()), "tweo_quantize_i8_rows")


def tweo_w8a8_linear_scaled(xq, wq, x_step, w_step, y_bf16):
    """x_step holds M steps (per token) or 1 (per tensor); w_step N (per channel) or 1."""
    M, K = xq.shape
    N = wq.shape[0]
    if x_step.numel() not in (1, M) or w_step.numel() not in (1, N):
        raise ValueError("step vectors must have 1 or M / N elements")
    _check(load().tweo_w8a8_linear_scaled(_ptr(xq), _ptr(wq), M, N, K, _ptr(x_step),
                                          1 if x_step.numel() > 1 else 0,
                                          _ptr(w_step), 1 if w_step.numel() > 1 else 0, _ptr(y_bf16),
                                          _stream()), "tweo_w8a8_linear_scaled")


def tweo_w8a8_linear_scaled_i8out(xq, wq, x_step, w_step, inv_step_out, yq):
    """INT8 result with the static step 1 / inv_step_out * 127 (quantised residual stream)."""
    M, K = xq.shape
    N = wq.shape[0]
    if x_step.numel() not in (1, M) or w_step.numel() not in (1, N):
        raise ValueError("step vectors must have 1 or M / N elements")
    _check(load().tweo_w8a8_linear_scaled_i8out(_ptr(xq), _ptr(wq), M, N, K, _ptr(x_step),
                                                1 if x_step.numel() > 1 else 0, _ptr(w_step),
                                                1 if w_step.numel() > 1 else 0, float(inv_step_out), _ptr(yq),
                                                _stream()), "tweo_w8a8_linear_scaled_i8out")


def make_saved(xq, xqT, wq, wqT, scalars):
    return Fp8Saved(xq.data_ptr(), xqT.data_ptr(), wq.data_ptr(), wqT.data_ptr(), scalars.data_ptr())


def tweo_fp8_linear_fwd_bf16(x_bf16, w_bf16, y_bf16, saved, residual_bf16=None, pen=None,
                             penalty_sum=None, workspace=None):
    M, K = x_bf16.shape
    N = w_bf16.shape[0]
    wp, wb = _ws(workspace)
    _check(load().tweo_fp8_linear_fwd_bf16(_ptr(x_bf16), _ptr(w_bf16), _ptr(residual_bf16), M, N, K,
                                           _ptr(y_bf16), _pen(pen), _ptr(penalty_sum),
                                           ctypes.byref(saved), wp, wb, _stream()),
           "tweo_fp8_linear_fwd_bf16")


def tweo_fp8_linear_bwd_bf16(dy_bf16, saved, K, dyq, dyqT, dx_bf16=None, dw_bf16=None,
                             workspace=None):
    M, N = dy_bf16.shape
    wp, wb = _ws(workspace)
    _check(load().tweo_fp8_linear_bwd_bf16(_ptr(dy_bf16), ctypes.byref(saved), M, N, K, _ptr(dyq),
                                           _ptr(dyqT), _ptr(dx_bf16), _ptr(dw_bf16), wp, wb,
                                           _stream()), "tweo_fp8_linear_bwd_bf16")


def tweo_fp8_linear_bwd_bf16_inject(dy_bf16, a_bf16, pen, g, saved, K, dyq, dyqT, dx_bf16=None, dw_bf16=None,
                                    workspace=None, dy_e5m2=False):
    M, N = dy_bf16.shape
    wp, wb = _ws(workspace)
    cfg = PenaltyCfg(float(pen[0]), float(pen[1]), int(pen[2]))
    _check(load().tweo_fp8_linear_bwd_bf16_inject(_ptr(dy_bf16), _ptr(a_bf16), ctypes.byref(cfg), float(g),
                                                  1 if dy_e5m2 else 0, ctypes.byref(saved), M, N, K, _ptr(dyq),
                                                  _ptr(dyqT), _ptr(dx_bf16), _ptr(dw_bf16), wp, wb, _stream()),
           "tweo_fp8_linear_bwd_bf16_inject")


def tweo_fp8_linear_bwd_bf16_hybrid(dy_bf16, saved, K, dyq, dyqT, dx_bf16=None, dw_bf16=None,
                                    workspace=None):
    M, N = dy_bf16.shape
    wp, wb = _ws(workspace)
    _check(load().tweo_fp8_linear_bwd_bf16_hybrid(_ptr(dy_bf16), ctypes.byref(saved), M, N, K, _ptr(dyq),
                                                  _ptr(dyqT), _ptr(dx_bf16), _ptr(dw_bf16), wp, wb,
                                                  _stream()), "tweo_fp8_linear_bwd_bf16_hybrid")
