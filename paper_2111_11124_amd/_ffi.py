"""ctypes binding of libmesa.so: argument marshalling only.

Every function below has the name and the argument order of the C entry point it calls
(include/mesa.h); tensors are torch tensors on the GPU, whose data pointers and current stream are
passed through.  No arithmetic of the method happens in Python, and there is no fallback: if the
shared library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
from pathlib import Path

import torch  # noqa: F401  (first, so that libmesa binds to the HIP runtime torch has loaded)

_LIB_PATH = Path(__file__).resolve().parent / "libmesa.so"

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_LAUNCH = range(5)
F32, F16, BF16 = 0, 1, 2
ROUND_NEAREST_EVEN, ROUND_STOCHASTIC = 0, 1
OP_UPDATE_RUNNING_PARAMS, OP_LAYERNORM_BWD_Q, OP_LINEAR_DW_Q, OP_SOFTMAX_FWD_Q, OP_LAYERNORM_FWD_Q = 0, 1, 2, 3, 4

EXPORTS = [
    "mesa_update_running_params", "mesa_update_running_params_sym", "mesa_update_running_params_fixed_beta", "mesa_update_running_scale_sym", "mesa_quantize_sym", "mesa_dequantize_sym", "mesa_update_running_params_static", "mesa_static_scratch_bytes", "mesa_quantize_headwise", "mesa_quantize_update_fused", "mesa_gelu_fwd_q", "mesa_softmax_fwd_q", "mesa_layernorm_fwd_q", "mesa_dequantize", "mesa_quantize_headwise_b4", "mesa_dequantize_b4", "mesa_gelu_bwd_q_b4", "mesa_softmax_bwd_q",
    "mesa_gelu_bwd_q", "mesa_relu_bwd_q", "mesa_layernorm_bwd_q", "mesa_linear_dw_q", "mesa_conv2d_dw_q", "mesa_conv2d_dw_q_workspace_bytes", "mesa_attn_av_bwd_q", "mesa_attn_qk_bwd_q",
    "mesa_workspace_bytes",
    "mesa_status_string", "mesa_version", "mesa_stream_copy", "mesa_stream_read", "mesa_stream_fill", "mesa_mfma_probe", "mesa_event_create", "mesa_event_record",
    "mesa_event_elapsed_ms", "mesa_event_destroy",
]


class MesaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class Layout(C.Structure):
    _fields_ = [("outer", C.c_int64), ("groups", C.c_int64), ("inner", C.c_int64)]


class Conv2d(C.Structure):
    """mesa_conv2d: the sizes of a convolution, in the header's order"""
    _fields_ = [(n, C.c_int64) for n in ("B", "C_in", "H", "W", "C_out", "KH", "KW", "stride_h", "stride_w", "pad_h", "pad_w",
                                         "dil_h", "dil_w")]

    def out_hw(self):
        return ((self.H + 2 * self.pad_h - self.dil_h * (self.KH - 1) - 1) // self.stride_h + 1,
                (self.W + 2 * self.pad_w - self.dil_w * (self.KW - 1) - 1) // self.stride_w + 1)


_lib = None
_vp, _i64, _u64, _int, _f32, _sz = C.c_void_p, C.c_int64, C.c_uint64, C.c_int, C.c_float, C.c_size_t


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not _LIB_PATH.exists():
            raise RuntimeError(f"{_LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                               "(there is no fallback path)")
        L = C.CDLL(str(_LIB_PATH))
        L.mesa_update_running_params.argtypes = [_vp, _int, Layout, _vp, _vp, _f32, _int, _vp, _sz, _vp]
        L.mesa_update_running_params_sym.argtypes = L.mesa_update_running_params.argtypes
        L.mesa_update_running_params_fixed_beta.argtypes = [_vp, _int, Layout, _vp, _vp, _f32, _int, _f32, _vp, _sz, _vp]
        L.mesa_update_running_scale_sym.argtypes = [_vp, _int, Layout, _vp, _f32, _int, _vp, _sz, _vp]
        L.mesa_quantize_sym.argtypes = [_vp, _int, Layout, _vp, _vp, _int, _u64, _u64, _vp]
        L.mesa_dequantize_sym.argtypes = [_vp, Layout, _vp, _vp, _int, _vp]
        L.mesa_update_running_params_static.argtypes = [_vp, _int, Layout, _vp, _vp, _f32, _int, _vp]
        L.mesa_static_scratch_bytes.argtypes = []
        L.mesa_static_scratch_bytes.restype = _sz
        L.mesa_quantize_headwise.argtypes = [_vp, _int, Layout, _vp, _vp, _vp, _int, _u64, _u64, _vp]
        L.mesa_quantize_update_fused.argtypes = [_vp, _int, Layout, _vp, _vp, _f32, _vp, _int, _u64, _u64, _vp, _sz, _vp]
        L.mesa_gelu_fwd_q.argtypes = [_vp, _int, Layout, _vp, _vp, _f32, _vp, _vp, _int, _u64, _u64, _vp, _sz, _vp]
        L.mesa_softmax_fwd_q.argtypes = [_vp, _i64, _i64, _i64, _i64, _vp, _vp, _f32, _vp, _vp, _int, _u64, _u64, _vp, _sz, _int, _vp]
        L.mesa_layernorm_fwd_q.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _f32, _vp, _vp, _f32, _vp, _vp, _vp, _vp, _int, _u64, _u64,
                                           _vp, _sz, _int, _vp]
        L.mesa_dequantize.argtypes = [_vp, Layout, _vp, _vp, _vp, _int, _vp]
        L.mesa_quantize_headwise_b4.argtypes = L.mesa_quantize_headwise.argtypes
        L.mesa_dequantize_b4.argtypes = L.mesa_dequantize.argtypes
        L.mesa_gelu_bwd_q_b4.argtypes = [_vp, Layout, _vp, _vp, _vp, _vp, _int, _vp]
        L.mesa_softmax_bwd_q.argtypes = [_vp, _i64, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _int, _vp]
        L.mesa_gelu_bwd_q.argtypes = [_vp, Layout, _vp, _vp, _vp, _vp, _int, _vp]
        L.mesa_relu_bwd_q.argtypes = L.mesa_gelu_bwd_q.argtypes
        L.mesa_layernorm_bwd_q.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _int,
                                           _vp, _sz, _vp]
        L.mesa_linear_dw_q.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _vp, _i64, _int, _vp, _vp, _vp, _sz, _vp]
        L.mesa_attn_av_bwd_q.argtypes = [_vp, _vp, _i64, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _int, _vp]
        L.mesa_attn_qk_bwd_q.argtypes = [_vp, _vp, _i64, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _f32, _vp, _vp, _int, _vp]
        L.mesa_workspace_bytes.argtypes = [_int, _i64, _i64, _i64, _int]
        L.mesa_workspace_bytes.restype = _sz
        L.mesa_status_string.argtypes = [_int]
        L.mesa_status_string.restype = C.c_char_p
        L.mesa_version.restype = _int
        L.mesa_stream_copy.argtypes = [_vp, _vp, _sz, _vp]
        L.mesa_stream_read.argtypes = [_vp, _sz, _vp, _vp]
        L.mesa_stream_fill.argtypes = [_vp, _sz, C.c_uint32, _vp]
        L.mesa_mfma_probe.argtypes = [C.c_int, _i64, _vp, _sz, _vp, _vp]
        L.mesa_event_create.argtypes = [C.POINTER(_vp)]
        L.mesa_event_record.argtypes = [_vp, _vp]
        L.mesa_event_elapsed_ms.argtypes = [_vp, _vp, C.POINTER(_f32)]
        L.mesa_event_destroy.argtypes = [_vp]
        L.mesa_conv2d_dw_q.argtypes = [_vp, Conv2d, _i64, _vp, _vp, _vp, _int, _vp, _vp, _vp, _sz, _vp]
        L.mesa_conv2d_dw_q_workspace_bytes.argtypes = [Conv2d, _int]
        L.mesa_conv2d_dw_q_workspace_bytes.restype = _sz
        for name in EXPORTS:
            fn = getattr(L, name)
            if name not in ("mesa_workspace_bytes", "mesa_status_string", "mesa_version", "mesa_static_scratch_bytes",
                            "mesa_conv2d_dw_q_workspace_bytes"):
                fn.restype = _int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().mesa_status_string(int(status)).decode()


def version() -> int:
    return int(lib().mesa_version())


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.float16:
        return F16
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("libmesa takes device tensors only")
    if not t.is_contiguous():
        raise ValueError("libmesa takes contiguous tensors only")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _check(status: int, where: str):
    if status != OK:
        raise MesaError(status, where)


def workspace_bytes(op: int, d0: int, d1: int, d2: int, dtype: int = F16) -> int:
    return int(lib().mesa_workspace_bytes(op, d0, d1, d2, dtype))


def _ws_args(ws):
    return (_ptr(ws), ws.numel() * ws.element_size()) if ws is not None else (None, 0)


def mesa_update_running_params(x, layout, alpha, beta, lam, first_call, ws):
    p, n = _ws_args(ws)
    _check(lib().mesa_update_running_params(_ptr(x), _dt(x), Layout(*layout), _ptr(alpha), _ptr(beta), float(lam),
                                            int(bool(first_call)), p, n, _stream()), "mesa_update_running_params")


def mesa_update_running_params_sym(x, layout, alpha, beta, lam, first_call, ws):
    p, n = _ws_args(ws)
    _check(lib().mesa_update_running_params_sym(_ptr(x), _dt(x), Layout(*layout), _ptr(alpha), _ptr(beta), float(lam),
                                                int(bool(first_call)), p, n, _stream()), "mesa_update_running_params_sym")


def mesa_update_running_params_fixed_beta(x, layout, alpha, beta, lam, first_call, beta_fixed, ws):
    p, n = _ws_args(ws)
    _check(lib().mesa_update_running_params_fixed_beta(_ptr(x), _dt(x), Layout(*layout), _ptr(alpha), _ptr(beta), float(lam),
                                                       int(bool(first_call)), float(beta_fixed), p, n, _stream()),
           "mesa_update_running_params_fixed_beta")


def mesa_update_running_scale_sym(x, layout, m, lam, first_call, ws):
    p, n = _ws_args(ws)
    _check(lib().mesa_update_running_scale_sym(_ptr(x), _dt(x), Layout(*layout), _ptr(m), float(lam), int(bool(first_call)), p, n,
                                               _stream()), "mesa_update_running_scale_sym")


def mesa_quantize_sym(x, layout, m, q, mode=ROUND_STOCHASTIC, seed=0, offset=0):
    _check(lib().mesa_quantize_sym(_ptr(x), _dt(x), Layout(*layout), _ptr(m), _ptr(q), int(mode), int(seed), int(offset),
                                   _stream()), "mesa_quantize_sym")


def mesa_dequantize_sym(q, layout, m, x_hat):
    _check(lib().mesa_dequantize_sym(_ptr(q), Layout(*layout), _ptr(m), _ptr(x_hat), _dt(x_hat), _stream()), "mesa_dequantize_sym")


def mesa_update_running_params_static(x, layout, alpha, beta, lam, first_call):
    _check(lib().mesa_update_running_params_static(_ptr(x), _dt(x), Layout(*layout), _ptr(alpha), _ptr(beta), float(lam),
                                                   int(bool(first_call)), _stream()), "mesa_update_running_params_static")


def static_scratch_bytes() -> int:
    return int(lib().mesa_static_scratch_bytes())


def mesa_quantize_headwise(x, layout, alpha, beta, q, mode=ROUND_STOCHASTIC, seed=0, offset=0):
    _check(lib().mesa_quantize_headwise(_ptr(x), _dt(x), Layout(*layout), _ptr(alpha), _ptr(beta), _ptr(q), int(mode),
                                        int(seed), int(offset), _stream()), "mesa_quantize_headwise")


def mesa_quantize_update_fused(x, layout, alpha, beta, lam, q, ws, mode=ROUND_STOCHASTIC, seed=0, offset=0):
    p, n = _ws_args(ws)
    _check(lib().mesa_quantize_update_fused(_ptr(x), _dt(x), Layout(*layout), _ptr(alpha), _ptr(beta), float(lam), _ptr(q),
                                            int(mode), int(seed), int(offset), p, n, _stream()), "mesa_quantize_update_fused")


def mesa_gelu_fwd_q(x, layout, alpha, beta, lam, y, q, ws, mode=ROUND_STOCHASTIC, seed=0, offset=0):
    assert y.dtype == x.dtype
    p, n = _ws_args(ws)
    _check(lib().mesa_gelu_fwd_q(_ptr(x), _dt(x), Layout(*layout), _ptr(alpha), _ptr(beta), float(lam), _ptr(y), _ptr(q),
                                 int(mode), int(seed), int(offset), p, n, _stream()), "mesa_gelu_fwd_q")


def mesa_softmax_fwd_q(s, B, H, rows, cols, alpha, beta, lam, y, q, ws, mode=ROUND_STOCHASTIC, seed=0, offset=0):
    assert y.dtype == s.dtype
    p, n = _ws_args(ws)
    _check(lib().mesa_softmax_fwd_q(_ptr(s), B, H, rows, cols, _ptr(alpha), _ptr(beta), float(lam), _ptr(y), _ptr(q), int(mode),
                                    int(seed), int(offset), p, n, _dt(s), _stream()), "mesa_softmax_fwd_q")


def mesa_layernorm_fwd_q(x, M, D, G, gamma, bias, eps, alpha, beta, lam, y, mean, rstd, q, ws, mode=ROUND_STOCHASTIC, seed=0, offset=0):
    assert y.dtype == x.dtype == gamma.dtype == bias.dtype
    p, n = _ws_args(ws)
    _check(lib().mesa_layernorm_fwd_q(_ptr(x), M, D, G, _ptr(gamma), _ptr(bias), float(eps), _ptr(alpha), _ptr(beta), float(lam),
                                      _ptr(y), _ptr(mean), _ptr(rstd), _ptr(q), int(mode), int(seed), int(offset), p, n, _dt(x),
                                      _stream()), "mesa_layernorm_fwd_q")


def mesa_dequantize(q, layout, alpha, beta, x_hat):
    _check(lib().mesa_dequantize(_ptr(q), Layout(*layout), _ptr(alpha), _ptr(beta), _ptr(x_hat), _dt(x_hat), _stream()),
           "mesa_dequantize")


def mesa_quantize_headwise_b4(x, layout, alpha, beta, q4, mode=ROUND_STOCHASTIC, seed=0, offset=0):
    _check(lib().mesa_quantize_headwise_b4(_ptr(x), _dt(x), Layout(*layout), _ptr(alpha), _ptr(beta), _ptr(q4), int(mode),
                                           int(seed), int(offset), _stream()), "mesa_quantize_headwise_b4")


def mesa_dequantize_b4(q4, layout, alpha, beta, x_hat):
    _check(lib().mesa_dequantize_b4(_ptr(q4), Layout(*layout), _ptr(alpha), _ptr(beta), _ptr(x_hat), _dt(x_hat), _stream()),
           "mesa_dequantize_b4")


def mesa_gelu_bwd_q_b4(q4, layout, alpha, beta, dy, dx):
    assert dx.dtype == dy.dtype
    _check(lib().mesa_gelu_bwd_q_b4(_ptr(q4), Layout(*layout), _ptr(alpha), _ptr(beta), _ptr(dy), _ptr(dx), _dt(dy), _stream()),
           "mesa_gelu_bwd_q_b4")


def mesa_softmax_bwd_q(yq, B, H, rows, cols, alpha, beta, dy, dx):
    assert dx.dtype == dy.dtype
    _check(lib().mesa_softmax_bwd_q(_ptr(yq), B, H, rows, cols, _ptr(alpha), _ptr(beta), _ptr(dy), _ptr(dx), _dt(dy),
                                    _stream()), "mesa_softmax_bwd_q")


def mesa_gelu_bwd_q(xq, layout, alpha, beta, dy, dx):
    assert dx.dtype == dy.dtype
    _check(lib().mesa_gelu_bwd_q(_ptr(xq), Layout(*layout), _ptr(alpha), _ptr(beta), _ptr(dy), _ptr(dx), _dt(dy), _stream()),
           "mesa_gelu_bwd_q")


def mesa_relu_bwd_q(xq, layout, alpha, beta, dy, dx):
    assert dx.dtype == dy.dtype
    _check(lib().mesa_relu_bwd_q(_ptr(xq), Layout(*layout), _ptr(alpha), _ptr(beta), _ptr(dy), _ptr(dx), _dt(dy), _stream()),
           "mesa_relu_bwd_q")


def mesa_attn_av_bwd_q(aq, vq, B, H, N, Dh, alpha_a, beta_a, alpha_v, beta_v, dO, dA, dV):
    assert dA.dtype == dO.dtype == dV.dtype
    _check(lib().mesa_attn_av_bwd_q(_ptr(aq), _ptr(vq), B, H, N, Dh, _ptr(alpha_a), _ptr(beta_a), _ptr(alpha_v), _ptr(beta_v),
                                    _ptr(dO), _ptr(dA), _ptr(dV), _dt(dO), _stream()), "mesa_attn_av_bwd_q")


def mesa_attn_qk_bwd_q(qq, kq, B, H, N, Dh, alpha_q, beta_q, alpha_k, beta_k, dS, scale, dQ, dK):
    assert dQ.dtype == dS.dtype == dK.dtype
    _check(lib().mesa_attn_qk_bwd_q(_ptr(qq), _ptr(kq), B, H, N, Dh, _ptr(alpha_q), _ptr(beta_q), _ptr(alpha_k), _ptr(beta_k),
                                    _ptr(dS), float(scale), _ptr(dQ), _ptr(dK), _dt(dS), _stream()), "mesa_attn_qk_bwd_q")


def mesa_layernorm_bwd_q(xq, M, D, G, alpha, beta, mean, rstd, gamma, dy, dx, dgamma, dbeta, ws):
    assert dx.dtype == dy.dtype == gamma.dtype
    p, n = _ws_args(ws)
    _check(lib().mesa_layernorm_bwd_q(_ptr(xq), M, D, G, _ptr(alpha), _ptr(beta), _ptr(mean), _ptr(rstd), _ptr(gamma),
                                      _ptr(dy), _ptr(dx), _ptr(dgamma), _ptr(dbeta), _dt(dy), p, n, _stream()),
           "mesa_layernorm_bwd_q")


def mesa_linear_dw_q(xq, M, K, G, alpha, beta, dy, N_out, dW, db, ws):
    p, n = _ws_args(ws)
    _check(lib().mesa_linear_dw_q(_ptr(xq), M, K, G, _ptr(alpha), _ptr(beta), _ptr(dy), N_out, _dt(dy), _ptr(dW), _ptr(db),
                                  p, n, _stream()), "mesa_linear_dw_q")


def conv2d_dw_q_workspace_bytes(cv: Conv2d, dtype: int = F16) -> int:
    return int(lib().mesa_conv2d_dw_q_workspace_bytes(cv, int(dtype)))


def mesa_conv2d_dw_q(xq, cv: Conv2d, G, alpha, beta, dy, dW, db, ws):
    p, n = _ws_args(ws)
    _check(lib().mesa_conv2d_dw_q(_ptr(xq), cv, G, _ptr(alpha), _ptr(beta), _ptr(dy), _dt(dy), _ptr(dW), _ptr(db), p, n, _stream()),
           "mesa_conv2d_dw_q")


def mesa_stream_copy(src, dst, nbytes):
    _check(lib().mesa_stream_copy(_ptr(src), _ptr(dst), int(nbytes), _stream()), "mesa_stream_copy")


def mesa_stream_read(src, nbytes, sink):
    _check(lib().mesa_stream_read(_ptr(src), int(nbytes), _ptr(sink), _stream()), "mesa_stream_read")


def mesa_stream_fill(dst, nbytes, word=0):
    _check(lib().mesa_stream_fill(_ptr(dst), int(nbytes), int(word), _stream()), "mesa_stream_fill")


MFMA_PROBE_WAVES = 256 * 4          # per launch
MFMA_PROBE_FLOPS_PER_STEP = 16 * 2 * 32 * 32 * 16   # per wave


def mesa_mfma_probe(form, steps, feed, sink):
    nbytes = 0 if feed is None else feed.numel() * feed.element_size()
    _check(lib().mesa_mfma_probe(int(form), int(steps), _ptr(feed), nbytes, _ptr(sink), _stream()), "mesa_mfma_probe")


class Event:
    """A HIP event recorded on the stream the kernels are launched on."""

    def __init__(self):
        self._h = _vp()
        _check(lib().mesa_event_create(C.byref(self._h)), "mesa_event_create")

    def record(self):
        _check(lib().mesa_event_record(self._h, _stream()), "mesa_event_record")

    def elapsed_ms(self, stop: "Event") -> float:
        ms = _f32()
        _check(lib().mesa_event_elapsed_ms(self._h, stop._h, C.byref(ms)), "mesa_event_elapsed_ms")
        return float(ms.value)

    def __del__(self):
        try:
            if self._h:
                lib().mesa_event_destroy(self._h)
        except Exception:
            pass
