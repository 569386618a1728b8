"""ctypes shim over the CPU oracle (oracle/mesa_ref.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  It never imports the GPU package and the GPU
package never imports it.  Arrays are numpy; binary16 tensors are passed as
numpy float16 arrays (their raw bits are what the C side reads).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "mesa_ref.c"
_LIB = _HERE / "libmesa_ref.so"

F32, F16, BF16 = 0, 1, 2
ROUND_NEAREST, ROUND_STOCHASTIC = 0, 1


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc; -ffp-contract=off keeps every binary32
    operation separately rounded, which the bit-exact comparisons rely on."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".tmp{os.getpid()}.so")
        cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-shared", "-fPIC", "-o", str(tmp), str(_SRC), "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(str(build()))
        _lib.mesa_ref_half_to_float.restype = C.c_float
        _lib.mesa_ref_half_to_float.argtypes = [C.c_uint16]
        _lib.mesa_ref_float_to_half.restype = C.c_uint16
        _lib.mesa_ref_float_to_half.argtypes = [C.c_float]
        _lib.mesa_ref_bf16_to_float.restype = C.c_float
        _lib.mesa_ref_bf16_to_float.argtypes = [C.c_uint16]
        _lib.mesa_ref_float_to_bf16.restype = C.c_uint16
        _lib.mesa_ref_float_to_bf16.argtypes = [C.c_float]
        _lib.mesa_ref_sr_uniform.restype = C.c_float
        _lib.mesa_ref_sr_uniform.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64]
        _lib.mesa_ref_num_threads.restype = C.c_int
    return _lib


def _dt(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.float16:
        return F16
    raise TypeError(f"unsupported dtype {a.dtype}")


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _c(a, dtype=None):
    a = np.ascontiguousarray(a)
    if dtype is not None and a.dtype != dtype:
        a = a.astype(dtype)
    return a


I64 = C.c_int64


def num_threads() -> int:
    return int(lib().mesa_ref_num_threads())


def half_to_float(bits: int) -> float:
    return float(lib().mesa_ref_half_to_float(bits))


def float_to_half(v: float) -> int:
    return int(lib().mesa_ref_float_to_half(C.c_float(v)))


def philox4x32(ctr, key, rounds=10):
    c = (C.c_uint32 * 4)(*ctr)
    k = (C.c_uint32 * 2)(*key)
    out = (C.c_uint32 * 4)()
    lib().mesa_ref_philox4x32(c, k, C.c_int(rounds), out)
    return [int(v) for v in out]


def sr_uniform(seed: int, offset: int, e: int) -> float:
    return float(lib().mesa_ref_sr_uniform(seed, offset, e))


def group_minmax(x, layout):
    outer, groups, inner = layout
    x = _c(x)
    assert x.size == outer * groups * inner
    mn = np.empty(groups, np.float32)
    mx = np.empty(groups, np.float32)
    lib().mesa_ref_group_minmax(_p(x), _dt(x), I64(outer), I64(groups), I64(inner), _p(mn), _p(mx))
    return mn, mx


def update_running_params(x, layout, alpha, beta, lam, first_call):
    """Returns the new (alpha, beta); the inputs are not modified."""
    outer, groups, inner = layout
    x = _c(x)
    assert x.size == outer * groups * inner
    a = _c(alpha, np.float32).copy()
    b = _c(beta, np.float32).copy()
    assert a.size == groups and b.size == groups
    lib().mesa_ref_update_running_params(_p(x), _dt(x), I64(outer), I64(groups), I64(inner),
                                         _p(a), _p(b), C.c_float(lam), C.c_int(int(first_call)))
    return a, b


def update_running_params_sym(x, layout, alpha, beta, lam, first_call):
    """Symmetric-range variant (range [-max|x|, +max|x|] per group); returns the new (alpha, beta)."""
    outer, groups, inner = layout
    x = _c(x)
    assert x.size == outer * groups * inner
    a = _c(alpha, np.float32).copy()
    b = _c(beta, np.float32).copy()
    assert a.size == groups and b.size == groups
    lib().mesa_ref_update_running_params_sym(_p(x), _dt(x), I64(outer), I64(groups), I64(inner),
                                             _p(a), _p(b), C.c_float(lam), C.c_int(int(first_call)))
    return a, b


def update_running_params_fixed_beta(x, layout, alpha, lam, first_call, beta_fixed):
    """Fixed-offset variant (beta = beta_fixed in every group, alpha tracks max - beta_fixed); returns (alpha, beta)."""
    outer, groups, inner = layout
    x = _c(x)
    assert x.size == outer * groups * inner
    a = _c(alpha, np.float32).copy()
    b = np.empty(groups, np.float32)
    assert a.size == groups
    lib().mesa_ref_update_running_params_fixed_beta(_p(x), _dt(x), I64(outer), I64(groups), I64(inner), _p(a), _p(b),
                                                    C.c_float(lam), C.c_int(int(first_call)), C.c_float(beta_fixed))
    return a, b


def quantize_headwise(x, layout, alpha, beta, mode=ROUND_NEAREST, seed=0, offset=0):
    outer, groups, inner = layout
    x = _c(x)
    assert x.size == outer * groups * inner
    a = _c(alpha, np.float32)
    b = _c(beta, np.float32)
    assert a.size == groups and b.size == groups
    q = np.empty(x.size, np.int8)
    lib().mesa_ref_quantize_headwise(_p(x), _dt(x), I64(outer), I64(groups), I64(inner), _p(a), _p(b), _p(q),
                                     C.c_int(mode), C.c_uint64(seed), C.c_uint64(offset))
    return q.reshape(x.shape)


def quantize_update_fused(x, layout, alpha, beta, lam, mode=ROUND_NEAREST, seed=0, offset=0):
    """Codes with the parameters as given, then the parameters moved by this batch: returns (q, alpha', beta')."""
    outer, groups, inner = layout
    x = _c(x)
    assert x.size == outer * groups * inner
    a = _c(alpha, np.float32).copy()
    b = _c(beta, np.float32).copy()
    assert a.size == groups and b.size == groups
    q = np.empty(x.size, np.int8)
    lib().mesa_ref_quantize_update_fused(_p(x), _dt(x), I64(outer), I64(groups), I64(inner), _p(a), _p(b), C.c_float(lam),
                                         _p(q), C.c_int(mode), C.c_uint64(seed), C.c_uint64(offset))
    return q.reshape(x.shape), a, b


def gelu_fwd_q(x, layout, alpha, beta, lam, mode=ROUND_NEAREST, seed=0, offset=0):
    """A Mesa GELU layer's forward: returns (y in binary64, q, alpha', beta')."""
    outer, groups, inner = layout
    x = _c(x)
    assert x.size == outer * groups * inner
    a = _c(alpha, np.float32).copy()
    b = _c(beta, np.float32).copy()
    assert a.size == groups and b.size == groups
    q = np.empty(x.size, np.int8)
    y = np.empty(x.size, np.float64)
    lib().mesa_ref_gelu_fwd_q(_p(x), _dt(x), I64(outer), I64(groups), I64(inner), _p(a), _p(b), C.c_float(lam), _p(y),
                              _p(q), C.c_int(mode), C.c_uint64(seed), C.c_uint64(offset))
    return y.reshape(x.shape), q.reshape(x.shape), a, b


def quantize_headwise_b4(x, layout, alpha, beta, mode=ROUND_NEAREST, seed=0, offset=0):
    """Four-bit codes, two per byte (element e in byte e // 2, low nibble for even e); returns uint8[(numel + 1) // 2]."""
    outer, groups, inner = layout
    x = _c(x)
    n = outer * groups * inner
    assert x.size == n
    a = _c(alpha, np.float32)
    b = _c(beta, np.float32)
    q4 = np.empty((n + 1) // 2, np.uint8)
    lib().mesa_ref_quantize_headwise_b4(_p(x), _dt(x), I64(outer), I64(groups), I64(inner), _p(a), _p(b), _p(q4), C.c_int(mode),
                                        C.c_uint64(seed), C.c_uint64(offset))
    return q4


def dequantize_b4(q4, layout, alpha, beta, dtype=np.float32):
    outer, groups, inner = layout
    n = outer * groups * inner
    q4 = _c(q4, np.uint8)
    assert q4.size == (n + 1) // 2
    a = _c(alpha, np.float32)
    b = _c(beta, np.float32)
    if isinstance(dtype, str) and dtype == "bf16":
        out = np.empty(n, np.uint16)
        lib().mesa_ref_dequantize_b4(_p(q4), I64(outer), I64(groups), I64(inner), _p(a), _p(b), _p(out), BF16)
        return out
    out = np.empty(n, dtype)
    lib().mesa_ref_dequantize_b4(_p(q4), I64(outer), I64(groups), I64(inner), _p(a), _p(b), _p(out), _dt(out))
    return out


def gelu_bwd_q_b4(q4, layout, alpha, beta, dy):
    outer, groups, inner = layout
    n = outer * groups * inner
    q4 = _c(q4, np.uint8)
    dy = _c(dy)
    assert q4.size == (n + 1) // 2 and dy.size == n
    a = _c(alpha, np.float32)
    b = _c(beta, np.float32)
    dx = np.empty(n, np.float64)
    lib().mesa_ref_gelu_bwd_q_b4(_p(q4), I64(outer), I64(groups), I64(inner), _p(a), _p(b), _p(dy), _dt(dy), _p(dx))
    return dx


def update_running_scale_sym(x, layout, m, lam, first_call):
    """Scale-only symmetric scheme: the running estimate of max |x| per group; returns the new m."""
    outer, groups, inner = layout
    x = _c(x)
    assert x.size == outer * groups * inner
    m = _c(m, np.float32).copy()
    lib().mesa_ref_update_running_scale_sym(_p(x), _dt(x), I64(outer), I64(groups), I64(inner), _p(m), C.c_float(lam),
                                            C.c_int(int(bool(first_call))))
    return m


def quantize_sym(x, layout, m, mode=ROUND_NEAREST, seed=0, offset=0):
    outer, groups, inner = layout
    x = _c(x)
    assert x.size == outer * groups * inner
    m = _c(m, np.float32)
    q = np.empty(x.shape, np.int8)
    lib().mesa_ref_quantize_sym(_p(x), _dt(x), I64(outer), I64(groups), I64(inner), _p(m), _p(q), C.c_int(mode),
                                C.c_uint64(seed), C.c_uint64(offset))
    return q


def dequantize_sym(q, layout, m, dtype=np.float32):
    outer, groups, inner = layout
    q = _c(q, np.int8)
    assert q.size == outer * groups * inner
    m = _c(m, np.float32)
    if isinstance(dtype, str) and dtype == "bf16":
        out = np.empty(q.shape, np.uint16)
        lib().mesa_ref_dequantize_sym(_p(q), I64(outer), I64(groups), I64(inner), _p(m), _p(out), BF16)
        return out
    out = np.empty(q.shape, dtype)
    lib().mesa_ref_dequantize_sym(_p(q), I64(outer), I64(groups), I64(inner), _p(m), _p(out), _dt(out))
    return out


def dequantize(q, layout, alpha, beta, dtype=np.float32):
    """dtype: np.float32, np.float16, or the string "bf16" -- then the result is the bfloat16 bit patterns as uint16
    (numpy has no bfloat16)."""
    outer, groups, inner = layout
    q = _c(q, np.int8)
    assert q.size == outer * groups * inner
    a = _c(alpha, np.float32)
    b = _c(beta, np.float32)
    if isinstance(dtype, str) and dtype == "bf16":
        out = np.empty(q.shape, np.uint16)
        lib().mesa_ref_dequantize(_p(q), I64(outer), I64(groups), I64(inner), _p(a), _p(b), _p(out), BF16)
        return out
    out = np.empty(q.shape, dtype)
    lib().mesa_ref_dequantize(_p(q), I64(outer), I64(groups), I64(inner), _p(a), _p(b), _p(out), _dt(out))
    return out


def float_to_bf16(f: float) -> int:
    return int(lib().mesa_ref_float_to_bf16(C.c_float(f)))


def bf16_to_float(bits: int) -> float:
    return float(lib().mesa_ref_bf16_to_float(int(bits)))


def softmax_fwd(s, total_rows, cols):
    """Row softmax of s (binary16 or binary32 storage) in binary64."""
    s = _c(s)
    assert s.size == total_rows * cols
    y = np.empty(s.size, np.float64)
    lib().mesa_ref_softmax_fwd(_p(s), _dt(s), I64(total_rows), I64(cols), _p(y))
    return y.reshape(s.shape)


def softmax_bwd_q(yq, B, H, rows, cols, alpha, beta, dy):
    yq = _c(yq, np.int8)
    dy = _c(dy)
    assert yq.size == B * H * rows * cols == dy.size
    a = _c(alpha, np.float32)
    b = _c(beta, np.float32)
    dx = np.empty(yq.shape, np.float64)
    lib().mesa_ref_softmax_bwd_q(_p(yq), I64(B), I64(H), I64(rows), I64(cols), _p(a), _p(b), _p(dy), _dt(dy), _p(dx))
    return dx


def gelu_bwd_q(xq, layout, alpha, beta, dy):
    outer, groups, inner = layout
    xq = _c(xq, np.int8)
    dy = _c(dy)
    assert xq.size == outer * groups * inner == dy.size
    a = _c(alpha, np.float32)
    b = _c(beta, np.float32)
    dx = np.empty(xq.shape, np.float64)
    lib().mesa_ref_gelu_bwd_q(_p(xq), I64(outer), I64(groups), I64(inner), _p(a), _p(b), _p(dy), _dt(dy), _p(dx))
    return dx


def relu_bwd_q(xq, layout, alpha, beta, dy):
    outer, groups, inner = layout
    xq = _c(xq, np.int8)
    dy = _c(dy)
    assert xq.size == outer * groups * inner == dy.size
    a = _c(alpha, np.float32)
    b = _c(beta, np.float32)
    dx = np.empty(xq.shape, np.float64)
    lib().mesa_ref_relu_bwd_q(_p(xq), I64(outer), I64(groups), I64(inner), _p(a), _p(b), _p(dy), _dt(dy), _p(dx))
    return dx


def layernorm_fwd(x, M, D, gamma, bias, eps):
    """LayerNorm over the last axis in binary64: returns (y, mean, rstd)."""
    x = _c(x)
    gamma, bias = _c(gamma, x.dtype), _c(bias, x.dtype)
    assert x.size == M * D and gamma.size == D and bias.size == D
    y = np.empty((M, D), np.float64)
    mean = np.empty(M, np.float64)
    rstd = np.empty(M, np.float64)
    lib().mesa_ref_layernorm_fwd(_p(x), _dt(x), I64(M), I64(D), _p(gamma), _p(bias), C.c_double(eps), _p(y), _p(mean), _p(rstd))
    return y, mean, rstd


def layernorm_bwd_q(xq, M, D, G, alpha, beta, mean, rstd, gamma, dy):
    xq = _c(xq, np.int8)
    dy = _c(dy)
    gamma = _c(gamma, dy.dtype)
    assert xq.size == M * D == dy.size and gamma.size == D
    a = _c(alpha, np.float32)
    b = _c(beta, np.float32)
    mean = _c(mean, np.float32)
    rstd = _c(rstd, np.float32)
    assert mean.size == M and rstd.size == M
    dx = np.empty((M, D), np.float64)
    dg = np.empty(D, np.float64)
    db = np.empty(D, np.float64)
    rc = lib().mesa_ref_layernorm_bwd_q(_p(xq), I64(M), I64(D), I64(G), _p(a), _p(b), _p(mean), _p(rstd), _p(gamma),
                                        _p(dy), _dt(dy), _p(dx), _p(dg), _p(db))
    assert rc == 0
    return dx, dg, db


def attn_av_bwd_q(aq, vq, B, H, N, Dh, alpha_a, beta_a, alpha_v, beta_v, dO):
    """Backward of O = A V at the de-quantized A (B,H,N,N) and V (B,H,N,Dh): returns (dA, dV) in binary64."""
    aq, vq, dO = _c(aq, np.int8), _c(vq, np.int8), _c(dO)
    assert aq.size == B * H * N * N and vq.size == B * H * N * Dh and dO.size == B * H * N * Dh
    dA = np.empty((B, H, N, N), np.float64)
    dV = np.empty((B, H, N, Dh), np.float64)
    lib().mesa_ref_attn_av_bwd_q(_p(aq), _p(vq), I64(B), I64(H), I64(N), I64(Dh), _p(_c(alpha_a, np.float32)),
                                 _p(_c(beta_a, np.float32)), _p(_c(alpha_v, np.float32)), _p(_c(beta_v, np.float32)),
                                 _p(dO), _dt(dO), _p(dA), _p(dV))
    return dA, dV


def attn_qk_bwd_q(qq, kq, B, H, N, Dh, alpha_q, beta_q, alpha_k, beta_k, dS, scale):
    """Backward of S = scale Q K^T at the de-quantized Q, K (B,H,N,Dh): returns (dQ, dK) in binary64."""
    qq, kq, dS = _c(qq, np.int8), _c(kq, np.int8), _c(dS)
    assert qq.size == B * H * N * Dh and kq.size == B * H * N * Dh and dS.size == B * H * N * N
    dQ = np.empty((B, H, N, Dh), np.float64)
    dK = np.empty((B, H, N, Dh), np.float64)
    lib().mesa_ref_attn_qk_bwd_q(_p(qq), _p(kq), I64(B), I64(H), I64(N), I64(Dh), _p(_c(alpha_q, np.float32)),
                                 _p(_c(beta_q, np.float32)), _p(_c(alpha_k, np.float32)), _p(_c(beta_k, np.float32)),
                                 _p(dS), _dt(dS), C.c_double(scale), _p(dQ), _p(dK))
    return dQ, dK


def linear_dw_q(xq, M, K, G, alpha, beta, dy, N_out):
    xq = _c(xq, np.int8)
    dy = _c(dy)
    assert xq.size == M * K and dy.size == M * N_out
    a = _c(alpha, np.float32)
    b = _c(beta, np.float32)
    dW = np.empty((N_out, K), np.float64)
    db = np.empty(N_out, np.float64)
    rc = lib().mesa_ref_linear_dw_q(_p(xq), I64(M), I64(K), I64(G), _p(a), _p(b), _p(dy), I64(N_out), _dt(dy),
                                    _p(dW), _p(db))
    assert rc == 0
    return dW, db


def linear_dw_q_entries(xq, M, K, G, alpha, beta, dy, N_out, n_idx, k_idx):
    xq = _c(xq, np.int8)
    dy = _c(dy)
    n_idx = _c(n_idx, np.int64)
    k_idx = _c(k_idx, np.int64)
    a = _c(alpha, np.float32)
    b = _c(beta, np.float32)
    out = np.empty(n_idx.size, np.float64)
    rc = lib().mesa_ref_linear_dw_q_entries(_p(xq), I64(M), I64(K), I64(G), _p(a), _p(b), _p(dy), I64(N_out),
                                            _dt(dy), _p(n_idx), _p(k_idx), I64(n_idx.size), _p(out))
    assert rc == 0
    return out


def conv_geometry(B, C_in, H, W, C_out, KH, KW, stride=(1, 1), pad=(0, 0), dil=(1, 1)):
    """the thirteen integers the convolution functions take, and the output extent they imply"""
    geom = np.array([B, C_in, H, W, C_out, KH, KW, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1]], np.int64)
    OH = (H + 2 * pad[0] - dil[0] * (KH - 1) - 1) // stride[0] + 1
    OW = (W + 2 * pad[1] - dil[1] * (KW - 1) - 1) // stride[1] + 1
    return geom, OH, OW


def conv2d_dw_q(xq, geom, G, alpha, beta, dy):
    """weight gradient of a convolution at the de-quantized input (Eq. 2; Sec. 3.3, convolutional layers):
    (dW (C_out, C_in, KH, KW), db [C_out]) in binary64"""
    xq = _c(xq, np.int8)
    dy = _c(dy)
    geom = _c(geom, np.int64)
    a = _c(alpha, np.float32)
    b = _c(beta, np.float32)
    B, Cin, H, W, Cout, KH, KW = (int(v) for v in geom[:7])
    assert xq.size == B * Cin * H * W
    dW = np.empty((Cout, Cin, KH, KW), np.float64)
    db = np.empty(Cout, np.float64)
    rc = lib().mesa_ref_conv2d_dw_q(_p(xq), _p(geom), I64(G), _p(a), _p(b), _p(dy), _dt(dy), _p(dW), _p(db))
    assert rc == 0
    return dW, db


def conv2d_dw_q_entries(xq, geom, G, alpha, beta, dy, idx):
    """the same gradient at the (co, ci, kh, kw) rows of idx"""
    xq = _c(xq, np.int8)
    dy = _c(dy)
    geom = _c(geom, np.int64)
    idx = _c(idx, np.int64)
    a = _c(alpha, np.float32)
    b = _c(beta, np.float32)
    out = np.empty(idx.size // 4, np.float64)
    rc = lib().mesa_ref_conv2d_dw_q_entries(_p(xq), _p(geom), I64(G), _p(a), _p(b), _p(dy), _dt(dy), _p(idx), I64(idx.size // 4), _p(out))
    assert rc == 0
    return out
