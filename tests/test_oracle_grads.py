"""Pins for the oracle's layer gradients (Sec. 3.1, Eq. 2: the ordinary gradient function of the
layer evaluated at the de-quantized activation).

The paper prints no per-layer formula, so each one is pinned three ways: central finite
differences of a forward written here in numpy (with inputs placed on the quantization grid, so
x_hat = x and Eq. 2 is the true gradient), torch.autograd in fp64 at x_hat (a library routine for
this exact special case), and identities the formulas must satisfy.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import mesa_ref as R

GOLD = os.path.join(os.path.dirname(__file__), "golden")
erf = np.vectorize(math.erf)


def on_grid(rng, shape, G, step_log2=-5, lo=-4.0):
    """Random codes with per-group parameters whose step is a power of two: x_hat is exact."""
    codes = rng.integers(0, 256, size=shape)
    step = 2.0 ** step_log2
    alpha = np.full(G, 255.0 * step, np.float32)
    beta = (lo + np.arange(G) * 0.25).astype(np.float32)
    return codes, alpha, beta, step


def fd_grad(f, x, eps=1e-6):
    """dL/dx by central differences for scalar-valued f."""
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        xp, xm = x.copy(), x.copy()
        xp[i] += eps
        xm[i] -= eps
        g[i] = (f(xp) - f(xm)) / (2 * eps)
    return g


def relerr(a, b):
    return np.abs(a - b).max() / max(np.abs(b).max(), 1e-300)


# ----------------------------------------------------------------------------- softmax

def test_softmax_forward_is_the_library_softmax_rows_sum_to_one_and_shifts_cancel():
    rng = np.random.default_rng(17)
    for dt in (np.float32, np.float16):
        s = (rng.standard_normal((2, 3, 7, 19)) * 3).astype(dt)
        y = R.softmax_fwd(s, 2 * 3 * 7, 19)
        ref = torch.softmax(torch.from_numpy(s.astype(np.float64)), dim=-1).numpy()
        assert np.allclose(y, ref, rtol=1e-13, atol=1e-300)
        assert np.allclose(y.sum(-1), 1.0, rtol=1e-14)
        assert np.all(y > 0)
    s32 = (rng.integers(-256, 257, size=(5, 33)) / 64.0).astype(np.float32)   # a grid on which adding 4 is exact
    shifted = s32 + np.float32(4.0)
    assert np.array_equal(shifted.astype(np.float64) - 4.0, s32.astype(np.float64))
    assert np.allclose(R.softmax_fwd(shifted, 5, 33), R.softmax_fwd(s32, 5, 33), rtol=1e-12)
    one_hot = np.full((1, 8), -1e4, np.float32); one_hot[0, 3] = 0.0
    assert np.array_equal(R.softmax_fwd(one_hot, 1, 8), np.eye(8)[3:4])


def test_softmax_backward_against_finite_differences():
    rng = np.random.default_rng(0)
    B, H, rows, cols = 1, 2, 3, 6
    # rows of y = k/256 with sum 256: exactly representable, sums to one, step 2^-8 exact
    k = np.zeros((B, H, rows, cols), np.int64)
    for idx in np.ndindex(B, H, rows):
        cuts = np.sort(rng.choice(np.arange(1, 256), cols - 1, replace=False))
        k[idx] = np.diff(np.concatenate([[0], cuts, [256]]))
    assert k.max() <= 255 and (k.sum(-1) == 256).all()
    alpha, beta = np.full(H, 255.0 / 256.0, np.float32), np.zeros(H, np.float32)
    y = k / 256.0
    dy = rng.standard_normal(y.shape).astype(np.float32)
    dx = R.softmax_bwd_q((k - 128).astype(np.int8), B, H, rows, cols, alpha, beta, dy)
    z = np.log(y)

    def loss(zz):
        e = np.exp(zz - zz.max(-1, keepdims=True))
        return float((dy.astype(np.float64) * e / e.sum(-1, keepdims=True)).sum())

    assert relerr(dx, fd_grad(loss, z)) < 1e-6


def test_softmax_backward_rows_sum_to_zero_when_y_sums_to_one_and_in_general_to_d_times_the_defect():
    rng = np.random.default_rng(1)
    B, H, rows, cols = 2, 3, 5, 11
    k = rng.integers(0, 256, (B, H, rows, cols))
    alpha = np.array([0.7, 0.05, 0.3], np.float32)
    beta = np.array([0.0, 0.01, 0.002], np.float32)
    dy = rng.standard_normal(k.shape).astype(np.float32)
    q = (k - 128).astype(np.int8)
    dx = R.softmax_bwd_q(q, B, H, rows, cols, alpha, beta, dy)
    yh = R.dequantize(q, (B, H, rows * cols), alpha, beta).astype(np.float64).reshape(k.shape)
    d = (dy * yh).sum(-1)
    assert np.allclose(dx.sum(-1), d * (1.0 - yh.sum(-1)), rtol=1e-9, atol=1e-9)
    # exact-sum rows: the generalised identity collapses to a zero row sum
    k1 = np.zeros((1, 1, 4, 8), np.int64)
    k1[..., :] = [100, 50, 30, 20, 16, 24, 8, 8]
    dy1 = rng.standard_normal(k1.shape).astype(np.float32)
    dx1 = R.softmax_bwd_q((k1 - 128).astype(np.int8), 1, 1, 4, 8, [255.0 / 256.0], [0.0], dy1)
    assert np.abs(dx1.sum(-1)).max() < 1e-12


def test_softmax_backward_matches_torch_at_y_hat():
    rng = np.random.default_rng(2)
    B, H, rows, cols = 2, 3, 7, 13
    q = rng.integers(-128, 128, (B, H, rows, cols)).astype(np.int8)
    alpha, beta = np.array([0.9, 0.2, 0.5], np.float32), np.array([0.0, 0.003, 0.01], np.float32)
    for dt in (np.float32, np.float16):
        dy = rng.standard_normal(q.shape).astype(dt)
        dx = R.softmax_bwd_q(q, B, H, rows, cols, alpha, beta, dy)
        yh = torch.from_numpy(R.dequantize(q, (B, H, rows * cols), alpha, beta).reshape(q.shape)).double()
        want = torch._softmax_backward_data(torch.from_numpy(dy.astype(np.float64)), yh, -1, torch.float64).numpy()
        assert relerr(dx, want) < 1e-12


# ----------------------------------------------------------------------------- GELU

def gelu(x):
    return 0.5 * x * (1.0 + erf(x / math.sqrt(2.0)))


def test_gelu_backward_against_finite_differences_and_torch():
    rng = np.random.default_rng(3)
    outer, G, inner = 3, 2, 5
    codes, alpha, beta, step = on_grid(rng, (outer, G, inner), G)
    x = beta[None, :, None].astype(np.float64) + codes * step
    dy = rng.standard_normal(x.shape).astype(np.float32)
    dx = R.gelu_bwd_q((codes - 128).astype(np.int8), (outer, G, inner), alpha, beta, dy)
    assert relerr(dx, fd_grad(lambda v: float((dy * gelu(v)).sum()), x)) < 1e-6
    xt = torch.from_numpy(x).requires_grad_(True)
    torch.nn.functional.gelu(xt).backward(torch.from_numpy(dy.astype(np.float64)))
    assert relerr(dx, xt.grad.numpy()) < 1e-12


def test_relu_backward_against_finite_differences_torch_and_the_mask_it_is():
    # ReLU is among the CNN layers Sec. 3.3 lists; saved tensor: its input, channel-group codes
    rng = np.random.default_rng(31)
    outer, G, inner = 4, 3, 7
    codes, alpha, beta, step = on_grid(rng, (outer, G, inner), G, step_log2=-5, lo=-3.96875)   # no x_hat at exactly 0 ...
    x = beta[None, :, None].astype(np.float64) + codes * step
    assert np.all(np.abs(x) > 1e-3)
    dy = rng.standard_normal(x.shape).astype(np.float32)
    dx = R.relu_bwd_q((codes - 128).astype(np.int8), (outer, G, inner), alpha, beta, dy)
    assert relerr(dx, fd_grad(lambda v: float((dy * np.maximum(v, 0.0)).sum()), x)) < 1e-6
    xt = torch.from_numpy(x).requires_grad_(True)
    torch.relu(xt).backward(torch.from_numpy(dy.astype(np.float64)))
    assert np.array_equal(dx, xt.grad.numpy())
    assert np.array_equal(dx != 0, (x > 0) & (dy != 0))
    # ... and at exactly 0 the derivative is 0 (the library's convention too)
    a0, b0 = np.array([255.0 * step], np.float32), np.array([-128 * step], np.float32)
    q0 = np.array([0, 1, -1], np.int8)                      # x_bar = 128, 129, 127 -> x_hat = 0, +step, -step
    assert np.array_equal(R.relu_bwd_q(q0, (1, 1, 3), a0, b0, np.ones(3, np.float32)), [0.0, 1.0, 0.0])


def test_gelu_layer_forward_is_the_library_gelu_plus_the_single_pass_codes():
    # y against torch's exact GELU in binary64 and the erf formula typed out; its minimum is the -0.17 the paper prints;
    # codes and estimates are the single-pass forward's (pinned on its own)
    rng = np.random.default_rng(7)
    lay = (5, 3, 40)
    a0, b0 = np.array([6.0, 7.0, 8.0], np.float32), np.array([-3.0, -3.5, -4.0], np.float32)
    for dt in (np.float32, np.float16):
        x = (rng.standard_normal(lay) * 1.7).astype(dt)
        y, q, a, b = R.gelu_fwd_q(x, lay, a0, b0, 0.9, R.ROUND_STOCHASTIC, 5, 2)
        xd = x.astype(np.float64)
        assert np.allclose(y, torch.nn.functional.gelu(torch.from_numpy(xd)).numpy(), rtol=1e-13, atol=1e-15)
        assert np.allclose(y, gelu(xd), rtol=1e-13, atol=1e-15)
        q2, a2, b2 = R.quantize_update_fused(x, lay, a0, b0, 0.9, R.ROUND_STOCHASTIC, 5, 2)
        assert np.array_equal(q, q2) and np.array_equal(a, a2) and np.array_equal(b, b2)
    grid = np.linspace(-2, 0, 200001).astype(np.float32)
    yg = R.gelu_fwd_q(grid, (1, 1, grid.size), [1.0], [0.0], 0.9)[0]
    assert abs(yg.min() - (-0.16997)) < 1e-5


def test_gelu_derivative_vanishes_at_the_minimum_the_paper_prints():
    # FFN visualisation section: the offset of the second FC layer's input sits at min GELU = -0.17
    want = float([l for l in open(os.path.join(GOLD, "gelu_min.txt")) if not l.startswith("#")][0])
    step = 2.0 ** -10
    alpha, beta = np.array([255 * step], np.float32), np.array([-0.875], np.float32)
    codes = np.arange(256)
    g = R.gelu_bwd_q((codes - 128).astype(np.int8), (1, 1, 256), alpha, beta, np.ones(256, np.float32))
    x = -0.875 + codes * step
    s = np.nonzero(np.diff(np.sign(g)))[0]
    assert s.size == 1                        # one sign change of the derivative: the minimum
    xmin = 0.5 * (x[s[0]] + x[s[0] + 1])
    assert g[0] < 0 < g[-1]
    assert round(float(gelu(xmin)), 2) == want
    assert abs(float(gelu(xmin)) + 0.16997) < 2e-5


# ----------------------------------------------------------------------------- LayerNorm

def ln_forward(x, gamma, eps):
    mu = x.mean(-1, keepdims=True)
    var = ((x - mu) ** 2).mean(-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * gamma


def test_layernorm_forward_is_the_library_layer_norm_and_normalises_rows():
    rng = np.random.default_rng(23)
    M_, D = 7, 48
    for dt in (np.float32, np.float16):
        x = (rng.standard_normal((M_, D)) * 2 + 0.5).astype(dt)
        gamma = (1 + 0.1 * rng.standard_normal(D)).astype(dt)
        bias = (0.1 * rng.standard_normal(D)).astype(dt)
        y, mean, rstd = R.layernorm_fwd(x, M_, D, gamma, bias, 1e-5)
        xt = torch.from_numpy(x.astype(np.float64))
        ref = torch.nn.functional.layer_norm(xt, (D,), torch.from_numpy(gamma.astype(np.float64)), torch.from_numpy(bias.astype(np.float64)), 1e-5)
        assert np.allclose(y, ref.numpy(), rtol=1e-12, atol=1e-13)
        assert np.allclose(mean, x.astype(np.float64).mean(1), rtol=1e-14, atol=1e-15)
        assert np.allclose(rstd, 1 / np.sqrt(x.astype(np.float64).var(1) + 1e-5), rtol=1e-13)
    y1, _, _ = R.layernorm_fwd(x, M_, D, np.ones(D, dt), np.zeros(D, dt), 0.0)
    assert np.allclose(y1.mean(1), 0.0, atol=1e-13) and np.allclose((y1 ** 2).mean(1), 1.0, rtol=1e-12)


def test_layernorm_backward_against_finite_differences():
    rng = np.random.default_rng(4)
    M, D, G = 3, 8, 2
    codes, alpha, beta, step = on_grid(rng, (M, D), G)
    x = np.repeat(beta.astype(np.float64), D // G)[None, :] + codes * step
    gamma = rng.uniform(0.5, 1.5, D).astype(np.float32)
    dy = rng.standard_normal((M, D)).astype(np.float32)
    eps = 1e-5
    mean = x.mean(-1)
    rstd = 1.0 / np.sqrt(x.var(-1) + eps)
    dx, dg, db = R.layernorm_bwd_q((codes - 128).astype(np.int8), M, D, G, alpha, beta,
                                   mean.astype(np.float32), rstd.astype(np.float32), gamma, dy)
    g64 = gamma.astype(np.float64)
    assert relerr(dx, fd_grad(lambda v: float((dy * ln_forward(v, g64, eps)).sum()), x)) < 2e-6
    assert relerr(dg, fd_grad(lambda gm: float((dy * ln_forward(x, gm, eps)).sum()), g64)) < 2e-6
    assert np.allclose(db, dy.astype(np.float64).sum(0), rtol=1e-12)


@pytest.mark.parametrize("dt", [np.float32, np.float16])
def test_layernorm_backward_matches_torch_at_x_hat(dt):
    rng = np.random.default_rng(5)
    M, D, G = 6, 24, 3
    q = rng.integers(-128, 128, (M, D)).astype(np.int8)
    alpha, beta = np.array([3.0, 8.0, 1.5], np.float32), np.array([-1.0, -4.0, 0.5], np.float32)
    xh = R.dequantize(q, (M, G, D // G), alpha, beta).astype(np.float64)
    gamma = rng.uniform(0.5, 1.5, D).astype(dt)
    dy = rng.standard_normal((M, D)).astype(dt)
    eps = 1e-5
    mean, rstd = xh.mean(-1), 1.0 / np.sqrt(xh.var(-1) + eps)
    dx, dg, db = R.layernorm_bwd_q(q, M, D, G, alpha, beta, mean.astype(np.float32), rstd.astype(np.float32), gamma, dy)
    xt = torch.from_numpy(xh).requires_grad_(True)
    gt = torch.from_numpy(gamma.astype(np.float64)).requires_grad_(True)
    bt = torch.zeros(D, dtype=torch.float64, requires_grad=True)
    torch.nn.functional.layer_norm(xt, (D,), gt, bt, eps).backward(torch.from_numpy(dy.astype(np.float64)))
    assert relerr(dx, xt.grad.numpy()) < 1e-6      # mean / rstd were rounded to binary32 on the way in
    assert relerr(dg, gt.grad.numpy()) < 1e-6
    assert relerr(db, bt.grad.numpy()) < 1e-12


def test_layernorm_backward_row_identity():
    # sum_j dx_j = -rstd * mean(g * xn) * sum_j xn_j  (zero when the saved statistics are x_hat's own)
    rng = np.random.default_rng(6)
    M, D, G = 4, 16, 4
    q = rng.integers(-128, 128, (M, D)).astype(np.int8)
    alpha, beta = rng.uniform(1, 5, G).astype(np.float32), rng.uniform(-2, 0, G).astype(np.float32)
    xh = R.dequantize(q, (M, G, D // G), alpha, beta).astype(np.float64)
    mean = (xh.mean(-1) + 0.05).astype(np.float32)          # deliberately not x_hat's own statistics
    rstd = (1.0 / np.sqrt(xh.var(-1) + 1e-5) * 1.1).astype(np.float32)
    gamma = rng.uniform(0.5, 1.5, D).astype(np.float32)
    dy = rng.standard_normal((M, D)).astype(np.float32)
    dx, _, _ = R.layernorm_bwd_q(q, M, D, G, alpha, beta, mean, rstd, gamma, dy)
    xn = (xh - mean[:, None].astype(np.float64)) * rstd[:, None].astype(np.float64)
    gg = dy.astype(np.float64) * gamma.astype(np.float64)
    want = -rstd.astype(np.float64) * (gg * xn).mean(-1) * xn.sum(-1)
    assert np.allclose(dx.sum(-1), want, rtol=1e-9, atol=1e-12)


# ----------------------------------------------------------------------------- Linear dW

def test_linear_dw_is_exact_on_integers():
    # alpha = 255, beta = 0: x_hat = q + 128 are integers; integer dy -> exact integer result
    rng = np.random.default_rng(7)
    M, K, N = 37, 12, 9
    q = rng.integers(-128, 128, (M, K)).astype(np.int8)
    dy = rng.integers(-8, 9, (M, N)).astype(np.float32)
    dW, db = R.linear_dw_q(q, M, K, 3, np.full(3, 255.0, np.float32), np.zeros(3, np.float32), dy, N)
    want = dy.astype(np.int64).T @ (q.astype(np.int64) + 128)
    assert dW.shape == (N, K)
    assert np.array_equal(dW, want.astype(np.float64))
    assert np.array_equal(db, dy.astype(np.int64).sum(0).astype(np.float64))


@pytest.mark.parametrize("dt", [np.float32, np.float16])
def test_linear_dw_matches_torch_fd_and_the_factored_form(dt):
    rng = np.random.default_rng(8)
    M, K, N, G = 29, 8, 5, 2
    q = rng.integers(-128, 128, (M, K)).astype(np.int8)
    alpha, beta = np.array([2.0, 7.0], np.float32), np.array([-1.0, -3.0], np.float32)
    dy = rng.standard_normal((M, N)).astype(dt)
    dW, db = R.linear_dw_q(q, M, K, G, alpha, beta, dy, N)
    xh = R.dequantize(q, (M, G, K // G), alpha, beta).astype(np.float64)
    dy64 = dy.astype(np.float64)
    # autograd of y = x W^T
    Wt = torch.zeros((N, K), dtype=torch.float64, requires_grad=True)
    (torch.from_numpy(xh) @ Wt.T).backward(torch.from_numpy(dy64))
    assert relerr(dW, Wt.grad.numpy()) < 1e-13
    # finite differences (the loss is linear in W, so they are exact up to rounding)
    W0 = rng.standard_normal((N, K))
    assert relerr(dW, fd_grad(lambda w: float((dy64 * (xh @ w.T)).sum()), W0, eps=1e-3)) < 1e-8
    # factored form used by matrix-core implementations: s_g * (dy^T u) + beta_g * colsum(dy)
    s = np.repeat((alpha / np.float32(255.0)).astype(np.float64), K // G)
    bcol = np.repeat(beta.astype(np.float64), K // G)
    fact = (dy64.T @ (q.astype(np.float64) + 128)) * s[None, :] + dy64.sum(0)[:, None] * bcol[None, :]
    assert relerr(dW, fact) < 1e-6    # x_hat itself is rounded to binary32, the factored form is not
    # sampled entries agree with the full matrix
    n_idx, k_idx = np.array([0, 4, 2]), np.array([7, 0, 3])
    ent = R.linear_dw_q_entries(q, M, K, G, alpha, beta, dy, N, n_idx, k_idx)
    assert np.array_equal(ent, dW[n_idx, k_idx])


# ----------------------------------------------------------------------------- attention matrix products

def _attn_case(rng, B, H, N, Dh, dt):
    aq = rng.integers(-128, 128, (B, H, N, N)).astype(np.int8)
    vq = rng.integers(-128, 128, (B, H, N, Dh)).astype(np.int8)
    pa = (rng.uniform(0.5, 1.5, H).astype(np.float32), rng.uniform(0.0, 0.01, H).astype(np.float32))
    pv = (rng.uniform(3.0, 9.0, H).astype(np.float32), rng.uniform(-4.0, -1.0, H).astype(np.float32))
    dO = rng.standard_normal((B, H, N, Dh)).astype(dt)
    return aq, vq, pa, pv, dO


def test_attention_products_are_exact_on_integers():
    # alpha = 255, beta = 0: every de-quantized operand is the integer q + 128; integer upstream gradients
    rng = np.random.default_rng(21)
    B, H, N, Dh = 2, 3, 7, 4
    aq, vq, _, _, _ = _attn_case(rng, B, H, N, Dh, np.float32)
    one, zero = np.full(H, 255.0, np.float32), np.zeros(H, np.float32)
    dO = rng.integers(-5, 6, (B, H, N, Dh)).astype(np.float32)
    dA, dV = R.attn_av_bwd_q(aq, vq, B, H, N, Dh, one, zero, one, zero, dO)
    A, V, G = aq.astype(np.int64) + 128, vq.astype(np.int64) + 128, dO.astype(np.int64)
    assert np.array_equal(dA, np.einsum("bhid,bhjd->bhij", G, V).astype(np.float64))
    assert np.array_equal(dV, np.einsum("bhij,bhid->bhjd", A, G).astype(np.float64))
    dS = rng.integers(-5, 6, (B, H, N, N)).astype(np.float32)
    dQ, dK = R.attn_qk_bwd_q(vq, aq[..., :Dh].copy(), B, H, N, Dh, one, zero, one, zero, dS, 2.0)
    Q, K, S = vq.astype(np.int64) + 128, aq[..., :Dh].astype(np.int64) + 128, dS.astype(np.int64)
    assert np.array_equal(dQ, 2.0 * np.einsum("bhij,bhjd->bhid", S, K))
    assert np.array_equal(dK, 2.0 * np.einsum("bhij,bhid->bhjd", S, Q))


@pytest.mark.parametrize("dt", [np.float32, np.float16])
def test_attention_products_match_torch_autograd_at_the_dequantized_operands(dt):
    rng = np.random.default_rng(22)
    B, H, N, Dh = 2, 3, 11, 6
    aq, vq, pa, pv, dO = _attn_case(rng, B, H, N, Dh, dt)
    dA, dV = R.attn_av_bwd_q(aq, vq, B, H, N, Dh, pa[0], pa[1], pv[0], pv[1], dO)
    Ah = torch.from_numpy(R.dequantize(aq, (B, H, N * N), pa[0], pa[1]).astype(np.float64).reshape(B, H, N, N)).requires_grad_()
    Vh = torch.from_numpy(R.dequantize(vq, (B, H, N * Dh), pv[0], pv[1]).astype(np.float64).reshape(B, H, N, Dh)).requires_grad_()
    (Ah @ Vh).backward(torch.from_numpy(dO.astype(np.float64)))
    assert relerr(dA, Ah.grad.numpy()) < 1e-13 and relerr(dV, Vh.grad.numpy()) < 1e-13
    # S = scale Q K^T, heads with different parameters for Q and K
    qq, kq = vq, rng.integers(-128, 128, (B, H, N, Dh)).astype(np.int8)
    pq, pk = pv, (rng.uniform(1.0, 2.0, H).astype(np.float32), rng.uniform(-1.0, 0.0, H).astype(np.float32))
    dS = rng.standard_normal((B, H, N, N)).astype(dt)
    scale = Dh ** -0.5
    dQ, dK = R.attn_qk_bwd_q(qq, kq, B, H, N, Dh, pq[0], pq[1], pk[0], pk[1], dS, scale)
    Qh = torch.from_numpy(R.dequantize(qq, (B, H, N * Dh), pq[0], pq[1]).astype(np.float64).reshape(B, H, N, Dh)).requires_grad_()
    Kh = torch.from_numpy(R.dequantize(kq, (B, H, N * Dh), pk[0], pk[1]).astype(np.float64).reshape(B, H, N, Dh)).requires_grad_()
    (scale * (Qh @ Kh.transpose(-1, -2))).backward(torch.from_numpy(dS.astype(np.float64)))
    assert relerr(dQ, Qh.grad.numpy()) < 1e-13 and relerr(dK, Kh.grad.numpy()) < 1e-13


def test_attention_products_against_finite_differences_of_the_whole_attention():
    # L = sum(dO * (softmax(scale Q K^T) V)): chain the oracle's three backward steps (A V, softmax, Q K^T) with the
    # operands on the quantization grid (x_hat = x) and compare with central differences of that forward in numpy
    rng = np.random.default_rng(23)
    B, H, N, Dh = 1, 2, 5, 3
    step = 2.0 ** -6
    cq, ck, cv = (rng.integers(0, 256, (B, H, N, Dh)) for _ in range(3))
    alpha, beta = np.full(H, 255.0 * step, np.float32), np.array([-2.0, -1.5], np.float32)
    Q, K, V = (c * step + beta[None, :, None, None].astype(np.float64) for c in (cq, ck, cv))
    dO = rng.standard_normal((B, H, N, Dh))
    scale = 0.7

    def softmax(s):
        e = np.exp(s - s.max(-1, keepdims=True))
        return e / e.sum(-1, keepdims=True)

    def loss(q, k, v):
        return float((dO * np.einsum("bhij,bhjd->bhid", softmax(scale * np.einsum("bhid,bhjd->bhij", q, k)), v)).sum())

    A = softmax(scale * np.einsum("bhid,bhjd->bhij", Q, K))
    # the attention map is not on a grid; give the oracle a fine one so that A_hat ~ A to 2^-21
    astep = 2.0 ** -8
    ca = np.rint(A / astep).astype(np.int64)
    assert ca.max() <= 255
    Ahat = ca * astep
    a_alpha, a_beta = np.full(H, 255.0 * astep, np.float32), np.zeros(H, np.float32)
    to_q = lambda c: (c - 128).astype(np.int8)
    dA, dV = R.attn_av_bwd_q(to_q(ca), to_q(cv), B, H, N, Dh, a_alpha, a_beta, alpha, beta, dO.astype(np.float32))
    dS = R.softmax_bwd_q(to_q(ca), B, H, N, N, a_alpha, a_beta, dA.astype(np.float32))
    dQ, dK = R.attn_qk_bwd_q(to_q(cq), to_q(ck), B, H, N, Dh, alpha, beta, alpha, beta, dS.astype(np.float32), scale)
    # dV is linear in A_hat; compare it at A_hat exactly, and dQ / dK to the tolerance the 8-bit attention map allows
    assert relerr(dV, np.einsum("bhij,bhid->bhjd", Ahat, dO.astype(np.float32).astype(np.float64))) < 1e-12
    gq = fd_grad(lambda q: loss(q, K, V), Q.copy())
    gk = fd_grad(lambda k: loss(Q, k, V), K.copy())
    gv = fd_grad(lambda v: loss(Q, K, v), V.copy())
    assert relerr(dV, gv) < 2e-2 and relerr(dQ, gq) < 5e-2 and relerr(dK, gk) < 5e-2
