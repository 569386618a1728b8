"""Pins for the oracle's four-bit codes (Eq. 3-5 with 15 steps, two codes per byte): the packing order stated in the
header on a hand-written example, code range and error bounds, exact round trip on the grid, agreement with the 8-bit
path on values both grids share (255 = 15 x 17: every four-bit level is the 8-bit level 17 k), unbiasedness of Eq. 4,
and the GELU gradient against torch's autograd at the de-quantized input."""
import numpy as np
import pytest
import torch

from oracle import mesa_ref as R


def test_packing_order_low_nibble_first():
    # alpha = 15, beta = 0: v = x, codes = round(x).  Seven elements -> four bytes, the last high nibble zero.
    a, b = np.array([15.0], np.float32), np.array([0.0], np.float32)
    x = np.array([1, 2, 3, 4, 15, 0, 9], np.float32)
    q4 = R.quantize_headwise_b4(x, (1, 1, 7), a, b)
    assert q4.tolist() == [0x21, 0x43, 0x0F, 0x09]
    assert np.array_equal(R.dequantize_b4(q4, (1, 1, 7), a, b), x)


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_range_error_bounds_and_saturation(dtype):
    rng = np.random.default_rng(0)
    a, b = np.array([3.0, 7.5], np.float32), np.array([-1.0, -5.0], np.float32)
    lay = (40, 2, 33)                                    # odd slabs: nibble pairs straddle groups
    x = (b[None, :, None] + a[None, :, None] * rng.uniform(0, 1, lay)).astype(dtype)
    xf = x.astype(np.float64).reshape(-1)
    step = np.repeat((a.astype(np.float64) / 15.0)[None, :, None], 40, 0).repeat(33, 2).reshape(-1)
    for mode, bound in ((R.ROUND_NEAREST, 0.5), (R.ROUND_STOCHASTIC, 1.0)):
        q4 = R.quantize_headwise_b4(x, lay, a, b, mode, seed=4)
        xh = R.dequantize_b4(q4, lay, a, b).astype(np.float64)
        tol = 2e-3 if dtype == np.float16 else 1e-6        # the input's own rounding moves it off [beta, beta + alpha] a little
        assert np.all(np.abs(xh - xf) <= step * bound * (1 + 1e-5) + tol)
    far = np.array([-100.0, 100.0, -1.0, 2.0], np.float32)
    q4 = R.quantize_headwise_b4(far, (1, 1, 4), a[:1], b[:1])
    assert q4.tolist() == [0xF0, 0xF0]


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("mode", [R.ROUND_NEAREST, R.ROUND_STOCHASTIC])
def test_grid_round_trip_and_agreement_with_the_eight_bit_path(dtype, mode):
    # alpha = 15/8, beta = -1: r = 8, step 1/8, x = beta + k/8 exact in both storage types
    a, b = np.array([15.0 / 8.0], np.float32), np.array([-1.0], np.float32)
    k = np.tile(np.arange(16), 5)
    x = (b[0] + k / 8.0).astype(dtype)
    lay = (1, 1, x.size)
    q4 = R.quantize_headwise_b4(x, lay, a, b, mode, seed=9, offset=3)
    codes = np.stack([q4 & 15, q4 >> 4], 1).reshape(-1)[:x.size]
    assert np.array_equal(codes, k)
    xh = R.dequantize_b4(q4, lay, a, b, dtype)
    assert np.array_equal(xh.astype(np.float64), x.astype(np.float64))
    # the same values through Eq. 3 with 255 steps land on the codes 17 k and come back as the same numbers
    q8 = R.quantize_headwise(x, lay, a, b, mode, seed=9, offset=3).astype(np.int64) + 128
    assert np.array_equal(q8, 17 * k)
    assert np.array_equal(R.dequantize((q8 - 128).astype(np.int8), lay, a, b, np.float32).astype(np.float64), x.astype(np.float64))


def test_stochastic_rounding_is_unbiased_with_fifteen_steps():
    a, b = np.array([15.0], np.float32), np.array([0.0], np.float32)
    x = np.array([0.1, 3.25, 7.5, 14.9, 0.015625, 11.984375, 5.0, 9.75], np.float32)
    n = 20000
    xs = np.tile(x, n)
    q4 = R.quantize_headwise_b4(xs, (1, 1, xs.size), a, b, R.ROUND_STOCHASTIC, seed=31, offset=5)
    xh = R.dequantize_b4(q4, (1, 1, xs.size), a, b).astype(np.float64).reshape(n, x.size)
    assert np.all((xh == np.floor(x)[None, :]) | (xh == np.ceil(x)[None, :]))
    frac = (x - np.floor(x)).astype(np.float64)
    se = np.sqrt(np.maximum(frac * (1 - frac), 1e-12) / n)
    assert np.all(np.abs(xh.mean(axis=0) - x) <= 4 * se + 2.0 ** -16)


def test_gelu_gradient_at_the_four_bit_reconstruction_matches_autograd():
    rng = np.random.default_rng(2)
    lay = (7, 3, 19)
    a, b = np.array([6.0, 2.0, 9.0], np.float32), np.array([-3.0, -1.0, -4.0], np.float32)
    x = (rng.standard_normal(lay) * 1.5).astype(np.float32)
    dy = rng.standard_normal(lay).astype(np.float32)
    q4 = R.quantize_headwise_b4(x, lay, a, b, R.ROUND_STOCHASTIC, seed=1)
    xh = torch.from_numpy(R.dequantize_b4(q4, lay, a, b).astype(np.float64)).requires_grad_(True)
    torch.nn.functional.gelu(xh).backward(torch.from_numpy(dy.astype(np.float64).reshape(-1)))
    got = R.gelu_bwd_q_b4(q4, lay, a, b, dy)
    assert np.allclose(got, xh.grad.numpy(), rtol=1e-12, atol=1e-14)
