"""Pins for the oracle's scale-only symmetric scheme (the comparison scheme of the ablation "asymmetric vs.
symmetric quantization", Sec. 5.2): a scale factor only, no offset, zero is a code.

Against what the definition fixes, never the oracle's formula retyped: zero and the whole grid round-trip exactly,
codes stay in [-127, 127], the error is at most half a step (one step under stochastic rounding), the quantizer is an
odd function under nearest rounding, scaling input and range by a power of two changes nothing, Eq. (4) is unbiased
on both sides of zero, the running scale follows Eq. (6)'s closed form, and on a clipping range symmetric about zero
the asymmetric quantizer of Eq. (3) agrees with it up to the code offset and one code.
"""
import numpy as np
import pytest

from oracle import mesa_ref as R


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("mode", [R.ROUND_NEAREST, R.ROUND_STOCHASTIC])
def test_zero_and_the_grid_round_trip_exactly(dtype, mode):
    # m = 127/8: r = 8 and the step 1/8 are exact, x = k/8 is exact in both storage types -> code k, x_hat = x
    m = np.array([127.0 / 8.0], np.float32)
    k = np.arange(-127, 128)
    x = (k / 8.0).astype(dtype)
    q = R.quantize_sym(x, (1, 1, x.size), m, mode, seed=3, offset=9)
    assert np.array_equal(q.astype(np.int64), k)
    xh = R.dequantize_sym(q, (1, 1, x.size), m, dtype)
    assert np.array_equal(xh.view(np.uint16 if dtype == np.float16 else np.uint32), x.view(np.uint16 if dtype == np.float16 else np.uint32))
    # zero is a code whatever the scale, and comes back as +0.0 or -0.0, never as a small number
    for mm in (0.3, 1.0, 11.7, 1e-3):
        q0 = R.quantize_sym(np.zeros(8, dtype), (1, 1, 8), np.array([mm], np.float32), mode, seed=1)
        assert np.all(q0 == 0)
        assert np.all(R.dequantize_sym(q0, (1, 1, 8), np.array([mm], np.float32)) == 0.0)


def test_codes_stay_in_the_signed_range_and_saturate():
    rng = np.random.default_rng(0)
    m = np.array([2.0], np.float32)
    x = np.concatenate([rng.standard_normal(5000) * 3.0, [1e6, -1e6, 2.0, -2.0, 2.0001, -2.0001]]).astype(np.float32)
    for mode in (R.ROUND_NEAREST, R.ROUND_STOCHASTIC):
        q = R.quantize_sym(x, (1, 1, x.size), m, mode, seed=5).astype(np.int64)
        assert q.min() == -127 and q.max() == 127          # -128 is never used: the code set is symmetric
        xh = R.dequantize_sym(q.astype(np.int8), (1, 1, x.size), m).astype(np.float64)
        out = np.abs(x) > 2.0
        assert np.all(np.abs(xh[out]) == 2.0) and np.all(np.sign(xh[out]) == np.sign(x[out]))


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_error_is_half_a_step_for_nearest_and_one_step_for_stochastic(dtype):
    rng = np.random.default_rng(1)
    m = np.array([0.7, 3.0, 11.0], np.float32)
    x = (rng.uniform(-1, 1, (50, 3, 200)) * m[None, :, None]).astype(dtype)
    step = (m.astype(np.float64) / 127.0)[None, :, None]
    lay = (50, 3, 200)
    xf = x.astype(np.float64)
    e_n = np.abs(R.dequantize_sym(R.quantize_sym(x, lay, m), lay, m).astype(np.float64) - xf)
    assert np.all(e_n <= step * (0.5 + 1e-5) + 1e-7)
    e_s = np.abs(R.dequantize_sym(R.quantize_sym(x, lay, m, R.ROUND_STOCHASTIC, seed=8), lay, m).astype(np.float64) - xf)
    assert np.all(e_s < step * (1.0 + 1e-5) + 1e-7)
    assert e_s.max() > 0.9 * step.min()                     # and it does use the whole step


def test_nearest_quantizer_is_odd_and_invariant_under_power_of_two_scaling():
    rng = np.random.default_rng(2)
    m = np.array([1.3, 5.1], np.float32)
    x = (rng.standard_normal((40, 2, 64)) * 2.0).astype(np.float32)
    lay = (40, 2, 64)
    q = R.quantize_sym(x, lay, m).astype(np.int64)
    assert np.array_equal(R.quantize_sym(-x, lay, m).astype(np.int64), -q)          # ties to even are symmetric
    assert np.array_equal(R.quantize_sym(x * np.float32(8.0), lay, m * np.float32(8.0)).astype(np.int64), q)
    assert np.array_equal(R.quantize_sym(x * np.float32(0.25), lay, m * np.float32(0.25)).astype(np.int64), q)
    # every element uses its own group's scale: swapping the scales changes the codes of both groups
    q_sw = R.quantize_sym(x, lay, m[::-1].copy()).astype(np.int64)
    assert (q_sw[:, 0] != q[:, 0]).mean() > 0.5 and (q_sw[:, 1] != q[:, 1]).mean() > 0.5


def test_stochastic_rounding_is_unbiased_on_both_sides_of_zero():
    m = np.array([127.0], np.float32)       # x_hat = code
    x = np.array([-100.9, -17.5, -3.25, -0.1, 0.1, 3.25, 17.5, 100.9], np.float32)
    n = 20000
    xs = np.tile(x, n)
    q = R.quantize_sym(xs, (1, 1, xs.size), m, R.ROUND_STOCHASTIC, seed=99, offset=7).astype(np.float64).reshape(n, x.size)
    assert np.all((q == np.floor(x)[None, :]) | (q == np.ceil(x)[None, :]))
    frac = (x - np.floor(x)).astype(np.float64)
    se = np.sqrt(frac * (1 - frac) / n)
    assert np.all(np.abs(q.mean(axis=0) - x) <= 4 * se + 2.0 ** -16), (q.mean(axis=0) - x, se)


def test_running_scale_first_call_lambda_zero_and_closed_form():
    rng = np.random.default_rng(3)
    x = (rng.standard_normal((6, 4, 50)) * np.array([0.5, 1.0, 3.0, 9.0])[None, :, None]).astype(np.float32)
    lay = (6, 4, 50)
    want = np.abs(x).max(axis=(0, 2))
    m1 = R.update_running_scale_sym(x, lay, np.full(4, 77.0, np.float32), 0.9, True)
    assert np.array_equal(m1, want)
    assert np.array_equal(R.update_running_scale_sym(x, lay, np.full(4, 77.0, np.float32), 0.0, False), want)
    # constant statistics: m_t = lam^t m_0 + (1 - lam^t) max|x|, fixed point max|x|
    m = np.full(4, 2.0, np.float32)
    for t in range(1, 40):
        m = R.update_running_scale_sym(x, lay, m, 0.9, False)
        closed = 0.9 ** t * 2.0 + (1 - 0.9 ** t) * want.astype(np.float64)
        assert np.allclose(m, closed, rtol=5e-6)
    assert np.array_equal(R.update_running_scale_sym(x, lay, want.copy(), 0.9, False).round(4), want.round(4))
    # shared across samples: permuting the batch changes nothing; the sign of the data is irrelevant
    assert np.array_equal(R.update_running_scale_sym(x[::-1].copy(), lay, np.zeros(4, np.float32), 0.9, True), want)
    assert np.array_equal(R.update_running_scale_sym(-x, lay, np.zeros(4, np.float32), 0.9, True), want)


def test_agrees_with_the_asymmetric_quantizer_on_a_range_symmetric_about_zero():
    """Eq. (3) with beta = -m and alpha = 2 m * 255/254 has the same step m/127 and its code 127 (x_bar = 127, q = -1)
    sits exactly on zero: x_bar - 127 is then the symmetric code, wherever neither scheme clips; the two
    reconstructions differ by rounding only."""
    rng = np.random.default_rng(4)
    m = np.array([4.0], np.float32)                      # powers of two keep both scales' arithmetic exact
    x = rng.uniform(-3.9, 3.9, 20000).astype(np.float32)
    lay = (1, 1, x.size)
    qs = R.quantize_sym(x, lay, m).astype(np.int64)
    alpha = np.array([2.0 * 4.0 * 255.0 / 254.0], np.float32)
    qa = R.quantize_headwise(x, lay, alpha, -m).astype(np.int64) + 128 - 127
    assert np.abs(qa - qs).max() <= 1 and (qa == qs).mean() > 0.99
    xs = R.dequantize_sym(qs.astype(np.int8), lay, m).astype(np.float64)
    xa = R.dequantize(R.quantize_headwise(x, lay, alpha, -m), lay, alpha, -m).astype(np.float64)
    assert np.abs(xs - xa).max() <= 4.0 / 127.0 + 1e-6
