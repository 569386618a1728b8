"""Pins for the oracle's running estimates (Sec. 3.2, Eq. 6-7; initialisation per Sec. 5.1) and for
its counter-based generator (published known-answer vectors)."""
import os

import numpy as np

from oracle import mesa_ref as R

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _x(seed, shape, dtype=np.float32):
    return (np.random.default_rng(seed).standard_normal(shape) * 3).astype(dtype)


def test_group_extrema_match_numpy_reductions():
    for dtype in (np.float32, np.float16):
        x = _x(0, (5, 4, 33), dtype)
        mn, mx = R.group_minmax(x, (5, 4, 33))
        assert np.array_equal(mn, x.astype(np.float32).min(axis=(0, 2)))
        assert np.array_equal(mx, x.astype(np.float32).max(axis=(0, 2)))


def test_first_call_sets_range_and_minimum_exactly():
    x = _x(1, (6, 3, 50))
    a, b = R.update_running_params(x, (6, 3, 50), np.full(3, 77.0), np.full(3, -55.0), 0.9, True)
    mn, mx = x.min(axis=(0, 2)), x.max(axis=(0, 2))
    assert np.array_equal(b, mn) and np.array_equal(a, mx - mn)


def test_lambda_zero_tracks_the_current_batch():
    # the paper's lambda = 0 row: parameters are the current min / max every iteration
    a, b = np.full(3, 9.0, np.float32), np.full(3, 9.0, np.float32)
    for it in range(3):
        x = _x(10 + it, (4, 3, 20))
        a, b = R.update_running_params(x, (4, 3, 20), a, b, 0.0, False)
        mn, mx = x.min(axis=(0, 2)), x.max(axis=(0, 2))
        assert np.array_equal(b, mn) and np.array_equal(a, mx - mn)


def test_constant_statistics_follow_the_closed_form_of_the_recursion():
    # alpha_t = lam^t alpha_0 + (1 - lam^t) * range, beta_t likewise with the minimum
    x = _x(2, (4, 2, 30))
    mn, mx = x.min(axis=(0, 2)).astype(np.float64), x.max(axis=(0, 2)).astype(np.float64)
    lam = 0.9
    a0, b0 = np.array([10.0, 0.5]), np.array([-7.0, 3.0])
    a, b = a0.astype(np.float32), b0.astype(np.float32)
    for t in range(1, 41):
        a, b = R.update_running_params(x, (4, 2, 30), a, b, lam, False)
        lt = np.float64(np.float32(lam)) ** t
        assert np.allclose(a, lt * a0 + (1 - lt) * (mx - mn), rtol=2e-6, atol=1e-6)
        assert np.allclose(b, lt * b0 + (1 - lt) * mn, rtol=2e-6, atol=1e-6)
    for _ in range(400):
        a, b = R.update_running_params(x, (4, 2, 30), a, b, lam, False)
    assert np.allclose(a, mx - mn, rtol=1e-6) and np.allclose(b, mn, rtol=1e-6)   # fixed point


def test_parameters_are_shared_across_samples():
    # permuting the samples of the batch, or the positions inside a group, changes nothing
    x = _x(3, (8, 3, 40), np.float16)
    a0, b0 = np.full(3, 2.0, np.float32), np.full(3, -1.0, np.float32)
    a, b = R.update_running_params(x, (8, 3, 40), a0, b0, 0.9, False)
    rng = np.random.default_rng(4)
    xp = x[rng.permutation(8)][:, :, rng.permutation(40)]
    a2, b2 = R.update_running_params(xp, (8, 3, 40), a0, b0, 0.9, False)
    assert np.array_equal(a, a2) and np.array_equal(b, b2)
    assert a.shape == (3,) and b.shape == (3,)    # 2 * N_h parameters per layer


def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLD, "philox4x32_10_kat.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(t, 16) for t in r]
        assert R.philox4x32(v[0:4], v[4:6], 10) == v[6:10]


def test_random_fractions_follow_the_documented_bit_assignment():
    # block b = e // 8 -> counter offset + b (64-bit, words 0-1), key = seed; element j takes 16 bits
    seed, offset = 0x0123456789ABCDEF, (1 << 32) - 3
    for e in (0, 1, 7, 8, 29, 63, 1000, (1 << 35) + 5):
        c = offset + (e >> 3)
        out = R.philox4x32([c & 0xFFFFFFFF, c >> 32, 0, 0], [seed & 0xFFFFFFFF, seed >> 32], 10)
        w = out[(e & 7) >> 1]
        bits = (w >> 16) if (e & 1) else (w & 0xFFFF)
        assert R.sr_uniform(seed, offset, e) == bits / 65536.0
    # advancing the offset by one block is the same as moving on by eight elements
    assert R.sr_uniform(5, 11, 3) == R.sr_uniform(5, 0, 3 + 8 * 11)


def test_random_fractions_are_uniform():
    u = np.array([R.sr_uniform(42, 0, e) for e in range(40000)])
    assert 0.0 <= u.min() and u.max() < 1.0
    hist, _ = np.histogram(u, bins=64, range=(0, 1))
    exp = u.size / 64
    chi2 = ((hist - exp) ** 2 / exp).sum()
    assert chi2 < 120          # 63 degrees of freedom, p ~ 1e-5
    assert abs(np.corrcoef(u[:-1], u[1:])[0, 1]) < 0.02


# ---- single-pass forward: codes with the parameters on entry, then Eq. 6-7 -------------------------------------

def _numpy_codes_nearest(x, a, b):
    """Eq. 3 written out in numpy, binary32 step by step (round half to even, then clip)."""
    x = x.astype(np.float32)
    r = np.where(a > 0, np.float32(255.0) / a, np.float32(0.0)).astype(np.float32)[None, :, None]
    t = (x - b[None, :, None]).astype(np.float32)
    v = (t * r).astype(np.float32)
    return (np.clip(np.rint(v), 0, 255).astype(np.int32) - 128).astype(np.int8)


def test_fused_forward_quantizes_with_the_old_parameters_then_moves_them():
    lay = (7, 3, 41)
    x = _x(31, lay)
    a0 = np.array([4.0, 11.0, 25.0], np.float32)      # deliberately far from this batch's range
    b0 = np.array([-1.0, -6.0, -14.0], np.float32)
    q, a1, b1 = R.quantize_update_fused(x, lay, a0, b0, 0.9)
    # codes: those of Eq. 3 with (a0, b0), not with the updated parameters
    assert np.array_equal(q, _numpy_codes_nearest(x, a0, b0))
    assert not np.array_equal(q, _numpy_codes_nearest(x, a1, b1))
    # parameters: Eq. 6-7 from (a0, b0) and this batch's extrema, one binary32 operation at a time
    mn, mx = x.min(axis=(0, 2)), x.max(axis=(0, 2))
    lam, one_m = np.float32(0.9), np.float32(1.0) - np.float32(0.9)
    assert np.array_equal(a1, (lam * a0 + one_m * (mx - mn).astype(np.float32)).astype(np.float32))
    assert np.array_equal(b1, (lam * b0 + one_m * mn).astype(np.float32))


def test_fused_forward_lags_the_two_pass_order_by_exactly_one_step():
    # two-pass order (update, then quantize) at step t uses theta_t; the single pass uses theta_{t-1}:
    # feeding the single pass the parameters the two-pass order had one step earlier gives the same
    # parameter sequence, and its codes at step t equal two-pass codes taken with theta_{t-1}.
    lay = (5, 2, 64)
    xs = [_x(40 + t, lay, np.float16) for t in range(4)]
    a, b = R.update_running_params(xs[0], lay, np.zeros(2), np.zeros(2), 0.9, True)
    fa, fb = a.copy(), b.copy()
    for t in range(1, 4):
        q_prev_params = R.quantize_headwise(xs[t], lay, a, b, R.ROUND_STOCHASTIC, 5, 1000 * t)
        a, b = R.update_running_params(xs[t], lay, a, b, 0.9, False)
        fq, fa, fb = R.quantize_update_fused(xs[t], lay, fa, fb, 0.9, R.ROUND_STOCHASTIC, 5, 1000 * t)
        assert np.array_equal(fq, q_prev_params)
        assert np.array_equal(fa, a) and np.array_equal(fb, b)


def test_fused_forward_constant_group_and_saturation():
    lay = (3, 2, 16)
    x = np.zeros(lay, np.float32)
    x[:, 1, :] = np.linspace(-50, 50, 48, dtype=np.float32).reshape(3, 16)
    q, a1, b1 = R.quantize_update_fused(x, lay, np.array([0.0, 10.0], np.float32), np.array([0.0, -5.0], np.float32), 0.5)
    assert (q[:, 0, :] == -128).all()                      # alpha = 0: every code is 0 (stored -128)
    assert q[:, 1, :].min() == -128 and q[:, 1, :].max() == 127   # values outside [beta, beta + alpha] saturate
    assert a1[0] == 0.0 and b1[0] == 0.0 and a1[1] == np.float32(0.5 * 10.0 + 0.5 * 100.0) and b1[1] == np.float32(-2.5 - 25.0)


# ---- symmetric range (Sec. 5.2, asymmetric vs. symmetric quantization) --------------------------------

def test_symmetric_first_call_is_twice_and_minus_the_largest_magnitude():
    for dtype in (np.float32, np.float16):
        x = _x(40, (6, 3, 50), dtype)
        a, b = R.update_running_params_sym(x, (6, 3, 50), np.full(3, 77.0), np.full(3, -55.0), 0.9, True)
        m = np.abs(x.astype(np.float32)).max(axis=(0, 2))
        assert np.array_equal(a, 2 * m) and np.array_equal(b, -m)


def test_symmetric_update_equals_the_asymmetric_one_on_the_batch_with_its_mirror_image():
    # the extrema of the batch joined with its negation are -max|x| and +max|x|: Eq. (6)-(7) on that
    # joined batch is the symmetric update, whatever lambda and the previous estimates are
    lay, lay2 = (4, 2, 30), (8, 2, 30)
    a0, b0 = np.array([3.0, 5.0], np.float32), np.array([-1.0, -4.0], np.float32)
    for seed, lam in ((41, 0.9), (42, 0.5), (43, 0.0)):
        x = _x(seed, lay) + 0.7          # skewed, so that min != -max
        joined = np.concatenate([x, -x], axis=0)
        a, b = R.update_running_params_sym(x, lay, a0, b0, lam, False)
        a2, b2 = R.update_running_params(joined, lay2, a0, b0, lam, False)
        assert np.array_equal(a, a2) and np.array_equal(b, b2)
        assert not np.array_equal(R.update_running_params(x, lay, a0, b0, lam, False)[1], b)


def test_symmetric_range_bounds_the_nearest_rounding_error_and_centres_zero():
    lay = (5, 3, 64)
    x = _x(44, lay) - 1.0
    a, b = R.update_running_params_sym(x, lay, np.zeros(3), np.zeros(3), 0.9, True)
    q = R.quantize_headwise(x, lay, a, b, R.ROUND_NEAREST, 0, 0)
    xh = R.dequantize(q, lay, a, b)
    step = (a / 255.0)[None, :, None]
    assert np.all(np.abs(xh.reshape(lay) - x) <= 0.5 * step * (1 + 1e-5) + 1e-6)
    # zero sits in the middle of the code range: codes 127 / 128 (-1 / 0 as stored) dequantize to -+ step/2
    z = R.dequantize(np.array([[-1, 0]] * 3, np.int8).reshape(1, 3, 2), (1, 3, 2), a, b).reshape(3, 2)
    assert np.allclose(z[:, 0], -0.5 * a / 255, rtol=1e-5, atol=4e-6) and np.allclose(z[:, 1], 0.5 * a / 255, rtol=1e-5, atol=4e-6)


# ---- fixed offset (Sec. 6: beta of the second FFN layer's input stays at GELU's minimum) ---------------

def test_fixed_offset_tracks_the_maximum_above_it():
    lay = (6, 3, 50)
    bf = np.float32(-0.17)
    x0 = _x(50, lay)
    a, b = R.update_running_params_fixed_beta(x0, lay, np.full(3, 9.0), 0.9, True, bf)
    assert np.array_equal(b, np.full(3, bf)) and np.array_equal(a, x0.max(axis=(0, 2)) - bf)
    # lambda = 0: the current batch's maximum above the offset, every time
    for it in range(3):
        x = _x(51 + it, lay)
        a, b = R.update_running_params_fixed_beta(x, lay, a, 0.0, False, bf)
        assert np.array_equal(a, x.max(axis=(0, 2)) - bf) and np.array_equal(b, np.full(3, bf))


def test_fixed_offset_equals_the_general_update_when_the_minimum_is_the_offset():
    # a GELU output whose minimum the batch attains: Eq. (6) for alpha is the same recursion in both forms
    lay = (8, 2, 64)
    bf = np.float32(-0.17)
    rng = np.random.default_rng(55)
    a_g, a_f = np.array([2.0, 3.0], np.float32), np.array([2.0, 3.0], np.float32)
    b_g = np.full(2, bf)
    for it in range(4):
        x = np.maximum(rng.standard_normal(lay).astype(np.float32) * 2, bf)
        x[0, :, 0] = bf
        a_g, b_g = R.update_running_params(x, lay, a_g, b_g, 0.9, False)
        a_f, b_f = R.update_running_params_fixed_beta(x, lay, a_f, 0.9, False, bf)
        assert np.array_equal(a_g, a_f)
        assert np.allclose(b_g, bf, rtol=3e-7, atol=0) and np.array_equal(b_f, np.full(2, bf))
