"""Pins for the oracle's quantizer / dequantizer (Sec. 3.2, Eq. 3-5) and its binary16 conversions.

Every check here is against something the paper or the mathematics fixes, never against the
oracle's own formula retyped: code range, error bounds, exact round trip on the grid, brute force
over all 256 reconstruction levels, unbiasedness of Eq. (4), numpy's float16 as a library routine.
"""
import numpy as np
import pytest
import torch

import mesa_workloads as W
from oracle import mesa_ref as R


def test_half_conversions_match_numpy():
    rng = np.random.default_rng(0)
    # float -> half on random magnitudes across the whole half range, plus ties and specials
    v = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * np.float32(10.0) ** rng.integers(-9, 6, 20000).astype(np.float32),
        np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e-8, 2.0 ** -25, 2.0 ** -24, 3 * 2.0 ** -25,
                  1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -25, np.inf, -np.inf], np.float32),
    ])
    want = v.astype(np.float16).view(np.uint16)
    got = np.array([R.float_to_half(float(x)) for x in v], np.uint16)
    assert np.array_equal(got, want)
    # half -> float, every finite pattern
    bits = np.arange(65536, dtype=np.uint16)
    f = bits.view(np.float16).astype(np.float32)
    mine = np.array([R.half_to_float(int(b)) for b in bits], np.float32)
    fin = np.isfinite(f)
    assert np.array_equal(mine[fin].view(np.uint32), f[fin].view(np.uint32))


def test_codes_stay_in_int8_range_even_far_outside_the_clipping_range():
    # Eq. (3) clips to [0, 255]; stored signed that is [-128, 127]
    x = np.array([-1e30, -1e4, -3.0, -1.0, 0.0, 0.5, 1.0, 2.0, 1e4, 1e30], np.float32)
    for mode in (R.ROUND_NEAREST, R.ROUND_STOCHASTIC):
        q = R.quantize_headwise(x, (1, 1, x.size), [2.0], [-1.0], mode, seed=3)
        assert q.dtype == np.int8
        assert q.min() == -128 and q.max() == 127
        assert list(q[:3]) == [-128, -128, -128] and list(q[-3:]) == [127, 127, 127]


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_round_trip_error_is_at_most_half_a_step_for_nearest_and_one_step_for_stochastic(dtype):
    rng = np.random.default_rng(1)
    G, inner, outer = 4, 257, 9
    x = (rng.standard_normal((outer, G, inner)) * np.array([0.3, 1.0, 5.0, 40.0])[None, :, None]).astype(dtype)
    a, b = R.update_running_params(x, (outer, G, inner), np.zeros(G), np.zeros(G), 0.9, True)
    step = a.astype(np.float64) / 255.0
    xf = x.astype(np.float64)
    for mode, bound in ((R.ROUND_NEAREST, 0.5), (R.ROUND_STOCHASTIC, 1.0)):
        q = R.quantize_headwise(x, (outer, G, inner), a, b, mode, seed=5, offset=7)
        xh = R.dequantize(q, (outer, G, inner), a, b, np.float32).astype(np.float64)
        err = np.abs(xh - xf) / step[None, :, None]
        # slack: a few binary32 roundings of values up to 255 steps
        assert err.max() <= bound + 1e-4, (mode, err.max())
    # nearest rounding is the tight case: some element sits close to half a step away
    q = R.quantize_headwise(x, (outer, G, inner), a, b, R.ROUND_NEAREST)
    xh = R.dequantize(q, (outer, G, inner), a, b, np.float32).astype(np.float64)
    assert (np.abs(xh - xf) / step[None, :, None]).max() > 0.45


def test_saturation_error_is_distance_to_the_range_end():
    a, b = np.array([2.0], np.float32), np.array([-1.0], np.float32)
    x = np.array([-4.0, 3.5], np.float32)   # both outside [beta, beta + alpha] = [-1, 1]
    q = R.quantize_headwise(x, (1, 1, 2), a, b)
    xh = R.dequantize(q, (1, 1, 2), a, b)
    assert np.allclose(xh, [-1.0, 1.0], atol=1e-6)


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("mode", [R.ROUND_NEAREST, R.ROUND_STOCHASTIC])
def test_values_on_the_grid_round_trip_exactly(dtype, mode):
    # alpha = 255/8, beta = -4: step 1/8 and 255/alpha = 8 are exact, x = beta + k/8 is exact in
    # both storage types, so code k comes back as x bit for bit in either rounding mode
    k = np.arange(256)
    x = (-4.0 + k / 8.0).astype(dtype)
    a, b = np.array([255.0 / 8.0], np.float32), np.array([-4.0], np.float32)
    q = R.quantize_headwise(x, (1, 1, 256), a, b, mode, seed=99, offset=123)
    assert np.array_equal(q.astype(np.int64) + 128, k)
    xh = R.dequantize(q, (1, 1, 256), a, b, dtype)
    assert np.array_equal(xh.view(np.uint16 if dtype == np.float16 else np.uint32),
                          x.view(np.uint16 if dtype == np.float16 else np.uint32))


def test_nearest_codes_are_monotone_in_x():
    rng = np.random.default_rng(2)
    x = np.sort(rng.uniform(-3, 7, 5000).astype(np.float32))
    q = R.quantize_headwise(x, (1, 1, x.size), [9.3], [-2.9])
    assert np.all(np.diff(q.astype(np.int32)) >= 0)


def test_nearest_rounding_picks_the_closest_of_all_256_levels():
    rng = np.random.default_rng(3)
    a, b = np.array([3.7], np.float32), np.array([-1.3], np.float32)
    levels = R.dequantize(np.arange(-128, 128, dtype=np.int8), (1, 1, 256), a, b).astype(np.float64)
    x = rng.uniform(-1.3, 2.4, 4000).astype(np.float32)
    q = R.quantize_headwise(x, (1, 1, x.size), a, b).astype(np.int64) + 128
    d = np.abs(levels[None, :] - x.astype(np.float64)[:, None])
    best = d.argmin(axis=1)
    srt = np.sort(d, axis=1)
    clear = (srt[:, 1] - srt[:, 0]) > 1e-5   # leave out near-ties between two levels
    assert clear.mean() > 0.99
    assert np.array_equal(q[clear], best[clear])


def test_stochastic_rounding_takes_floor_or_ceil_and_is_unbiased():
    # Eq. (4): result is floor or ceil, ceil with probability frac -> E[x_hat] = x inside the range
    a, b = np.array([255.0], np.float32), np.array([0.0], np.float32)   # v = x, codes = integers
    x = np.array([0.1, 3.25, 17.5, 100.9, 254.01, 200.0], np.float32)
    n = 4096
    xs = np.tile(x, n)
    q = R.quantize_headwise(xs, (1, 1, xs.size), a, b, R.ROUND_STOCHASTIC, seed=2024).astype(np.int64) + 128
    q = q.reshape(n, x.size)
    assert np.all((q == np.floor(x)[None, :]) | (q == np.ceil(x)[None, :]))
    frac = x - np.floor(x)
    mean = q.mean(axis=0)
    se = np.sqrt(np.maximum(frac * (1 - frac), 1e-12) / n)
    assert np.all(np.abs(mean - x) <= 4 * se + 1e-6), (mean - x, se)
    # a different seed and a different offset give different draws
    q2 = R.quantize_headwise(xs, (1, 1, xs.size), a, b, R.ROUND_STOCHASTIC, seed=2025).astype(np.int64) + 128
    q3 = R.quantize_headwise(xs, (1, 1, xs.size), a, b, R.ROUND_STOCHASTIC, seed=2024, offset=10 ** 6).astype(np.int64) + 128
    assert (q2.reshape(n, -1) != q).mean() > 0.1 and (q3.reshape(n, -1) != q).mean() > 0.1


def test_each_element_uses_the_parameters_of_its_own_group():
    # x = 1 everywhere, alpha = 255, beta_g = -g  ->  code = 1 + g, whatever the position
    outer, G, inner = 3, 5, 7
    x = np.ones((outer, G, inner), np.float32)
    beta = -np.arange(G, dtype=np.float32)
    q = R.quantize_headwise(x, (outer, G, inner), np.full(G, 255.0, np.float32), beta).astype(np.int64) + 128
    want = np.broadcast_to((1 + np.arange(G))[None, :, None], (outer, G, inner))
    assert np.array_equal(q, want)
    xh = R.dequantize((want - 128).astype(np.int8), (outer, G, inner), np.full(G, 255.0, np.float32), beta)
    assert np.array_equal(xh, x)


def test_constant_group_gives_lowest_code_and_beta_back():
    x = np.full(50, 2.5, np.float32)
    a, b = R.update_running_params(x, (1, 1, 50), [0.0], [0.0], 0.9, True)
    assert a[0] == 0.0 and b[0] == 2.5
    for mode in (R.ROUND_NEAREST, R.ROUND_STOCHASTIC):
        q = R.quantize_headwise(x, (1, 1, 50), a, b, mode, seed=1)
        assert np.all(q == -128)
    assert np.array_equal(R.dequantize(q, (1, 1, 50), a, b), x)


def test_head_wise_error_is_far_below_layer_wise_on_heterogeneous_heads():
    # Sec. 3.2's motivation: heads with very different statistics need their own range and offset.
    # Pre-softmax logits of the tiny DeiT-Ti-shaped block, head std 0.5 / 1.5 / 4.0.
    spec = W.CONFIGS[1]
    B, H, N, _ = spec.attn
    g = torch.Generator().manual_seed(0)
    logits = (torch.randn((B, H, N, N), generator=g) * torch.tensor(spec.sigma).view(1, H, 1, 1)).numpy()
    lay_h = (B, H, N * N)
    a, b = R.update_running_params(logits, lay_h, np.zeros(H), np.zeros(H), 0.9, True)
    xh = R.dequantize(R.quantize_headwise(logits, lay_h, a, b), lay_h, a, b)
    lay_1 = (1, 1, logits.size)
    a1, b1 = R.update_running_params(logits, lay_1, [0.0], [0.0], 0.9, True)
    x1 = R.dequantize(R.quantize_headwise(logits, lay_1, a1, b1), lay_1, a1, b1)
    err_h = ((xh - logits) ** 2).reshape(B, H, -1).sum(axis=(0, 2))
    err_1 = ((x1.reshape(logits.shape) - logits) ** 2).reshape(B, H, -1).sum(axis=(0, 2))
    # the narrow heads gain the most; the total drops too
    assert err_h[0] < err_1[0] / 20 and err_h[1] < err_1[1] / 3
    assert err_h.sum() < 0.6 * err_1.sum()


def test_attention_offsets_are_non_negative():
    # the visualisation section notes that attention after softmax is non-negative, so beta >= 0 there
    spec = W.small_case()
    y = W.attention_map(spec).numpy()
    a, b = R.update_running_params(y, spec.attn_layout, np.zeros(spec.heads), np.zeros(spec.heads), 0.9, True)
    assert np.all(b >= 0) and np.all(a > 0) and np.all(a + b <= 1.0 + 1e-6)


def test_bfloat16_conversions_match_torch():
    """The oracle's own bfloat16 rounding (nearest, ties to even on the dropped 16 bits) against torch's CPU conversion,
    a library routine for exactly this, on random magnitudes plus ties, carries into the exponent and the overflow to
    infinity; widening back is exact."""
    rng = np.random.default_rng(1)
    v = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * np.float32(10.0) ** rng.integers(-30, 30, 20000).astype(np.float32),
        np.array([0.0, -0.0, 1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -7, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20,
                  1.99609375, 1.998046875, 3.3895313892515355e38, 3.4e38, -3.4e38, 1e-40, 2.0 ** -133, np.inf, -np.inf],
                 np.float32),
    ])
    want = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([R.float_to_bf16(float(x)) for x in v], np.uint16)
    assert np.array_equal(got, want), np.nonzero(got != want)[0][:5]
    bits = np.arange(0, 65536, 7, dtype=np.uint16)
    wide = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).float().numpy()
    mine = np.array([R.bf16_to_float(int(b)) for b in bits], np.float32)
    fin = np.isfinite(wide)
    assert np.array_equal(mine[fin].view(np.uint32), wide[fin].view(np.uint32))
    # and the de-quantizer's bfloat16 output is its binary32 output rounded that way
    q = np.arange(-128, 128, dtype=np.int8)
    a, b = np.array([3.7], np.float32), np.array([-1.3], np.float32)
    x32 = R.dequantize(q, (1, 1, 256), a, b, np.float32)
    xb = R.dequantize(q, (1, 1, 256), a, b, "bf16")
    assert np.array_equal(xb, torch.from_numpy(x32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_nearest_rounding_sends_exact_half_steps_to_the_even_code(dtype):
    """Tie rule of the nearest mode: x = beta + (k + 1/2) * s on a grid where everything is exact (s = 1/8, beta = -4:
    x is a multiple of 1/16, exact in binary16 too, and v = (x - beta) * 8 = k + 1/2 exactly) must give the EVEN
    neighbour for every k -- round-half-away-from-zero or round-half-up would give k + 1 throughout."""
    a, b = np.array([255.0 / 8.0], np.float32), np.array([-4.0], np.float32)
    k = np.arange(0, 255)
    x = (b[0] + (k + 0.5) / 8.0).astype(dtype)
    assert np.array_equal(x.astype(np.float64), -4.0 + (k + 0.5) / 8.0)          # the inputs are exact
    u = R.quantize_headwise(x, (1, 1, x.size), a, b, R.ROUND_NEAREST).astype(np.int64) + 128
    even = np.where(k % 2 == 0, k, k + 1)
    assert np.array_equal(u, even)
    assert np.all(u % 2 == 0)
    # a little off the tie (an eighth of a step or less; every value still exact) the nearer neighbour wins on either side
    e = -10 if dtype == np.float32 else -6
    d = dtype(2.0 ** e)
    lo = R.quantize_headwise(x - d, (1, 1, x.size), a, b, R.ROUND_NEAREST).astype(np.int64) + 128
    hi = R.quantize_headwise(x + d, (1, 1, x.size), a, b, R.ROUND_NEAREST).astype(np.int64) + 128
    assert np.array_equal((x - d).astype(np.float64), x.astype(np.float64) - 2.0 ** e)
    assert np.array_equal(lo, k) and np.array_equal(hi, k + 1)


def test_stochastic_rounding_is_unbiased_over_many_draws():
    """Eq. (4): E[x_hat] = x.  Twenty thousand independent draws (distinct counter blocks) per value, the mean
    reconstruction within four standard errors of x, for fractions across (0, 1) including tiny ones."""
    a, b = np.array([255.0], np.float32), np.array([0.0], np.float32)   # x_hat = code
    x = np.array([0.015625, 0.1, 3.25, 17.5, 100.9, 254.01, 77.984375, 200.0], np.float32)   # one Philox block per row
    n = 20000
    xs = np.tile(x, n)
    q = R.quantize_headwise(xs, (1, 1, xs.size), a, b, R.ROUND_STOCHASTIC, seed=777, offset=12345).astype(np.int64) + 128
    xh = R.dequantize((q - 128).astype(np.int8), (1, 1, xs.size), a, b).astype(np.float64).reshape(n, x.size)
    assert np.all((xh == np.floor(x)[None, :]) | (xh == np.ceil(x)[None, :]))
    frac = (x - np.floor(x)).astype(np.float64)
    se = np.sqrt(np.maximum(frac * (1 - frac), 1e-12) / n)
    assert np.all(np.abs(xh.mean(axis=0) - x) <= 4 * se + 2.0 ** -16), (xh.mean(axis=0) - x, se)
    # the empirical probability of rounding up is the fraction, to the generator's 16-bit resolution
    up = (xh == np.ceil(x)[None, :]).mean(axis=0)[frac > 0]
    assert np.all(np.abs(up - frac[frac > 0]) <= 4 * se[frac > 0] + 2.0 ** -16)
