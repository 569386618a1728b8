"""Pins for the oracle's convolution weight gradient (Eq. 2 for a convolutional layer, Sec. 3.3): a worked example
small enough to do by hand, the count of in-image positions per kernel tap (zero padding contributes nothing, whatever
beta is), torch's own weight gradient of conv2d on the de-quantized input over strides, paddings, dilations and
rectangular kernels, the 1x1 case against the Linear weight gradient, and the sampled-entries form against the full one."""
import numpy as np
import pytest
import torch

from oracle import mesa_ref as R


def test_worked_example_by_hand():
    # alpha = 255, beta = -128: x_hat equals the code.  One 3x3 image, one 2x2 kernel, no padding: 2x2 outputs.
    a, b = np.array([255.0], np.float32), np.array([-128.0], np.float32)
    xq = np.arange(1, 10, dtype=np.int8)                       # [[1,2,3],[4,5,6],[7,8,9]]
    dy = np.array([[1, 2], [3, 4]], np.float32)
    geom, OH, OW = R.conv_geometry(1, 1, 3, 3, 1, 2, 2)
    assert (OH, OW) == (2, 2)
    dW, db = R.conv2d_dw_q(xq, geom, 1, a, b, dy)
    # dW[kh,kw] = 1*x[kh,kw] + 2*x[kh,kw+1] + 3*x[kh+1,kw] + 4*x[kh+1,kw+1]
    assert dW.reshape(2, 2).tolist() == [[37.0, 47.0], [67.0, 77.0]]
    assert db.tolist() == [10.0]


def test_padding_contributes_nothing():
    # every code equal, beta far from zero: x_hat = c inside the image; outside it the forward saw zeros.
    a, b = np.array([2.55], np.float32), np.array([3.0], np.float32)
    xq = np.full(2 * 4 * 4, -28, np.int8)                      # x_hat = 100 * 0.01 + 3 = 4 (up to binary32 rounding)
    c = float(R.dequantize(xq[:1], (1, 1, 1), a, b)[0])
    assert abs(c - 4.0) < 1e-5
    dy = np.ones((1, 1, 4, 4), np.float32)
    geom, OH, OW = R.conv_geometry(1, 2, 4, 4, 1, 3, 3, pad=(1, 1))
    assert (OH, OW) == (4, 4)
    dW, _ = R.conv2d_dw_q(xq, geom, 1, a, b, dy)
    counts = np.array([[9, 12, 9], [12, 16, 12], [9, 12, 9]], np.float64)   # outputs whose tap lands inside a 4x4 image
    for ci in range(2):
        assert np.allclose(dW[0, ci], c * counts, rtol=0, atol=1e-12)


CASES = [  # B, Cin, H, W, Cout, KH, KW, stride, pad, dil, G
    (2, 4, 7, 9, 3, 3, 3, (1, 1), (1, 1), (1, 1), 2),
    (2, 6, 9, 8, 4, 3, 2, (2, 1), (0, 1), (1, 1), 3),
    (1, 4, 11, 10, 2, 3, 3, (1, 2), (2, 2), (2, 2), 1),
    (3, 2, 6, 6, 5, 1, 1, (1, 1), (0, 0), (1, 1), 2),
    (2, 3, 8, 8, 2, 4, 4, (4, 4), (0, 0), (1, 1), 3),
    (1, 2, 5, 12, 2, 1, 5, (1, 3), (0, 4), (1, 2), 1),
]


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_against_torch_conv2d_weight_gradient(case, dtype):
    B, Cin, H, W, Cout, KH, KW, stride, pad, dil, G = case
    rng = np.random.default_rng(sum(case[:7]))
    geom, OH, OW = R.conv_geometry(B, Cin, H, W, Cout, KH, KW, stride, pad, dil)
    xq = rng.integers(-128, 128, (B, Cin, H, W)).astype(np.int8)
    a = rng.uniform(0.5, 4.0, G).astype(np.float32)
    b = rng.uniform(-2.0, 1.0, G).astype(np.float32)
    dy = rng.standard_normal((B, Cout, OH, OW)).astype(dtype)
    dW, db = R.conv2d_dw_q(xq, geom, G, a, b, dy)
    xh = R.dequantize(xq.reshape(-1), (B, G, (Cin // G) * H * W), a, b).reshape(B, Cin, H, W).astype(np.float64)
    ref = torch.nn.grad.conv2d_weight(torch.from_numpy(xh), (Cout, Cin, KH, KW), torch.from_numpy(dy.astype(np.float64)),
                                      stride=stride, padding=pad, dilation=dil).numpy()
    assert np.allclose(dW, ref, rtol=1e-11, atol=1e-11)
    assert np.allclose(db, dy.astype(np.float64).sum(axis=(0, 2, 3)), rtol=1e-12, atol=1e-12)


def test_one_by_one_kernel_is_the_linear_weight_gradient():
    rng = np.random.default_rng(5)
    B, Cin, H, W, Cout, G = 2, 6, 5, 4, 3, 3
    geom, OH, OW = R.conv_geometry(B, Cin, H, W, Cout, 1, 1)
    xq = rng.integers(-128, 128, (B, Cin, H, W)).astype(np.int8)
    a = rng.uniform(0.5, 4.0, G).astype(np.float32)
    b = rng.uniform(-2.0, 1.0, G).astype(np.float32)
    dy = rng.standard_normal((B, Cout, OH, OW)).astype(np.float32)
    dW, db = R.conv2d_dw_q(xq, geom, G, a, b, dy)
    rows = B * H * W                                           # pixels as rows, channels last
    lw, lb = R.linear_dw_q(xq.transpose(0, 2, 3, 1).reshape(rows, Cin), rows, Cin, G, a, b,
                           dy.transpose(0, 2, 3, 1).reshape(rows, Cout), Cout)
    assert np.allclose(dW.reshape(Cout, Cin), lw, rtol=1e-12, atol=1e-12)
    assert np.allclose(db, lb, rtol=1e-12, atol=1e-12)


def test_sampled_entries_equal_the_full_gradient():
    case = CASES[1]
    B, Cin, H, W, Cout, KH, KW, stride, pad, dil, G = case
    rng = np.random.default_rng(8)
    geom, OH, OW = R.conv_geometry(B, Cin, H, W, Cout, KH, KW, stride, pad, dil)
    xq = rng.integers(-128, 128, (B, Cin, H, W)).astype(np.int8)
    a = rng.uniform(0.5, 4.0, G).astype(np.float32)
    b = rng.uniform(-2.0, 1.0, G).astype(np.float32)
    dy = rng.standard_normal((B, Cout, OH, OW)).astype(np.float16)
    dW, _ = R.conv2d_dw_q(xq, geom, G, a, b, dy)
    idx = np.stack([rng.integers(0, Cout, 40), rng.integers(0, Cin, 40), rng.integers(0, KH, 40), rng.integers(0, KW, 40)], 1)
    got = R.conv2d_dw_q_entries(xq, geom, G, a, b, dy, idx)
    assert np.array_equal(got, dW[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]])


def test_bad_geometry_is_refused():
    geom, _, _ = R.conv_geometry(1, 4, 3, 3, 1, 5, 5)          # kernel larger than the unpadded image
    rc = R.lib().mesa_ref_conv2d_dw_q(None, geom.ctypes.data_as(R.C.c_void_p), R.I64(2), None, None, None, 0, None, None)
    assert rc == 1
