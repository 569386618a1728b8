"""mesa_conv2d_dw_q against the oracle: the matrix-core path over ragged channel tiles, several row segments, kernel
shapes 3x3 and 1x1, row strides, dilations and paddings, widths that are and are not multiples of eight; the plain path over everything else (column strides and
dilations, other kernel shapes and column paddings, binary32 tensors); the empty batch and the error paths."""
import numpy as np
import pytest
import torch

from oracle import mesa_ref as R

pytestmark = pytest.mark.gpu

TOL = {torch.float32: 1e-5, torch.float16: 2e-3, torch.bfloat16: 2e-3}   # bfloat16 dy: products exact, sums binary32, like binary16


@pytest.fixture(scope="module")
def M():
    import paper_2111_11124_amd as m
    assert torch.cuda.is_available(), "these tests need the MI355X"
    m.lib()
    return m


def npy(t):
    return (t.float() if t.dtype == torch.bfloat16 else t).cpu().numpy()


def relerr(got, ref):
    return float(np.abs(np.asarray(got, np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def run_case(M, case, dtype, seed=0, dy_mean=0.0):
    B, Cin, H, W, Cout, KH, KW, stride, pad, dil, G = case
    cv = M.Conv2d(B, Cin, H, W, Cout, KH, KW, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1])
    OH, OW = cv.out_hw()
    gen = torch.Generator(device="cuda").manual_seed(seed + B * 1000 + Cin + 7 * Cout + H)
    xq = torch.randint(-128, 128, (B, Cin, H, W), dtype=torch.int8, device="cuda", generator=gen)
    dy = (torch.randn((B, Cout, OH, OW), device="cuda", generator=gen) + dy_mean).to(dtype)
    a = (0.5 + 4.0 * torch.rand(G, device="cuda", generator=gen)).float()
    b = (-2.5 + 2.0 * torch.rand(G, device="cuda", generator=gen)).float()
    dW = torch.full((Cout, Cin, KH, KW), float("nan"), device="cuda")
    db = torch.full((Cout,), float("nan"), device="cuda")
    dtc = {torch.float16: M.F16, torch.bfloat16: M.BF16, torch.float32: M.F32}[dtype]
    nws = M.conv2d_dw_q_workspace_bytes(cv, dtc)
    ws = torch.empty(max(nws, 16), dtype=torch.uint8, device="cuda")
    M.mesa_conv2d_dw_q(xq, cv, G, a, b, dy, dW, db, ws)
    torch.cuda.synchronize()
    geom, rOH, rOW = R.conv_geometry(B, Cin, H, W, Cout, KH, KW, stride, pad, dil)
    assert (rOH, rOW) == (OH, OW)
    dyr = npy(dy) if dtype != torch.bfloat16 else npy(dy).astype(np.float32)
    rW, rb = R.conv2d_dw_q(npy(xq), geom, G, npy(a), npy(b), dyr)
    return relerr(npy(dW), rW), relerr(npy(db), rb), nws


# B, Cin, H, W, Cout, KH, KW, stride, pad, dil, G   -- all on the matrix-core path for 16-bit tensors
FAST = [
    (2, 96, 16, 24, 80, 3, 3, (1, 1), (1, 1), (1, 1), 3),        # ragged channel tiles, a row narrower than a stage
    (1, 64, 5, 264, 64, 3, 3, (1, 1), (1, 1), (1, 1), 2),        # three row segments, the last eight columns wide
    (3, 40, 17, 16, 24, 3, 3, (2, 1), (1, 1), (1, 1), 5),        # row stride 2
    (2, 32, 12, 32, 72, 3, 3, (1, 1), (2, 1), (2, 1), 1),        # row dilation 2
    (2, 64, 9, 40, 64, 3, 3, (1, 1), (0, 1), (1, 1), 4),         # no row padding; four contraction steps per stage
    (2, 64, 6, 72, 64, 3, 3, (1, 1), (1, 1), (1, 1), 4),         # eight steps per stage, the row ends half way through one
    (4, 200, 8, 16, 136, 1, 1, (1, 1), (0, 0), (1, 1), 4),       # 1x1: ragged 128-channel tiles
    (2, 128, 6, 136, 128, 1, 1, (2, 1), (0, 0), (1, 1), 2),      # 1x1: two segments, row stride
    (2, 256, 12, 48, 128, 1, 1, (1, 1), (3, 0), (1, 1), 2),      # 1x1 with row padding (rows of dy that meet no input row)
    (16, 64, 32, 32, 64, 3, 3, (1, 1), (1, 1), (1, 1), 4),       # many stages: several slices of the (image, row) range
    (2, 3, 6, 512, 72, 3, 3, (1, 1), (1, 1), (1, 1), 1),         # rows of 256 columns and more next to a ragged tile of output channels
    (1, 136, 3, 264, 40, 1, 1, (1, 1), (0, 0), (1, 1), 1),       # the same for 1x1
    # widths that are no multiples of eight: unaligned rows, a row's last vector loaded early and placed element by element
    (3, 40, 28, 28, 136, 3, 3, (1, 1), (1, 1), (1, 1), 2),       # 28 x 28 maps
    (4, 72, 14, 14, 72, 3, 3, (1, 1), (1, 1), (1, 1), 3),        # 14 x 14
    (2, 24, 5, 9, 10, 3, 3, (1, 1), (1, 1), (1, 1), 1),          # one column more than a vector; the tensors' last rows end the buffers
    (1, 8, 3, 8, 4, 3, 3, (1, 1), (1, 1), (1, 1), 1),            # the narrowest width this path takes
    (2, 64, 4, 135, 64, 3, 3, (2, 1), (1, 1), (1, 1), 4),        # two segments, seven columns in the second
    (2, 64, 5, 129, 40, 3, 3, (1, 1), (1, 1), (1, 1), 1),        # one column in the second segment
    (2, 130, 6, 63, 70, 3, 3, (1, 1), (0, 1), (2, 1), 5),        # four steps per stage, the last column missing
    (2, 200, 14, 14, 136, 1, 1, (1, 1), (0, 0), (1, 1), 4),      # 1x1 on 14 x 14
    (2, 128, 4, 257, 128, 1, 1, (1, 1), (1, 0), (1, 1), 2),      # 1x1: three segments, one column in the last
    (3, 16, 7, 100, 24, 1, 1, (2, 1), (0, 0), (1, 1), 2),        # 1x1: rows that start at every alignment
    # maps of at most 16 columns: stages of one contraction step
    (4, 72, 16, 16, 136, 3, 3, (1, 1), (1, 1), (1, 1), 3),
    (5, 130, 8, 8, 70, 3, 3, (1, 1), (1, 1), (1, 1), 2),
    (3, 64, 9, 13, 64, 3, 3, (2, 1), (2, 1), (2, 1), 4),
    (3, 136, 11, 11, 200, 1, 1, (1, 1), (0, 0), (1, 1), 1),
    # maps narrower than eight columns: read from copies with rows of eight
    (4, 72, 7, 7, 136, 3, 3, (1, 1), (1, 1), (1, 1), 3),
    (3, 130, 7, 7, 70, 1, 1, (1, 1), (0, 0), (1, 1), 2),
    (2, 24, 5, 4, 10, 3, 3, (1, 1), (1, 1), (1, 1), 1),
    (2, 8, 3, 1, 4, 3, 3, (1, 1), (1, 1), (1, 1), 1),
    (2, 8, 9, 7, 5, 3, 3, (2, 1), (1, 1), (1, 1), 2),
    (5, 64, 4, 6, 64, 3, 3, (1, 1), (2, 1), (2, 1), 4),
]


@pytest.mark.parametrize("case", FAST, ids=[f"c{i}" for i in range(len(FAST))])
@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16], ids=["f16", "bf16"])
def test_conv_dw_matrix_core_path(M, case, dtype):
    eW, eb, nws = run_case(M, case, dtype)
    assert nws > 0, "expected the matrix-core path (it is the one that needs a workspace)"
    assert eW <= TOL[dtype] and eb <= 1e-5, (eW, eb)


PLAIN = [
    (2, 6, 9, 8, 4, 3, 2, (2, 1), (0, 1), (1, 1), 3),            # even kernel width
    (1, 4, 11, 10, 2, 3, 3, (1, 2), (2, 2), (2, 2), 1),          # column stride and dilation
    (2, 3, 8, 8, 2, 4, 4, (4, 4), (0, 0), (1, 1), 3),            # patch embedding: stride = kernel
    (1, 8, 14, 14, 6, 5, 5, (1, 1), (2, 2), (1, 1), 2),          # 5x5
    (2, 8, 9, 7, 5, 5, 5, (1, 1), (2, 2), (1, 1), 2),            # 5x5 on a map narrower than a vector
    (2, 48, 8, 16, 40, 3, 1, (1, 1), (1, 0), (1, 1), 3),         # 3x1 kernel
    (2, 48, 8, 16, 40, 1, 3, (1, 1), (0, 1), (1, 1), 3),         # 1x3 kernel
    (2, 16, 8, 24, 16, 3, 3, (1, 1), (1, 5), (1, 1), 2),         # 3x3 with wide column padding
    (2, 32, 6, 16, 32, 1, 1, (1, 1), (0, 4), (1, 1), 2),         # 1x1 with column padding
]


@pytest.mark.parametrize("case", PLAIN, ids=[f"p{i}" for i in range(len(PLAIN))])
@pytest.mark.parametrize("dtype", [torch.float32, torch.float16, torch.bfloat16], ids=["f32", "f16", "bf16"])
def test_conv_dw_plain_path(M, case, dtype):
    eW, eb, nws = run_case(M, case, dtype)
    assert nws == 0
    assert eW <= 1e-6 and eb <= 1e-6, (eW, eb)


@pytest.mark.parametrize("case", [FAST[0], FAST[1], FAST[10], FAST[12], FAST[14], FAST[16], FAST[17], FAST[20], FAST[21], FAST[24], FAST[26], FAST[27],
                                  FAST[29]],
                         ids=lambda c: "x".join(str(v) for v in c[:7]))
def test_conv_dw_reads_nothing_it_uses_from_outside_the_tensors(M, case):
    """Both inputs are the middle of larger buffers whose frames hold NaN (dy) and the extreme code (x): a vector that
    reaches over a tensor's end, or a masked load whose value were multiplied instead of discarded, would show in dW."""
    B, Cin, H, W, Cout, KH, KW, stride, pad, dil, G = case
    cv = M.Conv2d(B, Cin, H, W, Cout, KH, KW, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1])
    OH, OW = cv.out_hw()
    gen = torch.Generator(device="cuda").manual_seed(77 + Cin + Cout)
    nx, nd, fr = B * Cin * H * W, B * Cout * OH * OW, 256
    bx = torch.full((nx + 2 * fr,), 127, dtype=torch.int8, device="cuda")
    bd = torch.full((nd + 2 * fr,), float("nan"), dtype=torch.float16, device="cuda")
    xq = bx[fr:fr + nx].view(B, Cin, H, W)
    dy = bd[fr:fr + nd].view(B, Cout, OH, OW)
    xq.copy_(torch.randint(-128, 128, (B, Cin, H, W), dtype=torch.int8, device="cuda", generator=gen))
    dy.copy_(torch.randn((B, Cout, OH, OW), device="cuda", generator=gen).half())
    a = (0.5 + 4.0 * torch.rand(G, device="cuda", generator=gen)).float()
    b = (-2.5 + 2.0 * torch.rand(G, device="cuda", generator=gen)).float()
    dW = torch.full((Cout, Cin, KH, KW), float("nan"), device="cuda")
    db = torch.full((Cout,), float("nan"), device="cuda")
    nws = M.conv2d_dw_q_workspace_bytes(cv, M.F16)
    assert nws > 0
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    M.mesa_conv2d_dw_q(xq, cv, G, a, b, dy, dW, db, ws)
    torch.cuda.synchronize()
    geom, _, _ = R.conv_geometry(B, Cin, H, W, Cout, KH, KW, stride, pad, dil)
    rW, rb = R.conv2d_dw_q(npy(xq), geom, G, npy(a), npy(b), npy(dy))
    assert relerr(npy(dW), rW) <= 2e-3 and relerr(npy(db), rb) <= 1e-5


def test_conv_dw_binary32_tensors_take_the_plain_path(M):
    eW, eb, nws = run_case(M, FAST[0], torch.float32)
    assert nws == 0 and eW <= 1e-6 and eb <= 1e-6, (eW, eb, nws)


def test_conv_dw_upstream_gradient_with_a_mean(M):
    """binary16: the contracted operand is 1024 + x_bar, taken out again with the sums of dy over the in-image
    positions -- a mean in dy is the worst case for that cancellation (as for the Linear weight gradient)."""
    eW, eb, _ = run_case(M, (8, 64, 32, 32, 64, 3, 3, (1, 1), (1, 1), (1, 1), 4), torch.float16, dy_mean=0.5)
    assert eW <= 5e-4 and eb <= 1e-5, (eW, eb)


def test_conv_dw_empty_batch_and_errors(M):
    cv = M.Conv2d(0, 8, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 1)
    a = torch.ones(2, device="cuda")
    b = torch.zeros(2, device="cuda")
    dW = torch.full((4, 8, 3, 3), 5.0, device="cuda")
    db = torch.full((4,), 5.0, device="cuda")
    M.mesa_conv2d_dw_q(None, cv, 2, a, b, torch.empty(0, dtype=torch.half, device="cuda"), dW, db, None)
    torch.cuda.synchronize()
    assert float(dW.abs().max()) == 0.0 and float(db.abs().max()) == 0.0
    xq = torch.zeros((1, 8, 8, 8), dtype=torch.int8, device="cuda")
    dy = torch.zeros((1, 4, 8, 8), dtype=torch.half, device="cuda")
    cases = [
        (M.Conv2d(1, 8, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 1), 3, M.ERR_INVALID_ARG),      # C_in % G != 0
        (M.Conv2d(1, 8, 8, 8, 4, 11, 3, 1, 1, 1, 1, 1, 1), 2, M.ERR_INVALID_ARG),     # kernel taller than the padded image
        (M.Conv2d(1, 8, 8, 8, 4, 3, 3, 0, 1, 1, 1, 1, 1), 2, M.ERR_INVALID_ARG),      # zero stride
    ]
    for cv, G, status in cases:
        with pytest.raises(M.MesaError) as e:
            M.mesa_conv2d_dw_q(xq, cv, G, a[:1].expand(G).contiguous(), b[:1].expand(G).contiguous(), dy, dW, db, None)
        assert e.value.status == status
    good = M.Conv2d(1, 8, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 1)
    with pytest.raises(M.MesaError) as e:          # the matrix-core path without its workspace
        M.mesa_conv2d_dw_q(xq, good, 2, a, b, dy, dW, db, None)
    assert e.value.status == M.ERR_WORKSPACE
