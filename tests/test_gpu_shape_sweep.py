"""Seeded sweeps over extents around every kernel's size limits, outputs framed by guard zones.

Each case runs the HIP path on a buffer that carries 32 sentinel elements before and after the output, compares the
output with the oracle as the parity tests do, and checks that the sentinels are untouched: a kernel that writes a
partial vector or a ragged tile past its extent shows up here even when the values it owes are right.
"""
import random

import numpy as np
import pytest
import torch

from oracle import mesa_ref as R

pytestmark = pytest.mark.gpu
TOL = {torch.float32: 1e-5, torch.float16: 2e-3, torch.bfloat16: 1.6e-2}
GUARD = 32


@pytest.fixture(scope="module")
def M():
    import paper_2111_11124_amd as m
    assert torch.cuda.is_available()
    m.lib()
    return m


def npy(t):
    return (t.float() if t.dtype == torch.bfloat16 else t).cpu().numpy()


def relerr(got, ref):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def framed(shape, dtype, val=7):
    """(frame, view): a buffer of sentinels with the output in its middle (the view starts 16-byte aligned)."""
    n = int(np.prod(shape))
    frame = torch.full((n + 2 * GUARD,), val, dtype=dtype, device="cuda")
    return frame, frame[GUARD:GUARD + n].view(shape)


def intact(frame, val=7):
    return bool((frame[:GUARD] == val).all() and (frame[-GUARD:] == val).all())


ATTN_N = (8, 9, 15, 16, 17, 31, 32, 33, 48, 63, 64, 65, 96, 127, 128, 129, 160, 191, 192, 193, 197, 222, 223, 224, 225, 254, 255,
          256, 257)


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16], ids=["f16", "bf16"])
@pytest.mark.parametrize("Dh", [32, 64, 96, 128, 8, 40])
def test_attention_products_around_every_size_limit(M, Dh, dtype):
    """Sequence lengths on both sides of each dedicated kernel's limits (chunk sizes, LDS capacity, the general
    kernel's tiles) for the head sizes with dedicated kernels and two without."""
    rnd = random.Random(Dh)
    for idx, N in enumerate(ATTN_N):
        B, H = rnd.choice((1, 2, 3)), rnd.choice((1, 2, 3, 5))
        g = torch.Generator(device="cuda").manual_seed(1000 * Dh + idx)
        aq = torch.randint(-128, 128, (B, H, N, N), dtype=torch.int8, device="cuda", generator=g)
        qq, kq, vq = (torch.randint(-128, 128, (B, H, N, Dh), dtype=torch.int8, device="cuda", generator=g) for _ in range(3))
        dO = torch.randn((B, H, N, Dh), device="cuda", generator=g).to(dtype)
        dS = (torch.randn((B, H, N, N), device="cuda", generator=g) * 0.1).to(dtype)
        par = {k: (torch.linspace(1.0, 4.0, H, device="cuda") * s, torch.linspace(-2.0, -0.5, H, device="cuda") * s)
               for k, s in (("a", 0.25), ("q", 1.0), ("k", 1.5), ("v", 0.75))}
        fA, dA = framed((B, H, N, N), dtype)
        fV, dV = framed((B, H, N, Dh), dtype)
        fQ, dQ = framed((B, H, N, Dh), dtype)
        fK, dK = framed((B, H, N, Dh), dtype)
        M.mesa_attn_av_bwd_q(aq, vq, B, H, N, Dh, *par["a"], *par["v"], dO, dA, dV)
        M.mesa_attn_qk_bwd_q(qq, kq, B, H, N, Dh, *par["q"], *par["k"], dS, 0.2, dQ, dK)
        rp = {k: (npy(a), npy(b)) for k, (a, b) in par.items()}
        rdA, rdV = R.attn_av_bwd_q(npy(aq), npy(vq), B, H, N, Dh, *rp["a"], *rp["v"], npy(dO))
        rdQ, rdK = R.attn_qk_bwd_q(npy(qq), npy(kq), B, H, N, Dh, *rp["q"], *rp["k"], npy(dS), 0.2)
        errs = {"dA": relerr(npy(dA), rdA), "dV": relerr(npy(dV), rdV), "dQ": relerr(npy(dQ), rdQ), "dK": relerr(npy(dK), rdK)}
        assert all(v <= TOL[dtype] for v in errs.values()), ((B, H, N, Dh), errs)
        assert all(intact(f) for f in (fA, fV, fQ, fK)), (B, H, N, Dh)


SOFTMAX_COLS = (1, 2, 3, 5, 7, 8, 9, 16, 17, 31, 33, 49, 56, 57, 64, 100, 104, 105, 127, 128, 197, 199, 200, 201, 255, 256, 257, 264,
                511, 577, 1000, 1024)


@pytest.mark.parametrize("dtype", [torch.float16, torch.float32, torch.bfloat16], ids=["f16", "f32", "bf16"])
def test_softmax_layer_forward_and_backward_over_row_lengths(M, dtype):
    """Row lengths on both sides of every lane-group shape of the short-row kernels and into the long-row kernels;
    row counts that leave ragged tiles and tiles that straddle heads."""
    rnd = random.Random(str(dtype))
    for cols in SOFTMAX_COLS:
        B, H, rows = rnd.choice((1, 2, 7)), rnd.choice((1, 3, 4)), rnd.choice((1, 5, 17, 61, cols))
        n = B * H * rows * cols
        lay = (B, H, rows * cols)
        g = torch.Generator(device="cuda").manual_seed(cols)
        s = (torch.randn((B, H, rows, cols), device="cuda", generator=g) * 2).to(dtype)
        fy, y = framed((B, H, rows, cols), dtype)
        fq, q = framed((n,), torch.int8)
        a = torch.full((H,), 0.9, device="cuda")
        b = torch.full((H,), 0.01, device="cuda")
        ra, rb = npy(a).copy(), npy(b).copy()
        ws = torch.empty(max(M.workspace_bytes(M.OP_SOFTMAX_FWD_Q, B * H * rows, H, cols, M.F16), 16), dtype=torch.uint8, device="cuda")
        mode, rmode = rnd.choice(((M.ROUND_STOCHASTIC, R.ROUND_STOCHASTIC), (M.ROUND_NEAREST_EVEN, R.ROUND_NEAREST)))
        M.mesa_softmax_fwd_q(s, B, H, rows, cols, a, b, 0.9, y, q, ws, mode, 3, 1)
        yh = npy(y)
        assert relerr(yh, R.softmax_fwd(npy(s), B * H * rows, cols)) <= TOL[dtype], (B, H, rows, cols)
        rq, ra2, rb2 = R.quantize_update_fused(yh, lay, ra, rb, 0.9, rmode, 3, 1)
        assert np.array_equal(npy(q), rq.reshape(-1)), (B, H, rows, cols)
        assert np.array_equal(npy(a), ra2) and np.array_equal(npy(b), rb2), (B, H, rows, cols)
        assert intact(fy) and intact(fq), (B, H, rows, cols)
        # backward at the codes just taken, with the moved estimates
        dy = torch.randn((B, H, rows, cols), device="cuda", generator=g).to(dtype)
        fx, dx = framed((B, H, rows, cols), dtype)
        M.mesa_softmax_bwd_q(q, B, H, rows, cols, a, b, dy, dx)
        ref = R.softmax_bwd_q(npy(q), B, H, rows, cols, ra2, rb2, npy(dy))
        assert relerr(npy(dx).reshape(ref.shape), ref) <= TOL[dtype], (B, H, rows, cols)
        assert intact(fx), (B, H, rows, cols)


@pytest.mark.parametrize("dtype", [torch.float16, torch.float32, torch.bfloat16], ids=["f16", "f32", "bf16"])
def test_layernorm_and_gelu_layer_forwards_over_extents(M, dtype):
    rnd = random.Random("ln" + str(dtype))
    for D in (8, 16, 24, 64, 96, 128, 192, 384, 512, 520, 768, 1000, 1024, 1032, 1536, 2048):
        Mr = rnd.choice((1, 3, 31, 100, 257))
        G = rnd.choice([gg for gg in (1, 2, 3, 4, 6, 8, 12) if D % gg == 0 and (D // gg) % 8 == 0])
        g = torch.Generator(device="cuda").manual_seed(D)
        x = (torch.randn((Mr, D), device="cuda", generator=g) * 1.5 + 0.2).to(dtype)
        gamma = (1 + 0.1 * torch.randn(D, device="cuda", generator=g)).to(dtype)
        bias = (0.1 * torch.randn(D, device="cuda", generator=g)).to(dtype)
        fy, y = framed((Mr, D), dtype)
        fq, q = framed((Mr * D,), torch.int8)
        fm, mean = framed((Mr,), torch.float32)
        fr, rstd = framed((Mr,), torch.float32)
        a = torch.full((G,), 9.0, device="cuda")
        b = torch.full((G,), -4.5, device="cuda")
        ra, rb = npy(a).copy(), npy(b).copy()
        ws = torch.empty(max(M.workspace_bytes(M.OP_LAYERNORM_FWD_Q, Mr, D, G, M.F16), 16), dtype=torch.uint8, device="cuda")
        M.mesa_layernorm_fwd_q(x, Mr, D, G, gamma, bias, 1e-5, a, b, 0.9, y, mean, rstd, q, ws, M.ROUND_STOCHASTIC, 3, 1)
        ry, rm, rr = R.layernorm_fwd(npy(x), Mr, D, npy(gamma), npy(bias), 1e-5)
        rq, ra2, rb2 = R.quantize_update_fused(npy(x), (Mr, G, D // G), ra, rb, 0.9, R.ROUND_STOCHASTIC, 3, 1)
        assert relerr(npy(y), ry) <= TOL[dtype] and relerr(npy(mean), rm) <= 1e-5 and relerr(npy(rstd), rr) <= 1e-5, (Mr, D, G)
        assert np.array_equal(npy(q), rq.reshape(-1)) and np.array_equal(npy(a), ra2) and np.array_equal(npy(b), rb2), (Mr, D, G)
        assert all(intact(f) for f in (fy, fm, fr, fq)), (Mr, D, G)
    for lay in ((1, 1, 8), (1, 1, 9), (3, 2, 5), (7, 3, 333), (2, 40, 77), (5, 6, 256), (1, 1, 100003), (9, 12, 64)):
        G = lay[1]
        g = torch.Generator(device="cuda").manual_seed(lay[2])
        x = (torch.randn(lay, device="cuda", generator=g) * 2).to(dtype)
        fy, y = framed(lay, dtype)
        fq, q = framed((x.numel(),), torch.int8)
        a = torch.full((G,), 7.0, device="cuda")
        b = torch.full((G,), -3.5, device="cuda")
        ra, rb = npy(a).copy(), npy(b).copy()
        ws = torch.empty(max(M.workspace_bytes(M.OP_UPDATE_RUNNING_PARAMS, *lay, M.F16), 16), dtype=torch.uint8, device="cuda")
        M.mesa_gelu_fwd_q(x, lay, a, b, 0.9, y, q, ws, M.ROUND_STOCHASTIC, 3, 1)
        ry, rq, ra2, rb2 = R.gelu_fwd_q(npy(x), lay, ra, rb, 0.9, R.ROUND_STOCHASTIC, 3, 1)
        assert relerr(npy(y), ry) <= TOL[dtype], lay
        assert np.array_equal(npy(q), rq.reshape(-1)) and np.array_equal(npy(a), ra2) and np.array_equal(npy(b), rb2), lay
        assert intact(fy) and intact(fq), lay


@pytest.mark.parametrize("dtype", [torch.float16, torch.float32, torch.bfloat16], ids=["f16", "f32", "bf16"])
def test_stream_kernels_and_layernorm_backward_keep_inside_their_outputs(M, dtype):
    """Quantize, single-pass quantize, de-quantize, GELU / ReLU / LayerNorm backward on ragged layouts: results as
    in the parity tests, and nothing written outside the outputs."""
    rnd = random.Random("core" + str(dtype))
    layouts = [(1, 1, 1), (1, 1, 7), (1, 1, 8), (1, 1, 4097), (3, 2, 5), (7, 3, 333), (2, 40, 77), (5, 6, 256), (1, 1, 100003), (9, 12, 64),
               (37, 6, 64), (4, 3, 361), (1, 5, 2049), (129, 1, 24)]
    for lay in layouts:
        n = lay[0] * lay[1] * lay[2]
        G = lay[1]
        g = torch.Generator(device="cuda").manual_seed(n)
        x = (torch.randn(lay, device="cuda", generator=g) * 1.7 + 0.1).to(dtype)
        a = torch.zeros(G, device="cuda")
        b = torch.zeros(G, device="cuda")
        ws = torch.empty(max(M.workspace_bytes(M.OP_UPDATE_RUNNING_PARAMS, *lay, M.F16), 16), dtype=torch.uint8, device="cuda")
        M.mesa_update_running_params(x, lay, a, b, 0.9, True, ws)
        ra, rb = R.update_running_params(npy(x), lay, np.zeros(G, np.float32), np.zeros(G, np.float32), 0.9, True)
        mode, rmode = rnd.choice(((M.ROUND_STOCHASTIC, R.ROUND_STOCHASTIC), (M.ROUND_NEAREST_EVEN, R.ROUND_NEAREST)))
        fq, q = framed((n,), torch.int8)
        M.mesa_quantize_headwise(x, lay, a, b, q, mode, 9, 5)
        rq = R.quantize_headwise(npy(x), lay, ra, rb, rmode, 9, 5).reshape(-1)
        assert np.array_equal(npy(q), rq) and intact(fq), lay
        fq2, q2 = framed((n,), torch.int8)
        a2, b2 = a.clone(), b.clone()
        M.mesa_quantize_update_fused(x, lay, a2, b2, 0.9, q2, ws, mode, 9, 5)
        assert torch.equal(q2, q) and intact(fq2), lay
        fo, out = framed((n,), dtype)
        M.mesa_dequantize(q, lay, a, b, out)
        ref = R.dequantize(rq, lay, ra, rb, np.float32)
        assert relerr(npy(out), ref) <= TOL[dtype] and intact(fo), lay
        dy = torch.randn(lay, device="cuda", generator=g).to(dtype)
        for call, oracle in ((M.mesa_gelu_bwd_q, R.gelu_bwd_q), (M.mesa_relu_bwd_q, R.relu_bwd_q)):
            fx, dx = framed(lay, dtype)
            call(q, lay, a, b, dy, dx)
            ref = oracle(rq, lay, ra, rb, npy(dy))
            assert relerr(npy(dx).reshape(ref.shape), ref) <= TOL[dtype] and intact(fx), (lay, call.__name__)
    for Mr, D, G in ((1, 8, 1), (37, 48, 3), (333, 128, 4), (130, 512, 8), (259, 1024, 16), (77, 1032, 3), (19, 4096, 8), (5, 2056, 1)):
        g = torch.Generator(device="cuda").manual_seed(Mr * D)
        lay = (Mr, G, D // G)
        x = (torch.randn((Mr, D), device="cuda", generator=g) * 1.3 + 0.3).to(dtype)
        a = torch.zeros(G, device="cuda")
        b = torch.zeros(G, device="cuda")
        ws = torch.empty(max(M.workspace_bytes(M.OP_UPDATE_RUNNING_PARAMS, *lay, M.F16), 16), dtype=torch.uint8, device="cuda")
        M.mesa_update_running_params(x, lay, a, b, 0.9, True, ws)
        q = torch.empty(Mr * D, dtype=torch.int8, device="cuda")
        M.mesa_quantize_headwise(x, lay, a, b, q, M.ROUND_STOCHASTIC, 2, 0)
        xf = x.float()
        mean = xf.mean(-1).contiguous()
        rstd = (1.0 / torch.sqrt(xf.var(-1, unbiased=False) + 1e-5)).contiguous()
        gamma = (1 + 0.1 * torch.randn(D, device="cuda", generator=g)).to(dtype)
        dy = torch.randn((Mr, D), device="cuda", generator=g).to(dtype)
        fx, dx = framed((Mr, D), dtype)
        fg, dg = framed((D,), torch.float32)
        fb, db = framed((D,), torch.float32)
        w2 = torch.empty(max(M.workspace_bytes(M.OP_LAYERNORM_BWD_Q, Mr, D, G, M.F16), 16), dtype=torch.uint8, device="cuda")
        M.mesa_layernorm_bwd_q(q, Mr, D, G, a, b, mean, rstd, gamma, dy, dx, dg, db, w2)
        rdx, rdg, rdb = R.layernorm_bwd_q(npy(q), Mr, D, G, npy(a), npy(b), npy(mean), npy(rstd), npy(gamma), npy(dy))
        assert relerr(npy(dx), rdx) <= TOL[dtype] and relerr(npy(dg), rdg) <= TOL[dtype] and relerr(npy(db), rdb) <= TOL[dtype], (Mr, D, G)
        assert intact(fx) and intact(fg) and intact(fb), (Mr, D, G)


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16, torch.float32], ids=["f16", "bf16", "f32"])
def test_linear_dw_keeps_inside_its_outputs(M, dtype):
    """dW and db framed by sentinels, over every tile variant (256 x 256, 256 x 128, 128 x 128, the binary32 path)
    with partial tiles in both extents and ragged slices of m."""
    for Mr, K, N in ((31, 16, 8), (97, 128, 264), (3205, 256, 520), (909, 784, 136), (9000, 272, 1000), (5000, 96, 384), (777, 1280, 72),
                     (100, 40, 64), (333, 17, 5), (1000, 100, 12), (65, 3, 1), (700, 48, 20)):
        H = 1 if K % 3 else 3
        lay = (Mr, H, K // H)
        g = torch.Generator(device="cuda").manual_seed(Mr + K)
        q = torch.randint(-128, 128, (Mr * K,), dtype=torch.int8, device="cuda", generator=g)
        a = torch.linspace(1.0, 3.0, H, device="cuda")
        b = torch.linspace(-1.5, -0.5, H, device="cuda")
        dy = torch.randn((Mr, N), device="cuda", generator=g).to(dtype)
        fW, dW = framed((N, K), torch.float32)
        fb, db = framed((N,), torch.float32)
        dtc = {torch.float16: M.F16, torch.bfloat16: M.BF16, torch.float32: M.F32}[dtype]
        ws = torch.empty(max(M.workspace_bytes(M.OP_LINEAR_DW_Q, Mr, K, N, dtc), 16), dtype=torch.uint8, device="cuda")
        M.mesa_linear_dw_q(q, Mr, K, H, a, b, dy, N, dW, db, ws)
        rW, rb_ = R.linear_dw_q(npy(q), Mr, K, H, npy(a), npy(b), npy(dy), N)
        assert relerr(npy(dW), rW) <= 2e-3 and relerr(npy(db), rb_) <= 2e-3, (Mr, K, N)
        assert intact(fW) and intact(fb), (Mr, K, N)


def _conv_cases(seed, count):
    """Seeded convolution geometries that take the matrix-core path: 3x3 with one column of padding or 1x1 with none,
    unit column stride and dilation, any width (a third of them no multiples of 8, some below 8); everything else drawn freely (ragged channel
    tiles, one to three row segments, row strides, dilations and paddings, batch sizes that leave ragged slices)."""
    rnd = random.Random(seed)
    out = []
    while len(out) < count:
        k = rnd.choice((3, 3, 1))
        B = rnd.randint(1, 5)
        G = rnd.choice((1, 2, 3, 4, 6))
        Cin = G * rnd.randint(2, 40)
        Cout = rnd.randint(3, 150)
        W = 8 * rnd.choice((1, 2, 3, 4, 5, 8, 9, 16, 17, 33)) + rnd.choice((0, 0, rnd.randint(1, 7)))
        if rnd.random() < 0.15:
            W = rnd.randint(1, 7)
        sh, dh, ph = rnd.choice((1, 1, 2, 3)), rnd.choice((1, 1, 2, 3)), rnd.randint(0, 3)
        H = rnd.randint(max(1, dh * (k - 1) + 1 - 2 * ph), 22)
        if B * Cin * Cout * H * W > 3.0e8:           # keeps the oracle's binary64 loops to a second or two
            continue
        out.append((B, Cin, H, W, Cout, k, k, (sh, 1), (ph, 1 if k == 3 else 0), (dh, 1), G))
    return out


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16], ids=["f16", "bf16"])
@pytest.mark.parametrize("seed", [1, 2, 3])
def test_convolution_weight_gradient_over_seeded_geometries(M, seed, dtype):
    """dW and db framed by sentinels, against the oracle, over ten geometries per seed; every case must take the
    matrix-core path (a workspace is asked for)."""
    for case in _conv_cases(seed, 10):
        B, Cin, H, W, Cout, KH, KW, stride, pad, dil, G = case
        cv = M.Conv2d(B, Cin, H, W, Cout, KH, KW, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1])
        OH, OW = cv.out_hw()
        gen = torch.Generator(device="cuda").manual_seed(seed * 1000 + Cin + Cout)
        xq = torch.randint(-128, 128, (B, Cin, H, W), dtype=torch.int8, device="cuda", generator=gen)
        dy = torch.randn((B, Cout, OH, OW), device="cuda", generator=gen).to(dtype)
        a = (0.5 + 4.0 * torch.rand(G, device="cuda", generator=gen)).float()
        b = (-2.5 + 2.0 * torch.rand(G, device="cuda", generator=gen)).float()
        fW, dW = framed((Cout, Cin, KH, KW), torch.float32)
        fb, db = framed((Cout,), torch.float32)
        dtc = M.F16 if dtype == torch.float16 else M.BF16
        nws = M.conv2d_dw_q_workspace_bytes(cv, dtc)
        assert nws > 0, case
        fws = torch.full((nws + 512,), 0x5A, dtype=torch.uint8, device="cuda")
        ws = fws[256:256 + nws]
        M.mesa_conv2d_dw_q(xq, cv, G, a, b, dy, dW, db, ws)
        torch.cuda.synchronize()
        geom, rOH, rOW = R.conv_geometry(B, Cin, H, W, Cout, KH, KW, stride, pad, dil)
        assert (rOH, rOW) == (OH, OW)
        rW, rb = R.conv2d_dw_q(npy(xq), geom, G, npy(a), npy(b), npy(dy).astype(np.float32))
        assert relerr(npy(dW), rW) <= 2e-3 and relerr(npy(db), rb) <= 1e-5, (case, relerr(npy(dW), rW), relerr(npy(db), rb))
        assert intact(fW) and intact(fb), case
        assert bool((fws[:256] == 0x5A).all() and (fws[256 + nws:] == 0x5A).all()), case


def _mid(t, fill):
    """A copy of t in the middle of a larger buffer whose 256 elements on either side hold `fill`."""
    buf = torch.full((t.numel() + 512,), fill, dtype=t.dtype, device=t.device)
    view = buf[256:256 + t.numel()].view(t.shape)
    view.copy_(t)
    return view


def canon(a):
    return (np.asarray(a, np.float32) + np.float32(0.0)).view(np.uint32)


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16, torch.float32], ids=["f16", "bf16", "f32"])
@pytest.mark.parametrize("layout", [(3, 5, 1001), (7, 3, 197 * 197), (1, 12, 8 * 333 + 5), (50, 6, 64), (1, 2, 4099), (2, 3000, 13)])
def test_streaming_calls_use_nothing_from_outside_their_inputs(M, layout, dtype):
    """x lies between values far outside its range, the codes between extreme codes, the gradient between NaN: the
    extrema (hence alpha, beta), the codes and the gradients are the oracle's all the same -- ragged ends, prefetches and
    masked lanes take nothing from beyond a tensor's last element."""
    outer, G, inner = layout
    n = outer * G * inner
    gen = torch.Generator(device="cuda").manual_seed(n % 9973)
    big = 60000.0 if dtype == torch.float16 else 1.0e30
    x = _mid((torch.randn(n, device="cuda", generator=gen) * 1.5 + 0.2).to(dtype), big)
    a = torch.zeros(G, device="cuda")
    b = torch.zeros(G, device="cuda")
    dtc = {torch.float16: M.F16, torch.bfloat16: M.BF16, torch.float32: M.F32}[dtype]
    ws = torch.empty(max(M.workspace_bytes(M.OP_UPDATE_RUNNING_PARAMS, outer, G, inner, dtc), 16), dtype=torch.uint8, device="cuda")
    M.mesa_update_running_params(x, layout, a, b, 0.9, True, ws)
    ra, rb = R.update_running_params(npy(x), layout, np.zeros(G, np.float32), np.zeros(G, np.float32), 0.9, True)
    assert np.array_equal(canon(npy(a)), canon(ra)) and np.array_equal(canon(npy(b)), canon(rb))
    q = torch.empty(n, dtype=torch.int8, device="cuda")
    M.mesa_quantize_headwise(x, layout, a, b, q, M.ROUND_STOCHASTIC, 9, 3)
    rq = R.quantize_headwise(npy(x), layout, ra, rb, R.ROUND_STOCHASTIC, 9, 3).reshape(-1)
    assert np.array_equal(npy(q), rq)
    a2, b2 = a.clone(), b.clone()
    q2 = torch.empty_like(q)
    M.mesa_quantize_update_fused(x, layout, a2, b2, 0.9, q2, ws, M.ROUND_NEAREST_EVEN, 0, 0)
    rq2, ra2, rb2 = R.quantize_update_fused(npy(x), layout, ra, rb, 0.9, R.ROUND_NEAREST, 0, 0)
    assert np.array_equal(npy(q2), rq2.reshape(-1))
    assert np.array_equal(canon(npy(a2)), canon(ra2)) and np.array_equal(canon(npy(b2)), canon(rb2))
    qf = _mid(q, 127)
    xh = torch.empty(n, dtype=dtype, device="cuda")
    M.mesa_dequantize(qf, layout, a, b, xh)
    ref = R.dequantize(rq, layout, ra, rb)
    assert relerr(npy(xh), ref.reshape(-1)) <= TOL[dtype]
    dy = _mid(torch.randn(n, device="cuda", generator=gen).to(dtype), float("nan"))
    dx = torch.empty(n, dtype=dtype, device="cuda")
    M.mesa_gelu_bwd_q(qf, layout, a, b, dy, dx)
    g = npy(dx)
    assert np.all(np.isfinite(g))
    assert relerr(g, R.gelu_bwd_q(rq, layout, ra, rb, npy(dy)).reshape(-1)) <= TOL[dtype]


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16], ids=["f16", "bf16"])
@pytest.mark.parametrize("M_,K,N,G", [(1000, 256, 256, 4), (333, 96, 80, 3), (4097, 768, 144, 12), (65, 1024, 520, 8), (31, 64, 64, 1)])
def test_weight_gradient_uses_nothing_from_outside_its_inputs(M, M_, K, N, G, dtype):
    """The Linear weight gradient with its codes between extreme codes and dy between NaN: the prefetch ring runs past
    the last stage and the last rows do not fill one, and none of that may reach dW or db."""
    gen = torch.Generator(device="cuda").manual_seed(M_ + K + N)
    xq = _mid(torch.randint(-128, 128, (M_, K), dtype=torch.int8, device="cuda", generator=gen), 127)
    dy = _mid(torch.randn((M_, N), device="cuda", generator=gen).to(dtype), float("nan"))
    a = 0.5 + 3.0 * torch.rand(G, device="cuda", generator=gen)
    b = -2.0 * torch.rand(G, device="cuda", generator=gen)
    dW = torch.empty((N, K), device="cuda")
    db = torch.empty(N, device="cuda")
    dtc = M.F16 if dtype == torch.float16 else M.BF16
    ws = torch.empty(max(M.workspace_bytes(M.OP_LINEAR_DW_Q, M_, K, N, dtc), 16), dtype=torch.uint8, device="cuda")
    M.mesa_linear_dw_q(xq, M_, K, G, a, b, dy, N, dW, db, ws)
    rW, rb = R.linear_dw_q(npy(xq), M_, K, G, npy(a), npy(b), npy(dy), N)
    gW, gb = npy(dW), npy(db)
    assert np.all(np.isfinite(gW)) and np.all(np.isfinite(gb))
    assert relerr(gW, rW) <= 2e-3 and relerr(gb, rb) <= 2e-3, (relerr(gW, rW), relerr(gb, rb))


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16], ids=["f16", "bf16"])
def test_row_kernels_use_nothing_from_outside_their_inputs(M, dtype):
    """Softmax backward and LayerNorm backward over rows that end the buffers: codes between extreme codes, gradients
    between NaN."""
    gen = torch.Generator(device="cuda").manual_seed(5)
    for (B, H, rows, cols) in ((2, 3, 197, 197), (1, 2, 50, 49), (1, 1, 9, 577), (1, 2, 6, 1024), (1, 1, 3, 4104)):
        n = B * H * rows * cols
        yq = _mid(torch.randint(-128, 128, (n,), dtype=torch.int8, device="cuda", generator=gen), 127)
        dy = _mid(torch.randn((B, H, rows, cols), device="cuda", generator=gen).to(dtype), float("nan"))
        a = 0.5 + torch.rand(H, device="cuda", generator=gen)
        b = torch.zeros(H, device="cuda")
        dx = torch.empty((B, H, rows, cols), dtype=dtype, device="cuda")
        M.mesa_softmax_bwd_q(yq, B, H, rows, cols, a, b, dy, dx)
        g = npy(dx)
        assert np.all(np.isfinite(g)), (rows, cols)
        ref = R.softmax_bwd_q(npy(yq), B, H, rows, cols, npy(a), npy(b), npy(dy))
        assert relerr(g.reshape(ref.shape), ref) <= TOL[dtype], (rows, cols)
    for (Mr, D, G) in ((197, 768, 12), (33, 1024, 16), (50, 96, 3), (9, 2048, 4), (5, 520, 1), (7, 100, 1)):
        xq = _mid(torch.randint(-128, 128, (Mr, D), dtype=torch.int8, device="cuda", generator=gen), -128)
        dy = _mid(torch.randn((Mr, D), device="cuda", generator=gen).to(dtype), float("nan"))
        gamma = (1 + 0.1 * torch.randn(D, device="cuda", generator=gen)).to(dtype)
        mean = 0.1 * torch.randn(Mr, device="cuda", generator=gen)
        rstd = 0.5 + torch.rand(Mr, device="cuda", generator=gen)
        a = 4.0 + torch.rand(G, device="cuda", generator=gen)
        b = -2.0 - torch.rand(G, device="cuda", generator=gen)
        dx = torch.empty((Mr, D), dtype=dtype, device="cuda")
        dg = torch.empty(D, device="cuda")
        dbt = torch.empty(D, device="cuda")
        dtc = M.F16 if dtype == torch.float16 else M.BF16
        ws = torch.empty(max(M.workspace_bytes(M.OP_LAYERNORM_BWD_Q, Mr, D, G, dtc), 16), dtype=torch.uint8, device="cuda")
        M.mesa_layernorm_bwd_q(xq, Mr, D, G, a, b, mean, rstd, gamma, dy, dx, dg, dbt, ws)
        rdx, rdg, rdb = R.layernorm_bwd_q(npy(xq), Mr, D, G, npy(a), npy(b), npy(mean), npy(rstd), npy(gamma), npy(dy))
        for name, got, ref in (("dx", dx, rdx), ("dgamma", dg, rdg), ("dbeta", dbt, rdb)):
            gg = npy(got)
            assert np.all(np.isfinite(gg)), (name, Mr, D)
            assert relerr(gg.reshape(ref.shape), ref) <= TOL[dtype], (name, Mr, D, relerr(gg.reshape(ref.shape), ref))
