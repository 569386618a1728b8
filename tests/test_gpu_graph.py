"""The library's calls inside a captured HIP graph: none of them allocates, clears memory or synchronises,
so a captured step must replay to exactly what the same calls produce eagerly -- on every replay, with
eager work and synchronisations in between."""
import pytest
import torch

import mesa_workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def M():
    import paper_2111_11124_amd as m
    assert torch.cuda.is_available()
    m.lib()
    return m


def ws(m, op, a, b, c):
    return torch.empty(max(m.workspace_bytes(op, a, b, c, m.F16), 16), dtype=torch.uint8, device="cuda")


def test_a_captured_step_replays_to_the_eager_results(M):
    spec = W.small_case(torch.float16, B=6, H=3, N=49, D=96, mlp=384)
    dev = "cuda"
    B, H, N, _ = spec.attn
    Dh = spec.dim // spec.heads
    lay_a, lay_g = spec.attn_layout, spec.gelu_layout
    y = W.attention_map(spec, 0, dev)
    xg = W.gelu_input(spec, 0, dev)
    dy_a = W.upstream_grad(spec, "dy_attn", y.shape, dev)
    dy_g = W.upstream_grad(spec, "dy_gelu", xg.shape, dev)
    g = torch.Generator(device=dev).manual_seed(5)
    dO = torch.randn((B, H, N, Dh), device=dev, generator=g).half()
    vq = torch.randint(-128, 128, (B, H, N, Dh), dtype=torch.int8, device=dev, generator=g)
    xl = (torch.randn((B * N, spec.dim), device=dev, generator=g) * 0.7).half()
    dyl = torch.randn((B * N, spec.mlp), device=dev, generator=g).half()
    lay_l = (B * N, H, spec.dim // H)

    init = {"aa": torch.full((H,), 0.8, device=dev), "ba": torch.full((H,), 0.0, device=dev),
            "ag": torch.full((H,), 6.0, device=dev), "bg": torch.full((H,), -3.0, device=dev),
            "al": torch.full((H,), 5.0, device=dev), "bl": torch.full((H,), -2.5, device=dev)}
    st = {k: v.clone() for k, v in init.items()}
    buf = {"qa": torch.empty(y.numel(), dtype=torch.int8, device=dev), "qg": torch.empty(xg.numel(), dtype=torch.int8, device=dev),
           "ql": torch.empty(xl.numel(), dtype=torch.int8, device=dev), "dxa": torch.empty_like(dy_a), "dxg": torch.empty_like(dy_g),
           "dA": torch.empty((B, H, N, N), dtype=torch.half, device=dev), "dV": torch.empty_like(dO),
           "dW": torch.empty((spec.mlp, spec.dim), device=dev), "db": torch.empty(spec.mlp, device=dev)}
    w_a, w_g, w_l = (ws(M, M.OP_UPDATE_RUNNING_PARAMS, *l) for l in (lay_a, lay_g, lay_l))
    w_dw = ws(M, M.OP_LINEAR_DW_Q, B * N, spec.dim, spec.mlp)

    def step():
        M.mesa_update_running_params(y, lay_a, st["aa"], st["ba"], 0.9, False, w_a)
        M.mesa_quantize_headwise(y, lay_a, st["aa"], st["ba"], buf["qa"], M.ROUND_STOCHASTIC, 3, 0)
        M.mesa_quantize_update_fused(xg, lay_g, st["ag"], st["bg"], 0.9, buf["qg"], w_g, M.ROUND_STOCHASTIC, 4, 0)
        M.mesa_update_running_params_sym(xl, lay_l, st["al"], st["bl"], 0.9, False, w_l)
        M.mesa_quantize_headwise(xl, lay_l, st["al"], st["bl"], buf["ql"], M.ROUND_NEAREST_EVEN)
        M.mesa_softmax_bwd_q(buf["qa"], B, H, N, N, st["aa"], st["ba"], dy_a, buf["dxa"])
        M.mesa_gelu_bwd_q(buf["qg"], lay_g, st["ag"], st["bg"], dy_g, buf["dxg"])
        M.mesa_attn_av_bwd_q(buf["qa"], vq, B, H, N, Dh, st["aa"], st["ba"], st["ag"], st["bg"], dO, buf["dA"], buf["dV"])
        M.mesa_linear_dw_q(buf["ql"], B * N, spec.dim, H, st["al"], st["bl"], dyl, spec.mlp, buf["dW"], buf["db"], w_dw)

    # eager: three steps from the initial estimates, every step's results kept
    eager = []
    for _ in range(3):
        step()
        torch.cuda.synchronize()
        eager.append({k: v.clone() for k, v in list(st.items()) + list(buf.items())})

    # captured once, from the same initial estimates; replayed three times with eager work in between
    for k in st:
        st[k].copy_(init[k])
    for v in buf.values():
        v.zero_()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    scratch = torch.empty_like(dy_g)
    for t in range(3):
        graph.replay()
        M.mesa_dequantize(buf["qg"], lay_g, st["ag"], st["bg"], scratch)    # the program's own eager work
        scratch.mul_(2.0)
        torch.cuda.synchronize()
        for k, ref in eager[t].items():
            got = st[k] if k in st else buf[k]
            assert torch.equal(got, ref), (t, k)


def test_captured_layer_forwards_and_the_remaining_backwards_replay_exactly(M):
    """The calls the first test leaves out: the three layer forwards (dynamic LDS, running estimates read and
    moved inside one call), LayerNorm backward, the fixed-offset update, ReLU backward, de-quantize and the
    Q K^T product's backward."""
    dev = "cuda"
    B, H, N, Dh = 4, 3, 49, 32
    D, mlp = H * Dh, 4 * H * Dh
    Mr = B * N
    g = torch.Generator(device=dev).manual_seed(9)
    s = (torch.randn((B, H, N, N), device=dev, generator=g) * 2).half()
    xg = (torch.randn((Mr, mlp), device=dev, generator=g) * 1.5).half()
    xl = (torch.randn((Mr, D), device=dev, generator=g) + 0.3).half()
    gamma = (1 + 0.1 * torch.randn(D, device=dev, generator=g)).half()
    bias = (0.1 * torch.randn(D, device=dev, generator=g)).half()
    dyl = torch.randn((Mr, D), device=dev, generator=g).half()
    dyg = torch.randn((Mr, mlp), device=dev, generator=g).half()
    dS = (torch.randn((B, H, N, N), device=dev, generator=g) * 0.1).half()
    kq = torch.randint(-128, 128, (B, H, N, Dh), dtype=torch.int8, device=dev, generator=g)
    lay_g, lay_l = (Mr, H, mlp // H), (Mr, H, D // H)
    init = {"aa": torch.full((H,), 0.8, device=dev), "ba": torch.full((H,), 0.0, device=dev),
            "ag": torch.full((H,), 6.0, device=dev), "bg": torch.full((H,), -3.0, device=dev),
            "al": torch.full((H,), 5.0, device=dev), "bl": torch.full((H,), -2.5, device=dev),
            "af": torch.full((H,), 4.0, device=dev), "bf": torch.full((H,), -0.17, device=dev)}
    st = {k: v.clone() for k, v in init.items()}
    buf = {"y": torch.empty_like(s), "qa": torch.empty(s.numel(), dtype=torch.int8, device=dev),
           "yg": torch.empty_like(xg), "qg": torch.empty(xg.numel(), dtype=torch.int8, device=dev),
           "yl": torch.empty_like(xl), "ql": torch.empty(xl.numel(), dtype=torch.int8, device=dev),
           "mean": torch.empty(Mr, device=dev), "rstd": torch.empty(Mr, device=dev),
           "dxl": torch.empty_like(dyl), "dgamma": torch.empty(D, device=dev), "dbeta": torch.empty(D, device=dev),
           "dxr": torch.empty_like(dyg), "xhat": torch.empty_like(xg),
           "dQ": torch.empty((B, H, N, Dh), dtype=torch.half, device=dev), "dK": torch.empty((B, H, N, Dh), dtype=torch.half, device=dev)}
    w_s = ws(M, M.OP_SOFTMAX_FWD_Q, B * H * N, H, N)
    w_g = ws(M, M.OP_UPDATE_RUNNING_PARAMS, *lay_g)
    w_lf = ws(M, M.OP_LAYERNORM_FWD_Q, Mr, D, H)
    w_lb = ws(M, M.OP_LAYERNORM_BWD_Q, Mr, D, H)

    def step():
        M.mesa_softmax_fwd_q(s, B, H, N, N, st["aa"], st["ba"], 0.9, buf["y"], buf["qa"], w_s, M.ROUND_STOCHASTIC, 7, 0)
        M.mesa_gelu_fwd_q(xg, lay_g, st["ag"], st["bg"], 0.9, buf["yg"], buf["qg"], w_g, M.ROUND_STOCHASTIC, 8, 0)
        M.mesa_layernorm_fwd_q(xl, Mr, D, H, gamma, bias, 1e-5, st["al"], st["bl"], 0.9, buf["yl"], buf["mean"], buf["rstd"], buf["ql"],
                               w_lf, M.ROUND_NEAREST_EVEN, 0, 0)
        M.mesa_update_running_params_fixed_beta(buf["yg"], lay_g, st["af"], st["bf"], 0.9, False, -0.17, w_g)
        M.mesa_layernorm_bwd_q(buf["ql"], Mr, D, H, st["al"], st["bl"], buf["mean"], buf["rstd"], gamma, dyl, buf["dxl"], buf["dgamma"],
                               buf["dbeta"], w_lb)
        M.mesa_relu_bwd_q(buf["qg"], lay_g, st["ag"], st["bg"], dyg, buf["dxr"])
        M.mesa_dequantize(buf["qg"], lay_g, st["ag"], st["bg"], buf["xhat"])
        M.mesa_attn_qk_bwd_q(buf["ql"], kq, B, H, N, Dh, st["al"], st["bl"], st["ag"], st["bg"], dS, 0.25, buf["dQ"], buf["dK"])

    eager = []
    for _ in range(3):
        step()
        torch.cuda.synchronize()
        eager.append({k: v.clone() for k, v in list(st.items()) + list(buf.items())})
    for k in st:
        st[k].copy_(init[k])
    for v in buf.values():
        v.zero_()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    scratch = torch.empty_like(dyl)
    for t in range(3):
        graph.replay()
        scratch.copy_(buf["dxl"])                     # the program's own eager work between replays
        scratch.mul_(0.5)
        torch.cuda.synchronize()
        for k, ref in eager[t].items():
            got = st[k] if k in st else buf[k]
            assert torch.equal(got, ref), (t, k)


def test_captured_scale_only_four_bit_static_scratch_and_convolution_calls_replay_exactly(M):
    """The later additions: the scale-only symmetric trio, the four-bit trio, the update that keeps its partial
    extrema in the library's own static array (whose contents survive from replay to replay), and the convolution
    weight gradient on both of its paths (the matrix-core one raises its kernel's LDS limit on every call)."""
    dev = "cuda"
    Mr, H, mlp = 197 * 3, 3, 384
    g = torch.Generator(device=dev).manual_seed(21)
    x = (torch.randn((Mr, mlp), device=dev, generator=g) * 1.5).half()
    dy = torch.randn((Mr, mlp), device=dev, generator=g).half()
    lay = (Mr, H, mlp // H)
    n = x.numel()
    init = {"m": torch.full((H,), 5.0, device=dev), "a": torch.full((H,), 6.0, device=dev), "b": torch.full((H,), -3.0, device=dev)}
    st = {k: v.clone() for k, v in init.items()}
    buf = {"qs": torch.empty(n, dtype=torch.int8, device=dev), "xs": torch.empty_like(x),
           "q4": torch.empty((n + 1) // 2, dtype=torch.uint8, device=dev), "x4": torch.empty_like(x), "dx4": torch.empty_like(dy)}
    w = ws(M, M.OP_UPDATE_RUNNING_PARAMS, *lay)
    cv3 = M.Conv2d(2, 48, 12, 24, 40, 3, 3, 1, 1, 1, 1, 1, 1)          # matrix cores
    cv5 = M.Conv2d(2, 6, 9, 10, 4, 5, 5, 2, 2, 2, 2, 1, 1)             # the plain kernel
    xq3 = torch.randint(-128, 128, (2, 48, 12, 24), dtype=torch.int8, device=dev, generator=g)
    xq5 = torch.randint(-128, 128, (2, 6, 9, 10), dtype=torch.int8, device=dev, generator=g)
    dy3 = torch.randn((2, 40) + cv3.out_hw(), device=dev, generator=g).half()
    dy5 = torch.randn((2, 4) + cv5.out_hw(), device=dev, generator=g).half()
    buf.update({"dW3": torch.empty((40, 48, 3, 3), device=dev), "db3": torch.empty(40, device=dev),
                "dW5": torch.empty((4, 6, 5, 5), device=dev), "db5": torch.empty(4, device=dev)})
    w3 = torch.empty(max(M.conv2d_dw_q_workspace_bytes(cv3, M.F16), 16), dtype=torch.uint8, device=dev)

    def step():
        M.mesa_conv2d_dw_q(xq3, cv3, H, st["a"], st["b"], dy3, buf["dW3"], buf["db3"], w3)
        M.mesa_conv2d_dw_q(xq5, cv5, H, st["a"], st["b"], dy5, buf["dW5"], buf["db5"], None)
        M.mesa_update_running_scale_sym(x, lay, st["m"], 0.9, False, w)
        M.mesa_quantize_sym(x, lay, st["m"], buf["qs"], M.ROUND_STOCHASTIC, 11, 0)
        M.mesa_dequantize_sym(buf["qs"], lay, st["m"], buf["xs"])
        M.mesa_update_running_params_static(x, lay, st["a"], st["b"], 0.9, False)
        M.mesa_quantize_headwise_b4(x, lay, st["a"], st["b"], buf["q4"], M.ROUND_STOCHASTIC, 12, 0)
        M.mesa_dequantize_b4(buf["q4"], lay, st["a"], st["b"], buf["x4"])
        M.mesa_gelu_bwd_q_b4(buf["q4"], lay, st["a"], st["b"], dy, buf["dx4"])

    eager = []
    for _ in range(3):
        step()
        torch.cuda.synchronize()
        eager.append({k: v.clone() for k, v in list(st.items()) + list(buf.items())})
    for k in st:
        st[k].copy_(init[k])
    for v in buf.values():
        v.zero_()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    other = (torch.randn((64, H, 40), device=dev, generator=g)).half()
    oa, ob = torch.zeros(H, device=dev), torch.zeros(H, device=dev)
    for t in range(3):
        graph.replay()
        M.mesa_update_running_params_static(other, (64, H, 40), oa, ob, 0.9, True)   # eager work that dirties the static array
        torch.cuda.synchronize()
        for k, ref in eager[t].items():
            got = st[k] if k in st else buf[k]
            assert torch.equal(got, ref), (t, k)
