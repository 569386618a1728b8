"""The entry point for callers that cannot allocate: mesa_update_running_params_static (partial extrema in a
device array the library owns) against mesa_update_running_params (the same kernels on a caller's workspace),
through the C ABI, bit for bit, on two calls in a row -- the second on a smaller input, so that whatever the
first call left in the shared array must not leak into the second -- and against the CPU oracle."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import mesa_ref as R

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def M():
    import paper_2111_11124_amd as m
    assert torch.cuda.is_available(), "these tests need the MI355X"
    m.lib()
    return m


def bits(t):
    return (t.float().cpu().numpy() + np.float32(0.0)).view(np.uint32)


@pytest.mark.parametrize("dtype", [torch.float16, torch.float32, torch.bfloat16], ids=["f16", "f32", "bf16"])
def test_static_scratch_update_equals_workspace_update_twice_in_a_row(M, dtype):
    L = M.lib()
    stream = torch.cuda.current_stream().cuda_stream
    dtc = {torch.float32: M.F32, torch.float16: M.F16, torch.bfloat16: M.BF16}[dtype]
    g = torch.Generator(device="cuda").manual_seed(77)
    # the large call first (many workgroups' partials land in the array), then a small one whose grid is a
    # fraction of it, then one with more groups than either, then many groups on a tensor large enough that the
    # workspace form would use more workgroups than the array has room for (the static form runs on fewer)
    layouts = [(64, 12, 197 * 197), (3, 5, 361), (500, 48, 24), (1, 1024, 9001)]
    assert M.workspace_bytes(M.OP_UPDATE_RUNNING_PARAMS, 1, 1024, 9001, dtc) > M.static_scratch_bytes()
    for step, (outer, G, inner) in enumerate(layouts):
        x = (torch.randn((outer, G, inner), generator=g, device="cuda") * (1.0 + step) - 0.5 * step).to(dtype).contiguous()
        lay = M.Layout(outer, G, inner)
        for first_call in (1, 0):
            a0 = torch.full((G,), 3.0 + step, device="cuda")
            b0 = torch.full((G,), -1.0 - step, device="cuda")
            a1, b1 = a0.clone(), b0.clone()
            st = L.mesa_update_running_params_static(C.c_void_p(x.data_ptr()), dtc, lay, C.c_void_p(a1.data_ptr()),
                                                     C.c_void_p(b1.data_ptr()), C.c_float(0.9), first_call, C.c_void_p(stream))
            assert st == M.OK, M.status_string(st)
            ws = torch.empty(max(16, M.workspace_bytes(M.OP_UPDATE_RUNNING_PARAMS, outer, G, inner, dtc)), dtype=torch.uint8,
                             device="cuda")
            st = L.mesa_update_running_params(C.c_void_p(x.data_ptr()), dtc, lay, C.c_void_p(a0.data_ptr()),
                                              C.c_void_p(b0.data_ptr()), C.c_float(0.9), first_call, C.c_void_p(ws.data_ptr()),
                                              C.c_size_t(ws.numel()), C.c_void_p(stream))
            assert st == M.OK, M.status_string(st)
            torch.cuda.synchronize()
            assert np.array_equal(bits(a1), bits(a0)) and np.array_equal(bits(b1), bits(b0)), (step, first_call)
            xf = (x.float() if dtype == torch.bfloat16 else x).cpu().numpy()
            ra, rb = R.update_running_params(xf, (outer, G, inner), np.full(G, 3.0 + step, np.float32),
                                             np.full(G, -1.0 - step, np.float32), 0.9, bool(first_call))
            assert np.array_equal(bits(a1), (ra + np.float32(0)).view(np.uint32)), (step, first_call)
            assert np.array_equal(bits(b1), (rb + np.float32(0)).view(np.uint32)), (step, first_call)


def test_static_scratch_rejects_what_does_not_fit(M):
    L = M.lib()
    assert M.static_scratch_bytes() == 1 << 20
    x = torch.zeros(8 * 8192 * 8, dtype=torch.float16, device="cuda")
    a = torch.zeros(8192, device="cuda")
    b = torch.zeros(8192, device="cuda")
    lay = M.Layout(8, 8192, 8)
    assert M.workspace_bytes(M.OP_UPDATE_RUNNING_PARAMS, 8, 8192, 8, M.F16) > M.static_scratch_bytes()
    st = L.mesa_update_running_params_static(C.c_void_p(x.data_ptr()), M.F16, lay, C.c_void_p(a.data_ptr()), C.c_void_p(b.data_ptr()),
                                             C.c_float(0.9), 1, None)
    assert st == M.ERR_UNSUPPORTED
    assert L.mesa_update_running_params_static(C.c_void_p(x.data_ptr()), M.F16, M.Layout(1, 8, 8), C.c_void_p(a.data_ptr()),
                                               C.c_void_p(b.data_ptr()), C.c_float(1.5), 1, None) == M.ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert float(a.abs().max()) == 0.0 and float(b.abs().max()) == 0.0   # nothing was written
