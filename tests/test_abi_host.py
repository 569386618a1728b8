"""CPU-side checks of the product: the shared library loads and exports every symbol the header
declares, argument errors are reported before anything is launched, and the host-side integer
helpers (division by multiplication, launch planning) are exact."""
import ctypes as C
import os
import re
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "mesa.h")


@pytest.fixture(scope="module")
def M():
    import paper_2111_11124_amd as m
    if not os.path.exists(os.path.join(ROOT, "paper_2111_11124_amd", "libmesa.so")):
        from paper_2111_11124_amd.build import build
        build(verbose=False)
    m.lib()
    return m


def declared_functions():
    src = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(mesa_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol(M):
    names = declared_functions()
    assert len(names) >= 15 and {"mesa_quantize_headwise", "mesa_dequantize", "mesa_update_running_params",
                                 "mesa_softmax_bwd_q", "mesa_gelu_bwd_q", "mesa_layernorm_bwd_q",
                                 "mesa_linear_dw_q"} <= set(names)
    L = M.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(M.EXPORTS) == names
    assert M.version() >= 100 and M.status_string(M.ERR_WORKSPACE).startswith("workspace")


def test_argument_errors_are_reported_before_any_launch(M):
    L = M.lib()
    lay = M.Layout(2, 3, 64)
    P = 0x10000  # a 16-byte aligned fake address: never dereferenced on the host, and no call below passes the checks
    assert L.mesa_quantize_headwise(None, M.F16, lay, P, P, P, 0, 0, 0, None) == M.ERR_INVALID_ARG
    assert L.mesa_quantize_headwise(P + 2, M.F16, lay, P, P, P, 0, 0, 0, None) == M.ERR_INVALID_ARG       # misaligned
    assert L.mesa_quantize_headwise(P, 7, lay, P, P, P, 0, 0, 0, None) == M.ERR_INVALID_ARG               # dtype
    assert L.mesa_quantize_headwise(P, M.F16, lay, P, P, P, 5, 0, 0, None) == M.ERR_INVALID_ARG           # rounding mode
    assert L.mesa_quantize_headwise(P, M.F16, M.Layout(-1, 3, 4), P, P, P, 0, 0, 0, None) == M.ERR_INVALID_ARG
    assert L.mesa_quantize_headwise(P, M.F16, M.Layout(2, 9000, 4), P, P, P, 0, 0, 0, None) == M.ERR_UNSUPPORTED
    assert L.mesa_quantize_headwise(P, M.F16, M.Layout(2, 2, 1 << 30), P, P, P, 0, 0, 0, None) == M.ERR_UNSUPPORTED
    assert L.mesa_update_running_params(P, M.F16, lay, P, P, 1.5, 0, P, 1 << 20, None) == M.ERR_INVALID_ARG  # lambda
    assert L.mesa_update_running_params(P, M.F16, lay, P, P, float("nan"), 0, P, 1 << 20, None) == M.ERR_INVALID_ARG
    assert L.mesa_update_running_params(P, M.F16, lay, P, P, 0.9, 0, P, 8, None) == M.ERR_WORKSPACE
    assert L.mesa_update_running_params(P, M.F16, lay, P, P, 0.9, 0, None, 0, None) == M.ERR_WORKSPACE
    assert L.mesa_update_running_params_sym(P, M.F16, lay, P, P, 1.5, 0, P, 1 << 20, None) == M.ERR_INVALID_ARG
    assert L.mesa_update_running_params_sym(P, M.F16, lay, P, P, 0.9, 0, P, 8, None) == M.ERR_WORKSPACE
    assert L.mesa_update_running_params_fixed_beta(P, M.F16, lay, P, P, 0.9, 0, float("nan"), P, 1 << 20, None) == M.ERR_INVALID_ARG
    assert L.mesa_update_running_params_fixed_beta(P, M.F16, lay, P, P, 0.9, 0, float("inf"), P, 1 << 20, None) == M.ERR_INVALID_ARG
    assert L.mesa_update_running_params_fixed_beta(P, M.F16, lay, P, P, 0.9, 0, -0.17, P, 8, None) == M.ERR_WORKSPACE
    assert L.mesa_quantize_update_fused(P, M.F16, lay, P, P, 0.9, P, 0, 0, 0, P, 8, None) == M.ERR_WORKSPACE
    assert L.mesa_quantize_update_fused(P, M.F16, lay, P, P, -0.1, P, 0, 0, 0, P, 1 << 20, None) == M.ERR_INVALID_ARG   # lambda
    assert L.mesa_quantize_update_fused(P, M.F16, lay, P, P, 0.9, None, 0, 0, 0, P, 1 << 20, None) == M.ERR_INVALID_ARG  # q
    assert L.mesa_quantize_update_fused(P, M.F16, lay, P, P, 0.9, P, 3, 0, 0, P, 1 << 20, None) == M.ERR_INVALID_ARG     # mode
    P2 = 0x20000
    assert L.mesa_gelu_fwd_q(P, M.F16, lay, P, P, 0.9, None, P, 0, 0, 0, P, 1 << 20, None) == M.ERR_INVALID_ARG   # y missing
    assert L.mesa_gelu_fwd_q(P, M.F16, lay, P, P, 0.9, P, P, 0, 0, 0, P, 1 << 20, None) == M.ERR_INVALID_ARG      # y aliases x
    assert L.mesa_gelu_fwd_q(P, M.F16, lay, P, P, 0.9, P2, P, 0, 0, 0, P, 8, None) == M.ERR_WORKSPACE
    assert L.mesa_softmax_fwd_q(P, 2, 3, 19, 19, P, P, 0.9, P, P, 0, 0, 0, P, 1 << 20, M.F16, None) == M.ERR_INVALID_ARG   # y aliases s
    assert L.mesa_softmax_fwd_q(P, 2, 3, 19, 19, P, P, 0.9, P2, P, 0, 0, 0, P, 8, M.F16, None) == M.ERR_WORKSPACE
    assert L.mesa_softmax_fwd_q(P, 2, 3, 19, 3001, P, P, 0.9, P2, P, 0, 0, 0, P, 8, M.F16, None) == M.ERR_WORKSPACE  # the two-step path checks its workspace first
    assert L.mesa_softmax_fwd_q(P, 2, 9000, 19, 19, P, P, 0.9, P2, P, 0, 0, 0, P, 1 << 20, M.F16, None) == M.ERR_UNSUPPORTED  # heads
    assert L.mesa_softmax_fwd_q(P, 2, 3, 1 << 16, 1 << 15, P, P, 0.9, P2, P, 0, 0, 0, P, 1 << 20, M.F16, None) == M.ERR_UNSUPPORTED  # 2^31 elements a map
    assert M.workspace_bytes(M.OP_SOFTMAX_FWD_Q, 2 * 3 * 19, 3, 3001, M.F16) >= M.workspace_bytes(M.OP_UPDATE_RUNNING_PARAMS, 2, 3, 19 * 3001, M.F16)
    assert M.workspace_bytes(M.OP_SOFTMAX_FWD_Q, 6 * 7 * 1000, 7, 1025, M.F16) >= M.workspace_bytes(M.OP_UPDATE_RUNNING_PARAMS, 6, 7, 1000 * 1025, M.F16)
    assert M.workspace_bytes(M.OP_SOFTMAX_FWD_Q, 3 * 1500 * 64, 1500, 19, M.F16) >= M.workspace_bytes(M.OP_UPDATE_RUNNING_PARAMS, 3, 1500, 64 * 19, M.F16)
    assert L.mesa_softmax_fwd_q(P, 2, 3, 19, 19, P, P, 1.5, P2, P, 0, 0, 0, P, 1 << 20, M.F16, None) == M.ERR_INVALID_ARG  # lambda
    assert M.workspace_bytes(M.OP_SOFTMAX_FWD_Q, 128 * 6 * 197, 6, 197, M.F16) >= 768 * 2 * 6 * 4
    F = C.c_float
    assert L.mesa_layernorm_fwd_q(P, 100, 384, 6, P, P, F(1e-5), P, P, F(0.9), P, P, P, P, 0, 0, 0, P, 1 << 20, M.F16, None) == M.ERR_INVALID_ARG  # y aliases x
    assert L.mesa_layernorm_fwd_q(P, 100, 384, 6, P, P, F(1e-5), P, P, F(0.9), P2, P, P, P, 0, 0, 0, P, 8, M.F16, None) == M.ERR_WORKSPACE
    assert L.mesa_layernorm_fwd_q(P, 100, 4096, 8, P, P, F(1e-5), P, P, F(0.9), P2, P, P, P, 0, 0, 0, P, 8, M.F16, None) == M.ERR_WORKSPACE  # the two-step path
    assert L.mesa_layernorm_fwd_q(P, 100, 72000, 9000, P, P, F(1e-5), P, P, F(0.9), P2, P, P, P, 0, 0, 0, P, 1 << 24, M.F16, None) == M.ERR_UNSUPPORTED  # groups
    assert L.mesa_layernorm_fwd_q(P, 100, 384, 5, P, P, F(1e-5), P, P, F(0.9), P2, P, P, P, 0, 0, 0, P, 1 << 20, M.F16, None) == M.ERR_INVALID_ARG  # D % G
    assert L.mesa_layernorm_fwd_q(P, 100, 384, 6, P, P, F(-1.0), P, P, F(0.9), P2, P, P, P, 0, 0, 0, P, 1 << 20, M.F16, None) == M.ERR_INVALID_ARG  # eps
    assert L.mesa_dequantize(P, lay, P, None, P, M.F16, None) == M.ERR_INVALID_ARG
    assert L.mesa_gelu_bwd_q(P, lay, P, P, P + 8, P, M.F16, None) == M.ERR_INVALID_ARG
    assert L.mesa_softmax_bwd_q(P, 2, 3, 1 << 31, 40, P, P, P, P, M.F16, None) == M.ERR_UNSUPPORTED       # rows per head
    assert L.mesa_softmax_bwd_q(P, 1 << 20, 1 << 10, 5, 40, P, P, P, P, M.F16, None) == M.ERR_UNSUPPORTED  # 2^31 rows or more in all
    assert L.mesa_softmax_bwd_q(P, -2, 3, 5, 16, P, P, P, P, M.F16, None) == M.ERR_INVALID_ARG
    assert L.mesa_layernorm_bwd_q(P, 10, 1 << 31, 1, P, P, P, P, P, P, P, P, P, M.F16, P, 1 << 20, None) == M.ERR_UNSUPPORTED
    assert L.mesa_layernorm_bwd_q(P, 10, 96, 5, P, P, P, P, P, P, P, P, P, M.F16, P, 1 << 20, None) == M.ERR_INVALID_ARG
    assert L.mesa_layernorm_bwd_q(P, 10, 96, 3, P, P, P, P, P, P, P, P, P, M.F16, P, 16, None) == M.ERR_WORKSPACE
    assert L.mesa_linear_dw_q(P, 100, 1 << 20, 1, P, P, P, 1 << 12, M.F16, P, None, P, 1 << 30, None) == M.ERR_UNSUPPORTED   # K * N_out >= 2^31
    assert L.mesa_linear_dw_q(P, 100, 48, 5, P, P, P, 64, M.F16, P, None, P, 1 << 30, None) == M.ERR_INVALID_ARG   # K % G
    assert L.mesa_linear_dw_q(P, 100, 48, 3, P, P, P, 64, M.F16, P, None, P, 64, None) == M.ERR_WORKSPACE
    assert L.mesa_attn_av_bwd_q(P, P, 2, 3, 1 << 20, 8, P, P, P, P, P, P, P, M.F16, None) == M.ERR_UNSUPPORTED     # sequence too long
    assert L.mesa_attn_av_bwd_q(P, P, 2, 3, 19, 8, P, P, P, P, None, P, P, M.BF16, None) == M.ERR_INVALID_ARG      # bfloat16 is accepted
    assert L.mesa_attn_qk_bwd_q(P, P, 2, 3, 19, 8, P, P, P, P, None, 0.5, P, P, M.F32, None) == M.ERR_INVALID_ARG   # binary32 is accepted
    assert L.mesa_linear_dw_q(P, 100, 48, 3, P, P, P, 64, M.BF16, P, None, P, 64, None) == M.ERR_WORKSPACE        # bfloat16 is a valid type
    assert L.mesa_quantize_headwise(P, 3, lay, P, P, P, 0, 0, 0, None) == M.ERR_INVALID_ARG                       # one past the last type
    assert L.mesa_attn_av_bwd_q(P, P, 2, 3, 19, 8, P, P, P, P, None, P, P, M.F16, None) == M.ERR_INVALID_ARG
    assert L.mesa_attn_qk_bwd_q(P, P, 2, 3, 19, 8, P, P, P, P, P, float("nan"), P, P, M.F16, None) == M.ERR_INVALID_ARG
    assert L.mesa_attn_qk_bwd_q(P, P + 4, 2, 3, 19, 8, P, P, P, P, P, 0.5, P, P, M.F16, None) == M.ERR_INVALID_ARG
    assert L.mesa_attn_qk_bwd_q(None, None, 0, 3, 19, 8, None, None, None, None, None, 0.5, None, None, M.F16, None) == M.OK
    assert L.mesa_stream_copy(P, P, 24, None) == M.ERR_INVALID_ARG
    assert L.mesa_mfma_probe(4, 10, None, 0, P, None) == M.ERR_INVALID_ARG            # no such form
    assert L.mesa_mfma_probe(0, -1, None, 0, P, None) == M.ERR_INVALID_ARG
    assert L.mesa_mfma_probe(0, 10, None, 0, None, None) == M.ERR_INVALID_ARG         # no sink
    assert L.mesa_mfma_probe(2, 10, P, 4096, P, None) == M.ERR_INVALID_ARG            # feed below 2 MiB
    # zero elements: OK without touching anything
    assert L.mesa_quantize_headwise(None, M.F16, M.Layout(0, 3, 64), None, None, None, 0, 0, 0, None) == M.OK
    assert L.mesa_softmax_bwd_q(None, 0, 3, 5, 16, None, None, None, None, M.F16, None) == M.OK


def test_workspace_sizes(M):
    assert M.workspace_bytes(M.OP_UPDATE_RUNNING_PARAMS, 128, 6, 38809) >= 2 * 6 * 4
    assert M.workspace_bytes(M.OP_LAYERNORM_BWD_Q, 25216, 384, 6) >= 2 * 384 * 4
    n = M.workspace_bytes(M.OP_LINEAR_DW_Q, 25216, 384, 1536, M.F16)
    assert n >= (384 * 1536 + 1536) * 4 and n < (1 << 31)
    assert M.workspace_bytes(99, 1, 1, 1) == 0


HOST_TEST = r'''
#include <cstdio>
#include <cstdlib>
#include "host_math.hpp"
using namespace mesa;
int main() {
    // division by multiplication is exact for every dividend below 2^31 that matters: all small
    // dividends, and dividends around every multiple boundary and at the top of the range
    const uint32_t ds[] = {1, 2, 3, 5, 7, 8, 12, 16, 24, 32, 48, 49, 64, 96, 128, 197, 256, 384, 2401, 4096, 38809,
                           65535, 65536, 1000003, 16777216, 2147483647u};
    for (uint32_t d : ds) {
        FastDiv f = make_fastdiv(d);
        for (uint32_t n = 0; n < 200000; ++n) if (fastdiv_host(n, f) != n / d) { printf("FAIL d=%u n=%u\n", d, n); return 1; }
        for (uint64_t q = 1; q * d < 2147483648ull; q += (2147483648ull / d) / 997 + 1)
            for (int64_t o = -2; o <= 2; ++o) {
                int64_t n = int64_t(q * d) + o;
                if (n < 0 || n >= 2147483648ll) continue;
                if (fastdiv_host(uint32_t(n), f) != uint32_t(n) / d) { printf("FAIL d=%u n=%lld\n", d, (long long)n); return 1; }
            }
        if (fastdiv_host(2147483647u, f) != 2147483647u / d) { printf("FAIL top d=%u\n", d); return 1; }
    }
    // cursor constants: stepping by `step` elements moves (rem, g) as plain division says
    const int64_t cases[][3] = {{6, 38809, 2048 * 8 * 4}, {6, 64, 1365 * 8192}, {3, 2401, 777 * 8192}, {1, 12345, 8192}, {5, 3, 8192}};
    for (auto &c : cases) {
        GroupGeom g = make_geom(c[0], c[1], c[2]);
        for (int64_t e = 0; e < 100000; e += 8) {
            uint32_t rem = uint32_t(e % g.inner), grp = uint32_t((e / g.inner) % g.groups);
            uint32_t r = rem + g.step_rem; uint32_t carry = r >= g.inner; r -= carry ? g.inner : 0;
            uint32_t gg = grp + g.step_g + carry; if (gg >= g.groups) gg -= g.groups;
            int64_t e2 = e + c[2];
            if (r != uint32_t(e2 % g.inner) || gg != uint32_t((e2 / g.inner) % g.groups)) { printf("FAIL cursor\n"); return 1; }
        }
    }
    printf("OK\n");
    return 0;
}
'''


def test_host_integer_helpers_are_exact():
    with tempfile.TemporaryDirectory() as d:
        src = os.path.join(d, "t.cpp")
        open(src, "w").write(HOST_TEST)
        exe = os.path.join(d, "t")
        subprocess.run(["g++", "-O2", "-std=c++17", "-I", os.path.join(ROOT, "paper_2111_11124_amd", "csrc"), src, "-o", exe],
                       check=True)
        out = subprocess.run([exe], capture_output=True, text=True)
        assert out.returncode == 0 and out.stdout.strip() == "OK", out.stdout


def test_the_binding_has_no_fallback(monkeypatch, tmp_path):
    """Without the shared library every call fails loudly; host tensors are refused before anything is called."""
    import torch
    from paper_2111_11124_amd import _ffi
    monkeypatch.setattr(_ffi, "_lib", None)
    monkeypatch.setattr(_ffi, "_LIB_PATH", tmp_path / "libmesa.so")
    x = torch.zeros(64)
    with pytest.raises(RuntimeError, match="no fallback"):
        _ffi.lib()
    with pytest.raises(RuntimeError, match="no fallback"):
        _ffi.workspace_bytes(_ffi.OP_UPDATE_RUNNING_PARAMS, 1, 1, 64)
    monkeypatch.undo()
    _ffi.lib()
    q = torch.zeros(64, dtype=torch.int8)
    a = torch.ones(1)
    with pytest.raises(ValueError, match="device tensors"):
        _ffi.mesa_quantize_headwise(x, (1, 1, 64), a, a, q)


def test_softmax_forward_workspace_covers_the_two_step_path():
    """Rows that no single-pass softmax kernel takes (odd lengths above 1024, more than 1024 heads) run a plain softmax
    and then the single-pass quantizer, whose workspace depends on how the rows split into batch and rows per map -- which
    the size query is not told.  Its answer must cover every split."""
    import random
    import paper_2111_11124_amd as M
    rnd = random.Random(5)
    for _ in range(400):
        if rnd.random() < 0.5:
            H, cols = rnd.randint(1, 40), 2 * rnd.randint(513, 4000) + 1
        else:
            H, cols = rnd.randint(1025, 8192), rnd.randint(1, 300)
        B, rows = rnd.randint(1, 64), rnd.randint(1, 3000)
        if B * H * rows >= 1 << 31 or rows * cols >= 1 << 30:
            continue
        have = M.workspace_bytes(M.OP_SOFTMAX_FWD_Q, B * H * rows, H, cols, M.F16)
        need = M.workspace_bytes(M.OP_UPDATE_RUNNING_PARAMS, B, H, rows * cols, M.F16)
        assert have >= need, (B, H, rows, cols, have, need)
        # the same number of rows split the other way round
        need2 = M.workspace_bytes(M.OP_UPDATE_RUNNING_PARAMS, rows, H, B * cols, M.F16)
        assert have >= need2, (rows, H, B, cols, have, need2)
