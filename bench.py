#!/usr/bin/env python3
"""bench.py -- one-GPU throughput of libmesa's hot path.

Default workload: the DeiT-B-shaped 12-block saved-activation set at batch 256, fp16 (configs[3] of
the benchmark spec, the largest configuration that is a whole model's worth of calls).  A step is one
training iteration's worth of the method over that set:
  forward   blocks 0..11, for every saved tensor of a block -- LayerNorm-1 input, QKV input, attention
            map, projection input, LayerNorm-2 input, FC1 input, GELU input, FC2 input --
            mesa_update_running_params, then mesa_quantize_headwise (stochastic rounding);
  backward  blocks 11..0: mesa_linear_dw_q for the four Linear layers (3072->768, 768->3072, 768->768,
            768->2304), mesa_layernorm_bwd_q twice, mesa_gelu_bwd_q, mesa_softmax_bwd_q, and one
            stand-alone mesa_dequantize of the projection input's codes.
Every block has its own buffers (about 4 GB a block, 49 GB in all) and its own running estimates, so
whatever a kernel reads was last touched gigabytes of traffic earlier: cold for the 256 MB
memory-side cache.  The reuses that remain are the method's own: quantize re-reads the tensor whose
min/max were just taken, and the last block's backward follows its forward.
The other configurations (--config 2, 3, 5) are one block each; there three buffer sets rotate and the
backward half of step i consumes what step i-1 quantized.

All inputs are synthetic, seeded, and resident in HBM before the timed region.
Prints ONE JSON line (the fields are described in README.md).
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import math
import os
import re
import statistics
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import mesa_workloads as W  # noqa: E402

HBM_PEAK_GBS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2500.0
NSETS = 3
HEADLINE_CONFIG = 4
BLOCKS = {2: 1, 3: 1, 4: 12, 5: 1}        # blocks per step
LN_PER_BLOCK = {2: 1, 3: 1, 4: 2, 5: 1}   # the whole-model configuration has both LayerNorms of a block


def elem_bytes(dtype):
    return 4 if dtype == torch.float32 else 2


def dtype_code(m, dtype):
    return {torch.float32: m.F32, torch.float16: m.F16, torch.bfloat16: m.BF16}[dtype]


DTYPE_NAME = {torch.float32: "f32", torch.float16: "f16", torch.bfloat16: "bf16"}


def saved_tensors(spec, number):
    """The tensors one block saves: (name, kind, layout, shape); kind in softmax / gelu / ln / lin."""
    H = spec.heads
    out = [("attn", "softmax", spec.attn_layout, spec.attn), ("gelu", "gelu", spec.gelu_layout, (spec.tokens, spec.mlp))]
    for i in range(LN_PER_BLOCK.get(number, 1)):
        out.append((f"ln{i}", "ln", spec.ln_layout, (spec.tokens, spec.dim)))
    for i, (K, N) in enumerate(spec.linears):
        out.append((f"lin{i}", "lin", (spec.tokens, H, K // H), (spec.tokens, K)))
    return out


def algorithmic_bytes(spec, number=None):
    """Bytes each call of ONE block must move at the very least (per-element figures x elements)."""
    if number is None:
        number = next(k for k, v in W.CONFIGS.items() if v.name == spec.name or spec.name.startswith(v.name))
    T = elem_bytes(spec.dtype)
    b = {}
    for name, kind, layout, shape in saved_tensors(spec, number):
        n = layout[0] * layout[1] * layout[2]
        b[f"update_{name}"] = T * n
        b[f"quantize_{name}"] = (T + 1) * n
        if kind == "softmax":
            b["softmax_bwd_q"] = (1 + 2 * T) * n
        elif kind == "gelu":
            b["gelu_bwd_q"] = (1 + 2 * T) * n
        elif kind == "ln":
            b[f"layernorm_bwd_q_{name}"] = (1 + 2 * T) * n + 8 * spec.tokens + (T + 8) * spec.dim
        else:
            K, N = spec.linears[int(name[3:])]
            b[f"linear_dw_q_{name}"] = spec.tokens * K + T * spec.tokens * N + 4 * N * K + 4 * N
    if spec.linears:
        b["dequantize_lin0"] = (1 + T) * spec.tokens * spec.linears[0][0]
    return b


class Block:
    """One block's buffers: inputs, codes, upstream gradients, outputs.  `draw` makes the values distinct."""

    def __init__(self, m, spec, number, draw):
        dev = "cuda"
        self.t = {}
        for i, (name, kind, layout, shape) in enumerate(saved_tensors(spec, number)):
            d = draw * 8 + i
            if kind == "softmax":
                x = W.attention_map(spec, d, dev)
            elif kind == "gelu":
                x = W.gelu_input(spec, d, dev)
            elif kind == "ln":
                x = W.token_matrix(spec, "ln", d, dev)
            else:
                x = W.token_matrix(spec, "lin", d, dev, width=shape[1])
            e = {"x": x, "kind": kind, "layout": layout, "q": torch.empty(x.numel(), dtype=torch.int8, device=dev)}
            if kind == "lin":
                K, N = spec.linears[int(name[3:])]
                e["K"], e["N"] = K, N
                e["dy"] = W.upstream_grad(spec, "dy_lin", (spec.tokens, N), dev, draw=d)
                e["dW"] = torch.empty((N, K), device=dev)
                e["db"] = torch.empty(N, device=dev)
            else:
                e["dy"] = W.upstream_grad(spec, {"softmax": "dy_attn", "gelu": "dy_gelu", "ln": "dy_ln"}[kind], shape, dev, draw=d)
                e["dx"] = torch.empty_like(e["dy"])
            if kind == "ln":
                e["mean"], e["rstd"] = W.layernorm_stats(x)
                e["dgamma"] = torch.empty(spec.dim, device=dev)
                e["dbeta"] = torch.empty(spec.dim, device=dev)
            self.t[name] = e
        if spec.linears:
            self.xhat = torch.empty_like(self.t["lin0"]["x"])


class Path:
    """The calls of a step, each a closure that only enqueues work."""

    def __init__(self, m, spec, number):
        self.m, self.spec, self.number = m, spec, number
        H = spec.heads
        self.nblocks = BLOCKS[number]
        self.nsets = self.nblocks if self.nblocks > 1 else NSETS
        self.sets = [Block(m, spec, number, d) for d in range(self.nsets)]
        self.names = [n for n, _, _, _ in saved_tensors(spec, number)]
        # running estimates belong to a layer: one pair per block of the step and saved tensor
        self.alpha = {(l, k): torch.zeros(H, device="cuda") for l in range(self.nblocks) for k in self.names}
        self.beta = {(l, k): torch.zeros(H, device="cuda") for l in range(self.nblocks) for k in self.names}
        self.gamma = W.layernorm_gamma(spec, "cuda")
        dtc = dtype_code(m, spec.dtype)
        s0 = self.sets[0]
        sizes = [m.workspace_bytes(m.OP_UPDATE_RUNNING_PARAMS, *e["layout"]) for e in s0.t.values()]
        sizes.append(m.workspace_bytes(m.OP_LAYERNORM_BWD_Q, spec.tokens, spec.dim, H))
        sizes += [m.workspace_bytes(m.OP_LINEAR_DW_Q, spec.tokens, K, N, dtc) for K, N in spec.linears]
        self.ws = torch.empty(max(sizes + [16]), dtype=torch.uint8, device="cuda")
        self.step_no = 0
        self.first = True

    def blocks_of_step(self, i):
        """(layer, forward buffers, backward buffers) for each block of step i, in forward order."""
        if self.nblocks > 1:
            return [(l, self.sets[l], self.sets[l]) for l in range(self.nblocks)]
        return [(0, self.sets[i % self.nsets], self.sets[(i - 1) % self.nsets])]

    def forward_calls(self, layer, blk, step, single_pass=False):
        m, spec = self.m, self.spec
        out = []
        for i, k in enumerate(self.names):
            e = blk.t[k]
            a, b = self.alpha[(layer, k)], self.beta[(layer, k)]
            off = (step << 30) + ((layer * 16 + i) << 44)
            if single_pass and not self.first:
                out.append((f"quantize_update_fused_{k}", lambda e=e, a=a, b=b, off=off: m.mesa_quantize_update_fused(
                    e["x"], e["layout"], a, b, spec.lam, e["q"], self.ws, m.ROUND_STOCHASTIC, 2024, off)))
                continue
            out.append((f"update_{k}", lambda e=e, a=a, b=b: m.mesa_update_running_params(
                e["x"], e["layout"], a, b, spec.lam, self.first, self.ws)))
            out.append((f"quantize_{k}", lambda e=e, a=a, b=b, off=off: m.mesa_quantize_headwise(
                e["x"], e["layout"], a, b, e["q"], m.ROUND_STOCHASTIC, 2024, off)))
        return out

    def backward_calls(self, layer, blk):
        m, spec, H = self.m, self.spec, self.spec.heads
        out = []
        par = lambda k: (self.alpha[(layer, k)], self.beta[(layer, k)])  # noqa: E731
        lins = [k for k in self.names if k.startswith("lin")]
        for k in reversed(lins):
            e = blk.t[k]
            a, b = par(k)
            out.append((f"linear_dw_q_{k}", lambda e=e, a=a, b=b: m.mesa_linear_dw_q(
                e["q"], spec.tokens, e["K"], H, a, b, e["dy"], e["N"], e["dW"], e["db"], self.ws)))
        if lins:
            e = blk.t["lin0"]
            a, b = par("lin0")
            out.append(("dequantize_lin0", lambda e=e, a=a, b=b: m.mesa_dequantize(e["q"], e["layout"], a, b, blk.xhat)))
        for k in reversed([k for k in self.names if k.startswith("ln")]):
            e = blk.t[k]
            a, b = par(k)
            out.append((f"layernorm_bwd_q_{k}", lambda e=e, a=a, b=b: m.mesa_layernorm_bwd_q(
                e["q"], spec.tokens, spec.dim, H, a, b, e["mean"], e["rstd"], self.gamma, e["dy"], e["dx"], e["dgamma"],
                e["dbeta"], self.ws)))
        e = blk.t["gelu"]
        a, b = par("gelu")
        out.append(("gelu_bwd_q", lambda e=e, a=a, b=b: m.mesa_gelu_bwd_q(e["q"], e["layout"], a, b, e["dy"], e["dx"])))
        B, Hh, rows, cols = spec.attn
        e = blk.t["attn"]
        a, b = par("attn")
        out.append(("softmax_bwd_q", lambda e=e, a=a, b=b: m.mesa_softmax_bwd_q(e["q"], B, Hh, rows, cols, a, b, e["dy"], e["dx"])))
        return out

    def calls(self, single_pass=False):
        """Every call of the next step, in launch order."""
        i = self.step_no
        blocks = self.blocks_of_step(i)
        out = []
        for layer, fwd, _ in blocks:
            out += self.forward_calls(layer, fwd, i, single_pass)
        for layer, _, bwd in reversed(blocks):
            out += self.backward_calls(layer, bwd)
        return out

    def step(self, timed_call=None, events=None, single_pass=False, every_call=None, event_pool=None):
        # event_pool: events created beforehand (creating one costs the host far more than a launch)
        for name, fn in self.calls(single_pass):
            if every_call is not None or name == timed_call:
                e0, e1 = (event_pool.pop(), event_pool.pop()) if event_pool else (self.m.Event(), self.m.Event())
                e0.record()
                fn()
                e1.record()
                (every_call if every_call is not None else events).append((name, e0, e1))
            else:
                fn()
        self.step_no += 1
        self.first = False


def cpu_baseline(spec, number, threads_note=True):
    """The oracle as it stands, timed on the host cores over a bounded sample of the same workload: one block's calls on
    a few samples of the batch (every block of the step repeats the same calls), all cores, then one thread."""
    import ctypes
    import numpy as np
    from oracle import mesa_ref as R
    R.lib()

    def one_pass(s, tensors, seed):
        H = s.heads
        q, a, b = {}, {}, {}
        for k, e in tensors.items():
            a[k], b[k] = R.update_running_params(e["x"], e["layout"], np.zeros(H), np.zeros(H), s.lam, True)
            q[k] = R.quantize_headwise(e["x"], e["layout"], a[k], b[k], R.ROUND_STOCHASTIC, 2024, seed)
        for k, e in tensors.items():
            if e["kind"] == "lin":
                R.linear_dw_q(q[k], s.tokens, e["K"], H, a[k], b[k], e["dy"], e["N"])
            elif e["kind"] == "ln":
                R.layernorm_bwd_q(q[k], s.tokens, s.dim, H, a[k], b[k], e["mean"], e["rstd"], e["gamma"], e["dy"])
            elif e["kind"] == "gelu":
                R.gelu_bwd_q(q[k], e["layout"], a[k], b[k], e["dy"])
            else:
                Bq, Hq, r, c = s.attn
                R.softmax_bwd_q(q[k], Bq, Hq, r, c, a[k], b[k], e["dy"])
        if "lin0" in tensors:
            e = tensors["lin0"]
            R.dequantize(q["lin0"], e["layout"], a["lin0"], b["lin0"], np.float16 if s.dtype != torch.float32 else np.float32)

    def host_tensors(s):
        out = {}
        gamma = W.layernorm_gamma(s).numpy()
        for i, (name, kind, layout, shape) in enumerate(saved_tensors(s, number)):
            if kind == "softmax":
                x = W.attention_map(s, i)
            elif kind == "gelu":
                x = W.gelu_input(s, i)
            elif kind == "ln":
                x = W.token_matrix(s, "ln", i)
            else:
                x = W.token_matrix(s, "lin", i, width=shape[1])
            e = {"x": x.numpy(), "kind": kind, "layout": layout}
            if kind == "lin":
                K, N = s.linears[int(name[3:])]
                e["K"], e["N"] = K, N
                e["dy"] = W.upstream_grad(s, "dy_lin", (s.tokens, N)).numpy()
            else:
                e["dy"] = W.upstream_grad(s, {"softmax": "dy_attn", "gelu": "dy_gelu", "ln": "dy_ln"}[kind], shape).numpy()
            if kind == "ln":
                mean, rstd = W.layernorm_stats(x)
                e["mean"], e["rstd"], e["gamma"] = mean.numpy(), rstd.numpy(), gamma
            out[name] = e
        return out

    def timed(s, budget):
        tensors = host_tensors(s)
        t0 = time.perf_counter()
        passes = 0
        while True:
            one_pass(s, tensors, passes)
            passes += 1
            el = time.perf_counter() - t0
            if el > budget:
                break
        return sum(algorithmic_bytes(s, number).values()) * passes / el / 1e9, passes, el

    batch = spec.attn[0]
    # sample sizes: the fp64 weight gradient of the oracle sets the pace (a few GFLOP per sample of the batch)
    keep_all = {2: 8, 3: 256, 4: 2, 5: 1}[number]
    s_all = W.scaled(spec, max(1, batch // keep_all))
    cores = R.num_threads()
    v_all, p_all, el_all = timed(s_all, 8.0)
    out = {"value": round(v_all, 4), "unit": "GB/s", "cores": cores, "kind": "oracle",
           "sample": f"{p_all} pass(es) of one block's calls (update, quantize, every backward) over {s_all.attn[0]} of the "
                     f"{batch} batch entries, {s_all.tokens} tokens ({el_all:.1f} s of CPU work on {cores} threads; same "
                     f"algorithmic-byte accounting as the GPU figure; the step repeats these calls for each of its blocks)"}
    try:
        gomp = ctypes.CDLL("libgomp.so.1")
        gomp.omp_set_num_threads(1)
        s_one = W.scaled(spec, batch) if number != 3 else W.scaled(spec, batch // 32)
        v1, p1, el1 = timed(s_one, 4.0)
        gomp.omp_set_num_threads(cores)
        out["one_thread"] = {"value": round(v1, 4), "unit": "GB/s", "cores": 1,
                             "sample": f"{p1} pass(es) over {s_one.attn[0]} batch entr{'y' if s_one.attn[0] == 1 else 'ies'} ({el1:.1f} s)"}
    except OSError:
        pass
    return out


def timed_leg(fn, steps, warm=3):
    """median of `steps` event pairs around fn(i), in ms"""
    import paper_2111_11124_amd as m
    for i in range(warm):
        fn(i)
    torch.cuda.synchronize()
    evs = []
    for i in range(steps):
        e0, e1 = m.Event(), m.Event()
        e0.record()
        fn(i)
        e1.record()
        evs.append((e0, e1))
    torch.cuda.synchronize()
    return statistics.median(e0.elapsed_ms(e1) for e0, e1 in evs)


LEG_SETS = 6   # buffer sets the extra legs rotate over, enough to exceed twice the memory-side cache between reuses


def attention_matmul_leg(m, spec, steps):
    """Outside the headline figure: backward of the two attention matrix products at head-wise codes
    (mesa_attn_av_bwd_q, mesa_attn_qk_bwd_q) on the configuration's attention shape, synthetic codes."""
    if spec.dtype == torch.float32:
        return None
    B, H, N, _ = spec.attn
    Dh = spec.dim // spec.heads
    dev = "cuda"
    g = torch.Generator(device=dev).manual_seed(spec.seed)
    n2, nd = B * H * N * N, B * H * N * Dh
    nbytes = (n2 + nd + 2 * nd + 2 * n2 + 2 * nd) + (2 * nd + 2 * n2 + 4 * nd)
    nsets = max(3, min(LEG_SETS, int(math.ceil(600e6 / nbytes)) + 1))
    sets = []
    for _ in range(nsets):
        sets.append({
            "a": torch.randint(-128, 128, (B, H, N, N), dtype=torch.int8, device=dev, generator=g),
            "qkv": [torch.randint(-128, 128, (B, H, N, Dh), dtype=torch.int8, device=dev, generator=g) for _ in range(3)],
            "dO": torch.randn((B, H, N, Dh), device=dev, generator=g).to(spec.dtype),
            "dS": torch.randn((B, H, N, N), device=dev, generator=g).to(spec.dtype),
            "dA": torch.empty((B, H, N, N), dtype=spec.dtype, device=dev),
            "d3": [torch.empty((B, H, N, Dh), dtype=spec.dtype, device=dev) for _ in range(3)],
        })
    al = torch.full((H,), 3.0, device=dev)
    be = torch.full((H,), -1.5, device=dev)

    def run(i):
        t = sets[i % nsets]
        m.mesa_attn_av_bwd_q(t["a"], t["qkv"][2], B, H, N, Dh, al, be, al, be, t["dO"], t["dA"], t["d3"][2])
        m.mesa_attn_qk_bwd_q(t["qkv"][0], t["qkv"][1], B, H, N, Dh, al, be, al, be, t["dS"], Dh ** -0.5, t["d3"][0], t["d3"][1])

    ms = timed_leg(run, steps)
    flops = 4 * 2.0 * B * H * N * N * Dh
    return {"ms": round(ms, 4), "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1), "frac_hbm": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "tflops": round(flops / (ms * 1e-3) / 1e12, 1), "bytes": nbytes, "shape": [B, H, N, Dh], "buffer_sets": nsets,
            "note": "the four products dA, dV, dQ, dK of one block (two calls), median of event pairs; HBM-bound: codes, upstream "
                    "gradients and results each moved once"}


def layer_forward_legs(m, spec, steps):
    """Outside the headline figure: the three layer forwards in one pass (output and codes from one read of the input),
    each next to the two passes it replaces (the framework's own kernel followed by mesa_quantize_update_fused)."""
    dev = "cuda"
    dtc = dtype_code(m, spec.dtype)
    esz = elem_bytes(spec.dtype)
    out = {}

    def sets_for(nbytes):
        return max(3, min(LEG_SETS, int(math.ceil(600e6 / nbytes)) + 1))

    def entry(one, two, nbytes, nsets, note):
        return {"ms": round(one, 4), "GBps": round(nbytes / (one * 1e-3) / 1e9, 1),
                "frac_hbm": round(nbytes / (one * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "bytes": nbytes, "two_pass_ms": round(two, 4),
                "buffer_sets": nsets, "note": note}

    # GELU
    lay = spec.gelu_layout
    n = lay[0] * lay[1] * lay[2]
    nbytes = (2 * esz + 1) * n
    ns = sets_for(nbytes)
    g = torch.Generator(device=dev).manual_seed(spec.seed + 3)
    xs = [torch.randn(lay, device=dev, generator=g).to(spec.dtype) for _ in range(ns)]
    ys = [torch.empty(lay, dtype=spec.dtype, device=dev) for _ in range(ns)]
    qs = [torch.empty(n, dtype=torch.int8, device=dev) for _ in range(ns)]
    a = torch.full((lay[1],), 8.0, device=dev)
    b = torch.full((lay[1],), -4.0, device=dev)
    ws = torch.empty(max(m.workspace_bytes(m.OP_UPDATE_RUNNING_PARAMS, *lay, dtc), 16), dtype=torch.uint8, device=dev)
    one = timed_leg(lambda i: m.mesa_gelu_fwd_q(xs[i % ns], lay, a, b, 0.9, ys[i % ns], qs[i % ns], ws, m.ROUND_STOCHASTIC, 1, i), steps)
    two = timed_leg(lambda i: (torch.nn.functional.gelu(xs[i % ns]),
                               m.mesa_quantize_update_fused(xs[i % ns], lay, a, b, 0.9, qs[i % ns], ws, m.ROUND_STOCHASTIC, 1, i)), steps)
    out["gelu_layer_forward"] = entry(one, two, nbytes, ns, "mesa_gelu_fwd_q; two_pass_ms: the framework's own exact GELU kernel "
                                      "followed by mesa_quantize_update_fused")
    del xs, ys, qs

    # softmax
    B, H, r, c = spec.attn
    n = B * H * r * c
    wsn = m.workspace_bytes(m.OP_SOFTMAX_FWD_Q, B * H * r, H, c, dtc)
    if wsn > 16 and B * H * r < 2 ** 31:
        lay = (B, H, r * c)
        nbytes = (2 * esz + 1) * n
        ns = sets_for(nbytes)
        g = torch.Generator(device=dev).manual_seed(spec.seed + 4)
        ss = [W._randn((B, H, r, c), g, spec.dtype, dev) for _ in range(ns)]
        ys = [torch.empty((B, H, r, c), dtype=spec.dtype, device=dev) for _ in range(ns)]
        qs = [torch.empty(n, dtype=torch.int8, device=dev) for _ in range(ns)]
        a = torch.full((H,), 0.8, device=dev)
        b = torch.zeros(H, device=dev)
        ws = torch.empty(wsn, dtype=torch.uint8, device=dev)
        ws2 = torch.empty(max(m.workspace_bytes(m.OP_UPDATE_RUNNING_PARAMS, *lay, dtc), 16), dtype=torch.uint8, device=dev)
        one = timed_leg(lambda i: m.mesa_softmax_fwd_q(ss[i % ns], B, H, r, c, a, b, 0.9, ys[i % ns], qs[i % ns], ws, m.ROUND_STOCHASTIC, 1, i), steps)

        def two_pass(i):
            yy = torch.softmax(ss[i % ns], dim=-1)
            m.mesa_quantize_update_fused(yy, lay, a, b, 0.9, qs[i % ns], ws2, m.ROUND_STOCHASTIC, 1, i)

        two = timed_leg(two_pass, steps)
        out["softmax_layer_forward"] = entry(one, two, nbytes, ns, "mesa_softmax_fwd_q; two_pass_ms: the framework's own softmax kernel "
                                             "followed by mesa_quantize_update_fused")
        del ss, ys, qs
    else:
        out["softmax_layer_forward"] = None

    # LayerNorm
    M_, D, G = spec.tokens, spec.dim, spec.heads
    if m.workspace_bytes(m.OP_LAYERNORM_FWD_Q, M_, D, G, dtc) > 16 and (D // G) % 8 == 0:
        n = M_ * D
        lay = (M_, G, D // G)
        nbytes = (2 * esz + 1) * n + 8 * M_
        ns = sets_for(nbytes)
        g = torch.Generator(device=dev).manual_seed(spec.seed + 5)
        xs = [torch.randn((M_, D), device=dev, generator=g).to(spec.dtype) for _ in range(ns)]
        ys = [torch.empty((M_, D), dtype=spec.dtype, device=dev) for _ in range(ns)]
        qs = [torch.empty(n, dtype=torch.int8, device=dev) for _ in range(ns)]
        mean = torch.empty(M_, device=dev)
        rstd = torch.empty(M_, device=dev)
        gamma = torch.ones(D, device=dev).to(spec.dtype)
        bias = torch.zeros(D, device=dev).to(spec.dtype)
        a = torch.full((G,), 8.0, device=dev)
        b = torch.full((G,), -4.0, device=dev)
        ws = torch.empty(m.workspace_bytes(m.OP_LAYERNORM_FWD_Q, M_, D, G, dtc), dtype=torch.uint8, device=dev)
        ws2 = torch.empty(max(m.workspace_bytes(m.OP_UPDATE_RUNNING_PARAMS, *lay, dtc), 16), dtype=torch.uint8, device=dev)
        one = timed_leg(lambda i: m.mesa_layernorm_fwd_q(xs[i % ns], M_, D, G, gamma, bias, 1e-5, a, b, 0.9, ys[i % ns], mean, rstd,
                                                         qs[i % ns], ws, m.ROUND_STOCHASTIC, 1, i), steps)
        two = timed_leg(lambda i: (torch.nn.functional.layer_norm(xs[i % ns], (D,), gamma, bias, 1e-5),
                                   m.mesa_quantize_update_fused(xs[i % ns], lay, a, b, 0.9, qs[i % ns], ws2, m.ROUND_STOCHASTIC, 1, i)), steps)
        out["layernorm_layer_forward"] = entry(one, two, nbytes, ns, "mesa_layernorm_fwd_q; two_pass_ms: the framework's own layer_norm "
                                               "kernel followed by mesa_quantize_update_fused")
    else:
        out["layernorm_layer_forward"] = None
    return out


def symmetric_leg(m, spec, steps):
    """Outside the headline figure: the forward half (statistics + quantize) of the scale-only symmetric scheme the paper's
    ablation compares with (Sec. 5.2), next to the method's asymmetric forward, on the configuration's GELU input."""
    lay = spec.gelu_layout
    n = lay[0] * lay[1] * lay[2]
    dev = "cuda"
    esz = elem_bytes(spec.dtype)
    nbytes = (2 * esz + 1) * n
    ns = max(3, min(LEG_SETS, int(math.ceil(600e6 / nbytes)) + 1))
    g = torch.Generator(device=dev).manual_seed(spec.seed + 6)
    xs = [W._randn(lay, g, spec.dtype, dev) for _ in range(ns)]
    qs = [torch.empty(n, dtype=torch.int8, device=dev) for _ in range(ns)]
    a = torch.zeros(lay[1], device=dev)
    b = torch.zeros(lay[1], device=dev)
    mm = torch.zeros(lay[1], device=dev)
    ws = torch.empty(max(m.workspace_bytes(m.OP_UPDATE_RUNNING_PARAMS, *lay, dtype_code(m, spec.dtype)), 16), dtype=torch.uint8, device=dev)
    m.mesa_update_running_params(xs[0], lay, a, b, 0.9, True, ws)
    m.mesa_update_running_scale_sym(xs[0], lay, mm, 0.9, True, ws)
    asym = timed_leg(lambda i: (m.mesa_update_running_params(xs[i % ns], lay, a, b, 0.9, False, ws),
                                m.mesa_quantize_headwise(xs[i % ns], lay, a, b, qs[i % ns], m.ROUND_STOCHASTIC, 1, i)), steps)
    sym = timed_leg(lambda i: (m.mesa_update_running_scale_sym(xs[i % ns], lay, mm, 0.9, False, ws),
                               m.mesa_quantize_sym(xs[i % ns], lay, mm, qs[i % ns], m.ROUND_STOCHASTIC, 1, i)), steps)
    return {"symmetric_ms": round(sym, 4), "asymmetric_ms": round(asym, 4), "bytes": nbytes,
            "symmetric_GBps": round(nbytes / (sym * 1e-3) / 1e9, 1), "asymmetric_GBps": round(nbytes / (asym * 1e-3) / 1e9, 1),
            "note": "update + quantize of the GELU input, stochastic rounding: mesa_update_running_scale_sym + mesa_quantize_sym "
                    "against mesa_update_running_params + mesa_quantize_headwise; both read x twice and write one byte per element"}


def four_bit_leg(m, spec, steps):
    """Outside the headline figure: the lower bit width that Sec. 4.2 discusses, on the configuration's GELU input --
    quantize to four-bit codes (two per byte) and GELU backward from them, next to the eight-bit calls."""
    lay = spec.gelu_layout
    n = lay[0] * lay[1] * lay[2]
    dev = "cuda"
    esz = elem_bytes(spec.dtype)
    ns = max(3, min(LEG_SETS, int(math.ceil(600e6 / ((2 * esz + 1) * n))) + 1))
    g = torch.Generator(device=dev).manual_seed(spec.seed + 7)
    xs = [W._randn(lay, g, spec.dtype, dev) for _ in range(ns)]
    dys = [W._randn(lay, g, spec.dtype, dev) for _ in range(ns)]
    q8 = [torch.empty(n, dtype=torch.int8, device=dev) for _ in range(ns)]
    q4 = [torch.empty((n + 1) // 2, dtype=torch.uint8, device=dev) for _ in range(ns)]
    a = torch.zeros(lay[1], device=dev)
    b = torch.zeros(lay[1], device=dev)
    ws = torch.empty(max(m.workspace_bytes(m.OP_UPDATE_RUNNING_PARAMS, *lay, dtype_code(m, spec.dtype)), 16), dtype=torch.uint8, device=dev)
    m.mesa_update_running_params(xs[0], lay, a, b, 0.9, True, ws)
    for k in range(ns):
        m.mesa_quantize_headwise(xs[k], lay, a, b, q8[k], m.ROUND_STOCHASTIC, 1, k)
        m.mesa_quantize_headwise_b4(xs[k], lay, a, b, q4[k], m.ROUND_STOCHASTIC, 1, k)
    t = {"quantize_b8": timed_leg(lambda i: m.mesa_quantize_headwise(xs[i % ns], lay, a, b, q8[i % ns], m.ROUND_STOCHASTIC, 1, i), steps),
         "quantize_b4": timed_leg(lambda i: m.mesa_quantize_headwise_b4(xs[i % ns], lay, a, b, q4[i % ns], m.ROUND_STOCHASTIC, 1, i), steps),
         "gelu_bwd_b8": timed_leg(lambda i: m.mesa_gelu_bwd_q(q8[i % ns], lay, a, b, dys[i % ns], dys[i % ns]), steps),
         "gelu_bwd_b4": timed_leg(lambda i: m.mesa_gelu_bwd_q_b4(q4[i % ns], lay, a, b, dys[i % ns], dys[i % ns]), steps)}
    nb = {"quantize_b8": (esz + 1) * n, "quantize_b4": esz * n + (n + 1) // 2,
          "gelu_bwd_b8": (2 * esz + 1) * n, "gelu_bwd_b4": 2 * esz * n + (n + 1) // 2}
    return {k: {"ms": round(v, 5), "bytes": nb[k], "GBps": round(nb[k] / (v * 1e-3) / 1e9, 1),
                "frac_hbm": round(nb[k] / (v * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)} for k, v in t.items()}


CONV_SHAPES = [  # B, C_in, H, W, C_out, KH, KW, pad: the 3x3 and 1x1 convolutions of a segmentation head on 128 x 128 feature maps
    ("3x3 512->512", (2, 512, 128, 128, 512, 3, 3, 1)),
    ("1x1 2048->512", (2, 2048, 128, 128, 512, 1, 1, 0)),
    # the 3x3 convolutions of an image classifier's four stages, batch 16: maps of 56, 28, 14 and 7 columns (widths that
    # are a multiple of eight, no multiple of eight, and below eight: the kernel's three ways of staging a row)
    ("3x3 64->64 @56", (16, 64, 56, 56, 64, 3, 3, 1)),
    ("3x3 128->128 @28", (16, 128, 28, 28, 128, 3, 3, 1)),
    ("3x3 256->256 @14", (16, 256, 14, 14, 256, 3, 3, 1)),
    ("3x3 512->512 @7", (16, 512, 7, 7, 512, 3, 3, 1)),
]


def conv_dw_leg(m, spec, steps):
    """Outside the headline figure: the weight gradient of a convolution at group-wise codes (Sec. 3.3), on the shapes of
    a segmentation head (batch 2 per GPU, 128 x 128 feature maps) and of an image classifier's stages (batch 16), with the
    vendor library's convolution weight gradient on the de-quantized 16-bit input beside it."""
    dev = "cuda"
    out = {}
    dtc = dtype_code(m, spec.dtype)
    for name, (B, Cin, H, Wd, Cout, KH, KW, pad) in CONV_SHAPES:
        cv = m.Conv2d(B, Cin, H, Wd, Cout, KH, KW, 1, 1, pad, pad, 1, 1)
        OH, OW = cv.out_hw()
        G = 8
        g = torch.Generator(device=dev).manual_seed(spec.seed + Cin + KH)
        xq = [torch.randint(-128, 128, (B, Cin, H, Wd), dtype=torch.int8, device=dev, generator=g) for _ in range(3)]
        dy = [W._randn((B, Cout, OH, OW), g, spec.dtype, dev) for _ in range(3)]
        a = torch.full((G,), 8.0, device=dev)
        b = torch.full((G,), -4.0, device=dev)
        dW = torch.empty((Cout, Cin, KH, KW), device=dev)
        db = torch.empty(Cout, device=dev)
        ws = torch.empty(max(m.conv2d_dw_q_workspace_bytes(cv, dtc), 16), dtype=torch.uint8, device=dev)
        ms = timed_leg(lambda i: m.mesa_conv2d_dw_q(xq[i % 3], cv, G, a, b, dy[i % 3], dW, db, ws), steps)
        fl = 2.0 * B * OH * OW * Cin * Cout * KH * KW
        entry = {"ms": round(ms, 5), "tflops": round(fl / (ms * 1e-3) / 1e12, 1),
                 "mfma_frac": round(fl / (ms * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS, 4),
                 "shape": [B, Cin, H, Wd, Cout, KH, KW], "workspace_bytes": int(ws.numel())}
        xh = [torch.empty((B, Cin, H, Wd), dtype=spec.dtype, device=dev) for _ in range(3)]
        for k in range(3):
            m.mesa_dequantize(xq[k].view(-1), (B, G, (Cin // G) * H * Wd), a, b, xh[k])
        lib_ms = timed_leg(lambda i: torch.nn.grad.conv2d_weight(xh[i % 3], (Cout, Cin, KH, KW), dy[i % 3], padding=pad), steps)
        entry["library_conv_16bit_operands"] = {"ms": round(lib_ms, 5), "tflops": round(fl / (lib_ms * 1e-3) / 1e12, 1)}
        out[name] = entry
        del xq, dy, xh
    return out


def bandwidth_probes(m):
    """Untimed extras: what plain kernels reach on this GPU -- a copy (the known-traffic kernel the bandwidth counters are
    scaled against), a read-only and a write-only stream, 256 MiB each, three rotating buffers, median of event pairs."""
    n = 256 << 20
    src = [torch.empty(n, dtype=torch.uint8, device="cuda") for _ in range(3)]
    dst = [torch.empty(n, dtype=torch.uint8, device="cuda") for _ in range(3)]
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    out = {}
    for name, fn, nbytes in (("copy_probe", lambda i: m.mesa_stream_copy(src[i % 3], dst[i % 3], n), 2 * n),
                             ("read_probe", lambda i: m.mesa_stream_read(src[i % 3], n, sink), n),
                             ("write_probe", lambda i: m.mesa_stream_fill(dst[i % 3], n, 0), n)):
        ms = timed_leg(fn, 12, warm=2)
        out[name] = {"bytes": nbytes, "ms": round(ms, 5), "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1)}
    out["copy_probe"]["note"] = "mesa_stream_copy, 256 MiB read + 256 MiB written: the bandwidth a plain copy reaches on this GPU"
    out["read_probe"]["note"] = "mesa_stream_read, 256 MiB read, nothing written"
    out["write_probe"]["note"] = "mesa_stream_fill, 256 MiB written, nothing read"
    return out


def mfma_probes(m):
    """Untimed extras: the rate at which this GPU sustains the weight gradient's matrix-core instruction stream with the
    operands in registers, read from LDS, and with the tile's operand movement beside it (mesa_mfma_probe; one workgroup
    of four waves per CU, 640 contraction steps a launch).  `first_launches` is the median of the first 10 launches after
    an idle second, `sustained` the median of launches 200..299 of an unbroken sequence (the power limit has set in)."""
    steps = 640
    flops = m.MFMA_PROBE_WAVES * steps * m.MFMA_PROBE_FLOPS_PER_STEP
    sink = torch.empty(65536, dtype=torch.float32, device="cuda")
    gen = torch.Generator(device="cuda").manual_seed(77)
    feed = torch.randn(8 << 20, device="cuda", generator=gen).half()        # 16 MiB: 2 MiB per XCD, within its L2
    out = {}
    for form, name in ((0, "operands_in_registers"), (1, "operands_from_lds"), (2, "operands_from_lds_and_tile_loads"),
                       (3, "eight_waves_operands_from_lds_and_tile_loads")):
        torch.cuda.synchronize()
        time.sleep(1.0)
        evs = []
        for i in range(300):
            e0, e1 = m.Event(), m.Event()
            e0.record()
            m.mesa_mfma_probe(form, steps, feed if form >= 2 else None, sink)
            e1.record()
            evs.append((e0, e1))
        torch.cuda.synchronize()
        ms = [a.elapsed_ms(b) for a, b in evs]
        first, sust = statistics.median(ms[:10]), statistics.median(ms[200:])
        out[name] = {"first_launches": {"ms": round(first, 5), "tflops": round(flops / (first * 1e-3) / 1e12, 1)},
                     "sustained": {"ms": round(sust, 5), "tflops": round(flops / (sust * 1e-3) / 1e12, 1),
                                   "mfma_frac": round(flops / (sust * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS, 4)}}
    out["note"] = ("v_mfma_f32_32x32x16_f16 on 128 x 128 accumulator tiles per wave, pseudo-random binary16 operands; "
                   f"{flops / 1e9:.1f} GFLOP per launch; the ceiling the weight gradient's `mfma_frac` is to be read against")
    return {"mfma_probe": out}


def traffic_from_profile(spec, call):
    """HBM bytes per launch of the kernel behind `call`, from the rocprofv3 --pmc summary committed for this workload
    (FETCH_SIZE / WRITE_SIZE scaled by the copy kernel's reading); None when no summary covers it."""
    path = os.path.join(ROOT, "profiles", f"bench_step_{spec.name}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None, None
    pat = re.compile(r"^call=(\S+)\s+kernel=(\S+)\s+traffic_bytes=(\d+)")
    for line in open(path):
        mo = pat.match(line.strip())
        if mo and mo.group(1) == call:
            return int(mo.group(3)), os.path.relpath(path, ROOT)
    return None, None


def dw_only(m, spec, steps):
    """--only-dw: the configuration's weight-gradient calls alone, launched back to back over three rotating buffer sets
    (the sustained rate, and the launch sequence the per-kernel counter summaries in profiles/ are taken on)."""
    dev = "cuda"
    H = spec.heads
    out = {}
    dtc = dtype_code(m, spec.dtype)
    for K, N in spec.linears:
        g = torch.Generator(device=dev).manual_seed(spec.seed + K + N)
        qs = [torch.randint(-128, 128, (spec.tokens, K), dtype=torch.int8, device=dev, generator=g) for _ in range(3)]
        dys = [W._randn((spec.tokens, N), g, spec.dtype, dev) for _ in range(3)]
        a = torch.full((H,), 8.0, device=dev)
        b = torch.full((H,), -4.0, device=dev)
        dW = torch.empty((N, K), device=dev)
        db = torch.empty(N, device=dev)
        ws = torch.empty(m.workspace_bytes(m.OP_LINEAR_DW_Q, spec.tokens, K, N, dtc), dtype=torch.uint8, device=dev)
        ms = timed_leg(lambda i: m.mesa_linear_dw_q(qs[i % 3], spec.tokens, K, H, a, b, dys[i % 3], N, dW, db, ws), steps)
        fl = 2.0 * spec.tokens * K * N
        out[f"{K}->{N}"] = {"ms": round(ms, 5), "tflops": round(fl / (ms * 1e-3) / 1e12, 1),
                            "mfma_frac": round(fl / (ms * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS, 4), "shape": [spec.tokens, K, N]}
        # context, not part of the path: the vendor library's GEMM (through torch.matmul) on the same shape with the
        # activation already de-quantized to 16-bit floats in memory -- what this GPU sustains on this contraction without
        # the conversion of the codes in the loop
        xh = [torch.empty((spec.tokens, K), dtype=spec.dtype, device=dev) for _ in range(3)]
        for k in range(3):
            m.mesa_dequantize(qs[k].view(-1), (spec.tokens, H, K // H), a, b, xh[k])
        lib_out = torch.empty((N, K), dtype=spec.dtype, device=dev)
        lib_ms = timed_leg(lambda i: torch.matmul(dys[i % 3].t(), xh[i % 3], out=lib_out), steps)
        out[f"{K}->{N}"]["library_gemm_16bit_operands"] = {"ms": round(lib_ms, 5), "tflops": round(fl / (lib_ms * 1e-3) / 1e12, 1),
                                                          "mfma_frac": round(fl / (lib_ms * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS, 4)}
        del qs, dys, xh, lib_out
    return out


def workload_name(spec, number, nblocks):
    b, h, r, c = spec.attn
    lins = ", ".join(f"{k}->{n}" for k, n in spec.linears) if spec.linears else "no Linear layer named"
    what = f"{nblocks} consecutive blocks (distinct buffers and running estimates), summed" if nblocks > 1 else "one block"
    return (f"configs[{number - 1}]: {spec.name} -- {what}; attention maps ({b}, {h}, {r}, {c}), {spec.tokens} tokens, dim {spec.dim}, "
            f"MLP {spec.mlp}, {DTYPE_NAME[spec.dtype]}; stochastic rounding; dW of {lins}")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the legs outside the headline (layer forwards, attention products, "
                                                             "single-pass variant, probes)")
    ap.add_argument("--only-dw", action="store_true", help="run only the configuration's weight-gradient calls, back to back, and "
                                                           "print their figures (a measurement helper, not the benchmark line)")
    ap.add_argument("--only-leg", default=None, choices=["attention", "conv", "four_bit", "symmetric", "layer_forwards", "mfma_probe"],
                    help="run one of the legs outside the headline alone and print its figures (a measurement helper: the "
                         "launch sequence the per-kernel counter summaries in profiles/ are taken on)")
    ap.add_argument("--config", type=int, default=HEADLINE_CONFIG, choices=[2, 3, 4, 5],
                    help="which of the baseline configurations to run; the default (4) is the whole-model one, twelve blocks per "
                         "step; 2, 3 and 5 are single blocks")
    ap.add_argument("--storage", default="f16", choices=["f16", "bf16"],
                    help="storage type of activations and gradients: f16 (the paper's mixed precision, the headline) or bf16")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)

    import paper_2111_11124_amd as m
    m.lib()
    number = args.config
    spec = W.CONFIGS[number]
    if args.storage == "bf16":
        spec = dataclasses.replace(spec, dtype=torch.bfloat16)
    if args.only_dw:
        print(json.dumps({"only_dw": dw_only(m, spec, args.steps or 20), "config": spec.name,
                          "note": "weight gradients launched back to back: the sustained rate, below what the same calls reach "
                                  "between the memory-bound kernels of a whole step"}))
        return
    if args.only_leg:
        leg = {"attention": attention_matmul_leg, "conv": conv_dw_leg, "four_bit": four_bit_leg, "symmetric": symmetric_leg,
               "layer_forwards": layer_forward_legs, "mfma_probe": lambda m, spec, steps: mfma_probes(m)}[args.only_leg]
        print(json.dumps({"only_leg": args.only_leg, "config": spec.name, "result": leg(m, spec, args.steps or 20)}))
        return
    nblocks = BLOCKS[number]
    steps = args.steps if args.steps is not None else (30 if nblocks > 1 else 50)
    warmup = args.warmup if args.warmup is not None else (3 if nblocks > 1 else 10)
    bytes_per = algorithmic_bytes(spec, number)          # one block
    total_bytes = sum(bytes_per.values()) * nblocks      # one step
    path = Path(m, spec, number)
    torch.cuda.synchronize()

    # untimed: warm-up steps, the first of which initialises the running estimates
    for _ in range(max(warmup, 2)):
        path.step()
    torch.cuda.synchronize()

    # untimed: profiling steps with an event pair around every call; per call the median over >= 20 pairs
    per_call = {}
    prof_steps = max(2, int(math.ceil(20 / nblocks)))
    for _ in range(prof_steps):
        evs = []
        path.step(every_call=evs)
        torch.cuda.synchronize()
        for name, e0, e1 in evs:
            per_call.setdefault(name, []).append(e0.elapsed_ms(e1))
    per_call_ms = {k: statistics.median(v) for k, v in per_call.items()}
    hbm_calls = [k for k in per_call_ms if not k.startswith("linear_dw_q")]
    dominant = max(hbm_calls, key=lambda k: per_call_ms[k] * len(per_call[k]))

    # timed region: exactly `steps` steps between two synchronisations; an event pair around every step and around
    # every launch of the dominant HBM-bound call
    events, step_events = [], []
    # every event of the timed region exists before it starts, so that a short step is not timed at the host's pace
    pool = [m.Event() for _ in range(steps * (2 + 2 * len(per_call[dominant]) // prof_steps) + 16)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        s0, s1 = pool.pop(), pool.pop()
        s0.record()
        path.step(timed_call=dominant, events=events, event_pool=pool)
        s1.record()
        step_events.append((s0, s1))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    ms_step_median = statistics.median(a.elapsed_ms(b) for a, b in step_events)
    dom_ms = sum(e0.elapsed_ms(e1) for _, e0, e1 in events) / len(events)

    value = total_bytes / (ms_per_step * 1e-3) / 1e9
    achieved = bytes_per[dominant] / (dom_ms * 1e-3) / 1e9
    traffic, traffic_src = traffic_from_profile(spec, dominant)
    n_elems = sum(e["x"].numel() for e in path.sets[0].t.values()) * nblocks
    hbm_bytes = sum(bytes_per[k] for k in hbm_calls)
    hbm_ms = sum(per_call_ms[k] for k in hbm_calls)
    dw = {}
    for i, (K, N) in enumerate(spec.linears):
        ms = per_call_ms[f"linear_dw_q_lin{i}"]
        fl = 2.0 * spec.tokens * K * N
        dw[f"{K}->{N}"] = {"tflops": round(fl / (ms * 1e-3) / 1e12, 1), "mfma_frac": round(fl / (ms * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS, 4),
                           "ms": round(ms, 5), "shape": [spec.tokens, K, N],
                           "hbm_frac": round(bytes_per[f"linear_dw_q_lin{i}"] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    if dw:
        fl = sum(2.0 * spec.tokens * K * N for K, N in spec.linears)
        ms = sum(per_call_ms[f"linear_dw_q_lin{i}"] for i in range(len(spec.linears)))
        dw["all"] = {"tflops": round(fl / (ms * 1e-3) / 1e12, 1), "mfma_frac": round(fl / (ms * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS, 4),
                     "ms": round(ms, 5)}
    out = {
        "metric": "effective HBM GB/s (% of peak) for quantize + dequant-fused bwd; dW MFMA util",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "{0} storage, f32 arithmetic ({0} x {0} -> f32 MFMA for dW)".format(DTYPE_NAME[spec.dtype]), "data": "synthetic",
        "config": {"workload": workload_name(spec, number, nblocks), "blocks_per_step": nblocks,
                   "bytes_per_step": total_bytes, "elements_per_s": round(n_elems / (ms_per_step * 1e-3), 1)},
        "ms_per_step_median_of_event_pairs": round(ms_step_median, 4),
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "hbm_bound_calls": {"GBps": round(hbm_bytes / (hbm_ms * 1e-3) / 1e9, 1),
                            "frac_hbm": round(hbm_bytes / (hbm_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                            "note": "every call of a block except the weight gradients: algorithmic bytes / sum of the calls' "
                                    "median event-pair times"},
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": traffic_src,
                     "avg_launch_ms": round(dom_ms, 5), "launches_timed": len(events), "algorithmic_bytes": bytes_per[dominant]},
        "dw": dw or None,
        "per_call": {k: {"ms": round(v, 5), "GBps": round(bytes_per[k] / (v * 1e-3) / 1e9, 1),
                         "frac_hbm": round(bytes_per[k] / (v * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "samples": len(per_call[k])}
                     for k, v in per_call_ms.items()},
    }
    if not args.no_extras:
        # outside the headline figure: the same step with the single-pass forward variant (one call per tensor that
        # quantizes with the running estimates as they are and moves them afterwards), under its own byte accounting
        sp_steps = max(3, steps // 3)
        path.step(single_pass=True)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(sp_steps):
            path.step(single_pass=True)
        torch.cuda.synchronize()
        sp_ms = (time.perf_counter() - t2) * 1e3 / sp_steps
        esz = elem_bytes(spec.dtype)
        sp_bytes = total_bytes - esz * n_elems
        out["single_pass_forward"] = {"ms_per_step": round(sp_ms, 4), "GBps": round(sp_bytes / (sp_ms * 1e-3) / 1e9, 1),
                                      "bytes_per_step": sp_bytes,
                                      "note": "variant, not the headline: mesa_quantize_update_fused replaces update + quantize (x "
                                              "read once; parameters lag one step), the backward half unchanged"}
        del path
        torch.cuda.empty_cache()
        out.update(bandwidth_probes(m))
        out.update(mfma_probes(m))
        leg_steps = 20
        out["attention_matmul_bwd"] = attention_matmul_leg(m, spec, leg_steps if number != 5 else 5)
        out.update(layer_forward_legs(m, spec, leg_steps))
        out["symmetric_scale_only_forward"] = symmetric_leg(m, spec, leg_steps)
        out["four_bit_codes"] = four_bit_leg(m, spec, leg_steps)
        out["conv2d_dw_q"] = conv_dw_leg(m, spec, leg_steps)
    if not args.no_cpu_baseline and number in (2, HEADLINE_CONFIG):
        # the oracle reads binary16 or binary32 arrays: for bfloat16 runs it is timed on the binary16 workload (same bytes)
        out["cpu_baseline"] = cpu_baseline(dataclasses.replace(spec, dtype=torch.float16), number)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
