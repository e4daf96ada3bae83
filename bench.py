#!/usr/bin/env python3
"""Benchmark of the fused block-sparse SwiGLU MLP on one MI355X.

A step = one pass of the MLP of Eq. (1) (gate/up products, activation, down product; output written) through
the C ABI over one synthetic batch already resident in HBM.  Packing is done once before the timed region, like
loading a checkpoint.

Headline workload: the largest single-GPU configuration, the 405B-class layer (hidden 16384, intermediate 53248,
128x128 blocks, 95 % block sparsity, Zipf-skewed rows) at 2048 tokens; `value` is its effective TFLOP/s on stored
blocks.  The other configurations (single linear; 1B-shaped MLP at 1/16/128/2048 tokens; 3B-shaped sparsity sweep at
4096 tokens; 8B-shaped decode; 405B-class decode) are timed the same way and reported as compact rows under
"configs": prefill rows against the bf16 MFMA peak, decode rows as algorithmic HBM GB/s against the HBM peak.

Launch mode: the K steps are recorded once into a HIP graph (rotating weight copies) and replayed; `ms_per_step` is
the median of three timed replays of those K steps.  The same K calls issued eagerly from Python are reported beside
it ("eager").  If capture fails the eager figure is the headline and "launch" says so.

Cold-HBM protocol: every step uses a different copy of the packed block values (>= 768 MB in rotation), so no step
re-reads weights still sitting in the 256 MB last-level cache.

`roofline.traffic` is read at run time from the rocprofv3 counter summaries under profiles/ (lines starting with
"traffic_bytes"), keyed by workload, token count and kernel; null when no summary covers the timed kernel.
"""
from __future__ import annotations

import argparse
import ctypes as C
import glob
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # dense bf16 MFMA, MI355X
PEAK_HBM_GBS = 8000.0
HEADLINE = "llama405b_b128_s95_zipf"


def profile_traffic(workload: str, tokens: int, kernel: str):
    """HBM-side bytes per launch of `kernel` from the tracked counter summaries, or None.  A summary line reads
    traffic_bytes | <workload> | T=<tokens> | <kernel> | fetch=<bytes> | write=<bytes> | <file it came from>."""
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        for line in open(path):
            if not line.startswith("traffic_bytes"):
                continue
            f = [x.strip() for x in line.split("|")]
            if len(f) >= 6 and f[1] == workload and f[2] == "T=%d" % tokens and f[3] == kernel:
                return {"bytes": float(f[4].split("=")[1]) + float(f[5].split("=")[1]),
                        "source": os.path.relpath(path, ROOT)}
    return None


def short(name):
    return name.replace("llama", "")


def sig(x, n=4):
    return None if x is None else float("%.*g" % (n, x))


def hip_runtime():
    import torch  # noqa: F401  (loads the HIP runtime this process uses)

    for name in ("libamdhip64.so.7", "libamdhip64.so"):
        try:
            return C.CDLL(name)
        except OSError:
            continue
    raise RuntimeError("cannot open the HIP runtime")


class Events:
    """hipEvent_t triples recorded by blast_sparse_mlp_events on the launch stream."""

    def __init__(self, n_steps: int):
        self.hip = hip_runtime()
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [C.c_void_p]
        self.triples = []
        for _ in range(n_steps):
            arr = (C.c_void_p * 3)()
            for j in range(3):
                ev = C.c_void_p()
                assert self.hip.hipEventCreate(C.byref(ev)) == 0
                arr[j] = ev
            self.triples.append(arr)

    def elapsed(self, a, b) -> float:
        ms = C.c_float()
        assert self.hip.hipEventSynchronize(b) == 0
        assert self.hip.hipEventElapsedTime(C.byref(ms), a, b) == 0
        return float(ms.value)

    def destroy(self):
        self.hip.hipEventDestroy.argtypes = [C.c_void_p]
        for arr in self.triples:
            for j in range(3):
                self.hip.hipEventDestroy(arr[j])


def rotated_copies(p, n_copies):
    """Same structure, distinct addresses for the block values."""
    import copy

    out = [p]
    for _ in range(n_copies - 1):
        q = copy.copy(p)
        q.vals = p.vals.clone()
        out.append(q)
    return out



def event_pair():
    ev = Events(1)
    ev.hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
    return ev


def time_eager(torch, calls, steps, warmup):
    """Wall ms per step of `steps` prepared calls issued from this thread, after `warmup` untimed ones."""
    n = len(calls)
    for i in range(warmup):
        calls[i % n]()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        calls[(warmup + i) % n]()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def time_graph(torch, make_calls, steps, warmup, replays=3):
    """The same `steps` calls recorded once into a HIP graph and replayed: median wall ms per step over `replays`
    timed replays (one untimed replay first).  make_calls() builds the prepared calls on the capture stream's
    buffers.  None if the capture is refused."""
    try:
        st = torch.cuda.Stream()  # default priority
        torch.cuda.synchronize()
        with torch.cuda.stream(st):
            calls = make_calls()
            n = len(calls)
            for i in range(min(warmup, 2 * n)):
                calls[i % n]()
            st.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=st):
                for i in range(steps):
                    calls[(warmup + i) % n]()
            graph.replay()
            torch.cuda.synchronize()
            times = []
            for _ in range(replays):
                t0 = time.perf_counter()
                graph.replay()
                torch.cuda.synchronize()
                times.append((time.perf_counter() - t0) * 1e3 / steps)
        del graph
        return statistics.median(times)
    except Exception as e:  # the eager figure stands
        print("graph replay not measured: %r" % (e,), file=sys.stderr)
        return None


def time_phases_in_pass(api, torch, sets, x, T, E, steps, warmup):
    """(gate/up ms, down ms) inside whole MLP passes: `steps` eager blast_sparse_mlp_events calls (rotating
    weight copies), each recording an event on the launch stream before the gate/up launch, between the two
    products and after the down product; means of the two intervals.  The `warmup` passes run immediately
    before (after an idle spell of a few milliseconds the chip first overshoots its power limit and then
    throttles: kernels take up to a third longer for the next twenty milliseconds)."""
    y = torch.empty((T, E), dtype=torch.float32, device="cuda:0")
    g0, u0, d0 = sets[0]
    ws = torch.empty(max(api.mlp_workspace_bytes(g0, u0, d0, T), 256), dtype=torch.uint8, device="cuda:0")
    ev = Events(steps)
    n = len(sets)
    for i in range(warmup):
        api.sparse_mlp(*sets[i % n], x, out=y, ws=ws)
    for i in range(steps):
        api.sparse_mlp(*sets[(warmup + i) % n], x, out=y, ws=ws, events=ev.triples[i])
    torch.cuda.synchronize()
    gu = statistics.fmean(ev.elapsed(t[0], t[1]) for t in ev.triples)
    dn = statistics.fmean(ev.elapsed(t[1], t[2]) for t in ev.triples)
    ev.destroy()
    return gu, dn


class Layer:
    """One workload packed on the device (and, on request, by the oracle), with rotated weight copies."""

    def __init__(self, name, api, torch, synth, want_oracle=False):
        from tests.helpers import mask_dev, to_dev

        self.wl = wl = synth.WORKLOADS[name]
        self.api, self.torch, self.synth = api, torch, synth
        inp = synth.make_mlp(wl)
        b = wl.b
        packed = []
        self.ref = []
        for l in (inp.gate, inp.up, inp.down):
            w_ = to_dev(l.W)
            packed.append(api.bsr_pack(w_, b, mask=mask_dev(l.mask), nnz_cap=int(l.mask.sum())) if l.mask is not None
                          else api.bsr_pack(w_, b, sparsity=l.sparsity))
            del w_
            if want_oracle:
                from oracle import oracle as orc

                self.ref.append(orc.pack(l.W, b, l.mask) if l.mask is not None else orc.pack_topk(l.W, b, l.sparsity)[0])
        del inp
        g, u, d = packed
        self.g, self.u, self.d = api.with_joint_row_order(g, u), u, d
        self.nnz = g.nnz + u.nnz + d.nnz
        self.w_bytes = self.nnz * b * b * 2
        n_copies = max(2, -(-768 * 1024 * 1024 // self.w_bytes))
        self.sets = list(zip(rotated_copies(self.g, n_copies), rotated_copies(u, n_copies), rotated_copies(d, n_copies)))

    def x(self, T):
        from tests.helpers import to_dev

        return to_dev(self.synth.make_x(self.wl, T))

    def time(self, T, steps, warmup):
        """(graph ms per pass or None, eager ms per pass) at T tokens."""
        api, torch = self.api, self.torch
        x = self.x(T)
        E = self.wl.hidden

        def make_calls():
            y = torch.empty((T, E), dtype=torch.float32, device="cuda:0")
            ws = torch.empty(max(api.mlp_workspace_bytes(self.g, self.u, self.d, T), 256), dtype=torch.uint8, device="cuda:0")
            return [api.prepare_sparse_mlp(g, u, d, x, y, ws) for g, u, d in self.sets]

        eager = time_eager(torch, make_calls(), steps, warmup)
        graph = time_graph(torch, make_calls, steps, warmup)
        return graph, eager

    def row(self, T, steps, warmup):
        """Compact record: [workload, T, us per pass (graph replay; eager if capture failed), us eager, bound,
        achieved (TFLOP/s on stored blocks or algorithmic GB/s), fraction of the MI355X peak]."""
        graph, eager = self.time(T, steps, warmup)
        ms = graph if graph is not None else eager
        wl, b = self.wl, self.wl.b
        if T >= 512:
            ach = 2.0 * b * b * T * self.nnz / (ms * 1e-3) / 1e12
            return [short(wl.name), T, sig(ms * 1e3), sig(eager * 1e3), "mfma", sig(ach), sig(ach / PEAK_BF16_TFLOPS, 3)]
        alg = self.w_bytes + 4 * self.nnz + 2 * wl.hidden * T + 4 * wl.hidden * T
        ach = alg / (ms * 1e-3) / 1e9
        return [short(wl.name), T, sig(ms * 1e3), sig(eager * 1e3), "hbm", sig(ach), sig(ach / PEAK_HBM_GBS, 3)]

    def row_e5m2w(self, T, steps, warmup):
        """The same pass with the three weights in E5M2 (blast_sparse_mlp_e5m2w, two launches): algorithmic bytes
        count one byte per stored weight."""
        api, torch = self.api, self.torch
        b, wl = self.wl.b, self.wl
        x = self.x(T)
        n8 = max(2, -(-768 * 1024 * 1024 // (self.w_bytes // 2)))
        base = [api.quantize_e5m2(m.vals[: m.nnz * b * b].contiguous()) for m in (self.g, self.u, self.d)]
        sets8 = [base] + [[v.clone() for v in base] for _ in range(n8 - 1)]

        def make_calls():
            y = torch.empty((T, wl.hidden), dtype=torch.float32, device="cuda:0")
            ws = torch.empty(max(T * wl.inter * 2, 256), dtype=torch.uint8, device="cuda:0")
            return [(lambda v=v: api.sparse_mlp_e5m2w(self.g, v[0], self.u, v[1], self.d, v[2], x, out=y, ws=ws))
                    for v in sets8]

        eager = time_eager(torch, make_calls(), steps, warmup)
        graph = time_graph(torch, make_calls, steps, warmup)
        ms = graph if graph is not None else eager
        alg = self.w_bytes // 2 + 4 * self.nnz + 2 * wl.hidden * T + 4 * wl.hidden * T
        ach = alg / (ms * 1e-3) / 1e9
        return [short(wl.name) + "+e5m2w", T, sig(ms * 1e3), sig(eager * 1e3), "hbm", sig(ach), sig(ach / PEAK_HBM_GBS, 3)]


def linear_row(api, torch, synth, steps, warmup):
    """Configuration 1: the single block-sparse linear layer (latency-bound correctness case), timed like the rest."""
    from tests.helpers import mask_dev, to_dev

    wl = synth.WORKLOADS["linear_1024x4096_b32_s90"]
    lin = synth.make_linear(wl)
    p = api.bsr_pack(to_dev(lin.W), wl.b, mask=mask_dev(lin.mask))
    T = wl.tokens[0]
    x = to_dev(synth.make_x(wl, T))
    y = torch.empty((T, wl.inter), dtype=torch.float32, device="cuda:0")
    fn = lambda: api.bsr_spmm(p, x, out=y)
    eager = time_eager(torch, [fn], steps, warmup)
    graph = time_graph(torch, lambda: [fn], steps, warmup)
    ms = graph if graph is not None else eager
    alg = p.nnz * wl.b * wl.b * 2 + 2 * wl.hidden * T + 4 * wl.inter * T
    ach = alg / (ms * 1e-3) / 1e9
    return [short(wl.name), T, sig(ms * 1e3), sig(eager * 1e3), "hbm", sig(ach), sig(ach / PEAK_HBM_GBS, 3)]

def two_matrix_mlp(workload: str, steps: int, warmup: int, cpu: bool):
    """Y = W2 act(W1 X) (GELU) on a GPT-2-shaped block: wall-clock time per pass at the workload's token
    counts, plus the oracle's time and the parity of the timed configuration on a token sample."""
    import numpy as np
    import torch

    from paper_2507_03117_amd import api, synth
    from tests.helpers import mask_dev, to_dev

    wl = synth.WORKLOADS[workload]
    l1, l2 = synth.make_mlp2(wl)
    b = wl.b
    p1 = api.bsr_pack(to_dev(l1.W), b, mask=mask_dev(l1.mask))
    p2 = api.bsr_pack(to_dev(l2.W), b, mask=mask_dev(l2.mask))
    nnz = p1.nnz + p2.nnz
    w_bytes = nnz * b * b * 2
    n_copies = max(2, -(-768 * 1024 * 1024 // w_bytes))
    sets = list(zip(rotated_copies(p1, n_copies), rotated_copies(p2, n_copies)))
    n = len(sets)
    passes = []
    for T in wl.tokens:
        x = to_dev(synth.make_x(wl, T))
        ws = torch.empty(max(api.mlp2_workspace_bytes(p1, p2, T), 256), dtype=torch.uint8, device="cuda:0")
        y = torch.empty((T, wl.hidden), dtype=torch.float32, device="cuda:0")
        for i in range(warmup):
            api.sparse_mlp2(*sets[i % n], x, act="gelu", out=y, ws=ws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            api.sparse_mlp2(*sets[(warmup + i) % n], x, act="gelu", out=y, ws=ws)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        flops = 2.0 * b * b * T * nnz
        alg_bytes = w_bytes + 4 * nnz + 2 * wl.hidden * T + 4 * wl.hidden * T
        passes.append({"T": T, "ms_per_step": ms, "TFLOPs": flops / (ms * 1e-3) / 1e12,
                       "frac_mfma": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                       "GBps": alg_bytes / (ms * 1e-3) / 1e9, "frac_hbm": alg_bytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS})
    out = {"workload": wl.name, "hidden": wl.hidden, "intermediate": wl.inter, "block": b, "sparsity": wl.sparsity,
           "mask": wl.mask_kind, "activation": "gelu", "nnz_blocks": nnz, "weight_copies_in_rotation": n_copies,
           "passes": passes}
    if cpu:
        from oracle import oracle as orc

        T = max(wl.tokens)
        Ts = min(1024, T)
        r1, r2 = orc.pack(l1.W, b, l1.mask), orc.pack(l2.W, b, l2.mask)
        xs = synth.make_x(wl, T)
        t0 = time.perf_counter()
        y_or = orc.mlp2(r1, r2, np.ascontiguousarray(xs[:Ts]), activation="gelu")
        sec = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 2.0 * b * b * Ts * nnz / sec / 1e12, "unit": "TFLOP/s", "cores": orc.num_threads(),
                               "kind": "oracle", "seconds": sec,
                               "sample": "first %d of %d tokens, all rows; dense masked fp64 triple loop" % (Ts, T)}
        yd = api.sparse_mlp2(p1, p2, to_dev(xs), act="gelu")
        torch.cuda.synchronize()
        yh = yd[:Ts].cpu().numpy().astype(np.float64).T
        out["parity_on_sample"] = {"rel_fro": float(np.linalg.norm(yh - y_or) / np.linalg.norm(y_or)),
                                   "max_abs_over_rms": float(np.abs(yh - y_or).max() / np.sqrt((y_or ** 2).mean()))}
    return out


def backward_products(workload: str, T: int, steps: int, warmup: int, cpu: bool):
    """Backward pass of one sparse projection (the gate matrix of the workload): the packed transpose (once per
    re-packing), dX = W~^T dY and the gradient of the stored blocks, each timed between two hipEvents around
    `steps` launches; the oracle timed beside them on a sample, which doubles as a parity check."""
    import numpy as np
    import torch

    from paper_2507_03117_amd import api, synth
    from tests.helpers import mask_dev, to_dev

    wl = synth.WORKLOADS[workload]
    lin = synth.make_mlp(wl).gate
    b = wl.b
    p = api.bsr_pack(to_dev(lin.W), b, mask=mask_dev(lin.mask)) if lin.mask is not None else \
        api.bsr_pack(to_dev(lin.W), b, sparsity=lin.sparsity)
    rng = np.random.default_rng(synth.BASE_SEED + 77)
    x_h = synth.make_x(wl, T)
    dy_h = synth.gauss_bf16(rng, (T, wl.inter), 1.0)
    X, dY = to_dev(x_h), to_dev(dy_h)
    pt = api.bsr_transpose(p)
    dX = torch.empty((T, wl.hidden), dtype=torch.float32, device="cuda:0")
    dv = torch.empty((p.nnz, b, b), dtype=torch.float32, device="cuda:0")

    def timed(fn, n, w):
        for _ in range(w):
            fn()
        ev = Events(1)
        hip, stream = ev.hip, C.c_void_p(torch.cuda.current_stream().cuda_stream)
        hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        torch.cuda.synchronize()
        hip.hipEventRecord(ev.triples[0][0], stream)
        for _ in range(n):
            fn()
        hip.hipEventRecord(ev.triples[0][1], stream)
        torch.cuda.synchronize()
        ms = ev.elapsed(ev.triples[0][0], ev.triples[0][1]) / n
        ev.destroy()
        return ms

    flops = 2.0 * b * b * T * p.nnz
    ms_t = timed(lambda: api.bsr_transpose(p), 5, 2)
    ms_dx = timed(lambda: api.bsr_spmm(pt, dY, out=dX), steps, warmup)
    ms_dw = timed(lambda: api.bsr_sddmm(p, dY, X, out=dv), steps, warmup)
    out = {"workload": wl.name, "matrix": "gate (%d x %d)" % (wl.inter, wl.hidden), "block": b, "tokens": T,
           "nnz_blocks": p.nnz, "transpose_ms": ms_t,
           "dX": {"ms": ms_dx, "TFLOPs": flops / (ms_dx * 1e-3) / 1e12, "frac_mfma": flops / (ms_dx * 1e-3) / 1e12 / PEAK_BF16_TFLOPS},
           "dW": {"ms": ms_dw, "TFLOPs": flops / (ms_dw * 1e-3) / 1e12, "frac_mfma": flops / (ms_dw * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}}
    if cpu:
        from oracle import oracle as orc

        ref = orc.pack(lin.W, b, lin.mask) if lin.mask is not None else orc.pack_topk(lin.W, b, wl.sparsity)[0]
        sel = np.unique(np.concatenate(([0, T - 1], rng.choice(T, min(T, 62), replace=False))))
        t0 = time.perf_counter()
        dx_or = orc.spmm_t(ref, np.ascontiguousarray(dy_h[sel]))
        sec_dx = time.perf_counter() - t0
        qs = np.unique(np.concatenate(([0, ref.nnz - 1], rng.choice(ref.nnz, min(ref.nnz, 30), replace=False))))
        rr = np.repeat(np.arange(wl.inter // b), np.diff(ref.row_ptr))
        sub = np.zeros((wl.inter // b, wl.hidden // b), dtype=np.uint8)
        sub[rr[qs], ref.col_idx[qs]] = 1
        ref_sub = orc.pack(lin.W, b, sub)
        t0 = time.perf_counter()
        dv_or = orc.sddmm(ref_sub, dy_h, x_h)
        sec_dw = time.perf_counter() - t0
        api.bsr_spmm(pt, dY, out=dX)
        api.bsr_sddmm(p, dY, X, out=dv)
        torch.cuda.synchronize()
        dxh = dX.cpu().numpy()[sel].astype(np.float64).T
        dvh = dv.cpu().numpy()[qs].astype(np.float64)
        out["cpu_baseline"] = {
            "dX": {"value": 2.0 * b * b * sel.size * ref.nnz / sec_dx / 1e12, "unit": "TFLOP/s", "seconds": sec_dx,
                   "sample": "%d of %d tokens, all rows; dense masked fp64 loop" % (sel.size, T)},
            "dW": {"value": 2.0 * b * b * T * qs.size / sec_dw / 1e12, "unit": "TFLOP/s", "seconds": sec_dw,
                   "sample": "%d of %d stored blocks, all tokens; fp64 loop" % (qs.size, ref.nnz)},
            "cores": orc.num_threads(), "kind": "oracle"}
        out["parity_on_sample"] = {
            "dX_rel_fro": float(np.linalg.norm(dxh - dx_or) / np.linalg.norm(dx_or)),
            "dW_rel_fro": float(np.linalg.norm(dvh - dv_or) / np.linalg.norm(dv_or))}
    return out


def e5m2_product(workload: str, tokens, steps: int, warmup: int, cpu: bool):
    """The gate projection of the workload with both operands in E5M2 (Sec. 5.2 dtype) next to the bf16 product of
    the same matrix, each timed between two hipEvents around `steps` launches; oracle timed on a token sample."""
    import numpy as np
    import torch

    from paper_2507_03117_amd import api, synth
    from tests.helpers import mask_dev, to_dev

    wl = synth.WORKLOADS[workload]
    lin = synth.make_mlp(wl).gate
    b = wl.b
    p = api.bsr_pack(to_dev(lin.W), b, mask=mask_dev(lin.mask)) if lin.mask is not None else \
        api.bsr_pack(to_dev(lin.W), b, sparsity=lin.sparsity)
    v8 = api.quantize_e5m2(p.vals[: p.nnz * b * b].contiguous())

    def timed(fn, n, w):
        for _ in range(w):
            fn()
        ev = Events(1)
        hip, stream = ev.hip, C.c_void_p(torch.cuda.current_stream().cuda_stream)
        hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        torch.cuda.synchronize()
        hip.hipEventRecord(ev.triples[0][0], stream)
        for _ in range(n):
            fn()
        hip.hipEventRecord(ev.triples[0][1], stream)
        torch.cuda.synchronize()
        ms = ev.elapsed(ev.triples[0][0], ev.triples[0][1]) / n
        ev.destroy()
        return ms

    passes = []
    for T in tokens:
        x_h = synth.make_x(wl, T)
        X = to_dev(x_h)
        X8 = api.quantize_e5m2(X)
        Y = torch.empty((T, wl.inter), dtype=torch.float32, device="cuda:0")
        flops = 2.0 * b * b * T * p.nnz
        ms16 = timed(lambda: api.bsr_spmm(p, X, out=Y), steps, warmup)
        ms8 = timed(lambda: api.bsr_spmm_e5m2(p, v8, X8, out=Y), steps, warmup)
        rec = {"T": T, "bf16_ms": ms16, "e5m2_ms": ms8, "bf16_TFLOPs": flops / (ms16 * 1e-3) / 1e12,
               "e5m2_TFLOPs": flops / (ms8 * 1e-3) / 1e12}
        if b >= 64:  # activations quantised into column groups of 64 features (whole cache lines per copy)
            XG = api.quantize_e5m2_groups(X)
            msg = timed(lambda: api.bsr_spmm_e5m2(p, v8, XG, layout=api.COLUMN_GROUPS_64, out=Y), steps, warmup)
            rec["e5m2_column_groups_ms"] = msg
            rec["e5m2_column_groups_TFLOPs"] = flops / (msg * 1e-3) / 1e12
            ms8 = min(ms8, msg)
        rec["e5m2_frac_mfma_fp8_peak"] = flops / (ms8 * 1e-3) / 1e12 / 5000.0
        passes.append(rec)
    out = {"workload": wl.name, "matrix": "gate (%d x %d)" % (wl.inter, wl.hidden), "block": b, "nnz_blocks": p.nnz,
           "passes": passes}
    if cpu:
        from oracle import oracle as orc

        T = max(tokens)
        x_h = synth.make_x(wl, T)
        sel = np.unique(np.concatenate(([0, T - 1], np.random.default_rng(3).choice(T, min(T, 62), replace=False))))
        ref = orc.pack(lin.W, b, lin.mask) if lin.mask is not None else orc.pack_topk(lin.W, b, wl.sparsity)[0]
        v8_or = orc.e5m2_quantize(synth.bf16_bits_to_f32(ref.vals))
        x8_or = orc.e5m2_quantize(synth.bf16_bits_to_f32(x_h[sel]))
        t0 = time.perf_counter()
        y_or = orc.spmm_e5m2(ref, v8_or, x8_or)
        sec = time.perf_counter() - t0
        y = api.bsr_spmm_e5m2(p, v8, api.quantize_e5m2(to_dev(x_h)))
        torch.cuda.synchronize()
        yh = y.cpu().numpy()[sel].astype(np.float64).T
        out["cpu_baseline"] = {"value": 2.0 * b * b * sel.size * ref.nnz / sec / 1e12, "unit": "TFLOP/s", "seconds": sec,
                               "cores": orc.num_threads(), "kind": "oracle",
                               "sample": "%d of %d tokens, all rows; dense masked fp64 loop on decoded codes" % (sel.size, T)}
        out["parity_on_sample"] = {"rel_fro": float(np.linalg.norm(yh - y_or) / np.linalg.norm(y_or)),
                                   "codes_identical": bool(np.array_equal(v8.cpu().numpy().reshape(v8_or.shape), v8_or))}
    return out



def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--tokens", type=int, default=2048, help="token count of the headline step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="time the headline workload only")
    ap.add_argument("--extras", action="store_true",
                    help="also: packer and mask-update times, two-matrix MLP, backward products, E5M2 product, 16-wide blocks")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2507_03117_amd import api, synth
    from tests.helpers import check_close, stratified_tokens

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    from paper_2507_03117_amd import build as hip_build

    hip_build.ensure_built()
    api.lib()
    cpu = not args.no_cpu_baseline
    T = args.tokens

    # ---- headline ---------------------------------------------------------------------------------
    L = Layer(args.workload, api, torch, synth, want_oracle=cpu)
    wl, b = L.wl, L.wl.b
    graph_ms, eager_ms = L.time(T, args.steps, args.warmup)
    step_ms = graph_ms if graph_ms is not None else eager_ms
    flops = 2.0 * b * b * T * L.nnz
    tflops = flops / (step_ms * 1e-3) / 1e12
    alg_bytes = L.w_bytes + 4 * L.nnz + 2 * wl.hidden * T + 4 * wl.hidden * T
    prefill = T >= 512
    if prefill:
        # dominant kernel: the gated gate/up product (2/3 of the stored blocks), bracketed by events inside
        # whole passes
        ksteps = max(10, args.steps // 2)
        settle = max(args.warmup, int(30.0 / max(step_ms, 1e-3)) + 1)  # about 30 ms of passes
        gu_ms, dn_ms = time_phases_in_pass(api, torch, L.sets, L.x(T), T, wl.hidden, ksteps, settle)
        gu_tf = 2.0 * b * b * T * (L.g.nnz + L.u.nnz) / (gu_ms * 1e-3) / 1e12
        kname = ("k_spmm_b16<dual>" if b == 16 else "k_spmm_stream<%d,dual>" % b) + " (gate/up + activation)"
        tr = profile_traffic(wl.name, T, "gate_up")
        roofline = {"bound": "mfma", "kernel": kname, "achieved": sig(gu_tf), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": sig(gu_tf / PEAK_BF16_TFLOPS, 3), "kernel_ms": sig(gu_ms), "down_kernel_ms": sig(dn_ms),
                    "traffic": tr["bytes"] if tr else None, "traffic_source": tr["source"] if tr else None}
    else:
        gbs = alg_bytes / (step_ms * 1e-3) / 1e9
        tr = profile_traffic(wl.name, T, "mlp")
        roofline = {"bound": "hbm", "kernel": "whole MLP pass", "achieved": sig(gbs), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": sig(gbs / PEAK_HBM_GBS, 3), "kernel_ms": sig(step_ms),
                    "traffic": tr["bytes"] if tr else None, "traffic_source": tr["source"] if tr else None}
    out = {
        "metric": "fused BSR MLP effective TFLOP/s (stored blocks) + HBM GB/s vs roofline at 90-95% sparsity",
        "value": sig(tflops, 5), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sig(step_ms, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "tokens": T, "block": b, "sparsity": wl.sparsity, "mask": wl.mask_kind,
                   "nnz_blocks": L.nnz, "weight_copies": len(L.sets),
                   "launch": "graph_replay_median3" if graph_ms is not None else "eager"},
        "frac_mfma_peak": sig(tflops / PEAK_BF16_TFLOPS, 3), "eager_ms_per_step": sig(eager_ms, 5),
        "roofline": roofline,
    }

    if cpu:
        from oracle import oracle as orc

        sel = stratified_tokens(T, 64) if T > 64 else np.arange(T)
        xs = synth.make_x(wl, T)
        t0 = time.perf_counter()
        y_or = orc.mlp(*L.ref, np.ascontiguousarray(xs[sel]))
        sec = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": sig(2.0 * b * b * sel.size * L.nnz / sec / 1e12), "unit": "TFLOP/s",
                               "cores": orc.num_threads(), "kind": "oracle", "seconds": sig(sec),
                               "sample": "%d of %d tokens (all tiles and seams), all rows" % (sel.size, T)}
        # the same sample doubles as a parity check of the timed launch configuration
        y = api.sparse_mlp(L.g, L.u, L.d, L.x(T))
        torch.cuda.synchronize()
        fro, mx = check_close(y.cpu().numpy()[sel].T, y_or, "bench parity")
        out["parity_on_sample"] = {"rel_fro": sig(fro, 3), "max_abs_over_rms": sig(mx, 3)}
        del y, y_or
        L.ref = []

    # ---- the other configurations -----------------------------------------------------------------
    if not args.no_configs and args.workload == HEADLINE:
        rows = []
        dsteps = max(args.steps, 100)
        for Td in (1, 16):  # the same layer at decode token counts: weight bytes, not launches, set the time
            rows.append(L.row(Td, dsteps, args.warmup))
        rows.append(L.row_e5m2w(1, dsteps, args.warmup))
        del L
        torch.cuda.empty_cache()
        rows.insert(0, linear_row(api, torch, synth, dsteps, args.warmup))
        for name, toks, st in (("llama1b_b64_s90", (1, 16, 128, 2048), dsteps),
                               ("llama3b_b64_s70", (4096,), args.steps), ("llama3b_b64_s80", (4096,), args.steps),
                               ("llama3b_b64_s90", (4096,), args.steps), ("llama3b_b64_s95", (4096,), args.steps),
                               ("llama8b_b128_s95", (1, 8, 32), dsteps)):
            Lc = Layer(name, api, torch, synth)
            for Tc in toks:
                rows.append(Lc.row(Tc, st if Tc < 512 else args.steps, args.warmup))
            if name in ("llama1b_b64_s90", "llama8b_b128_s95"):  # E5M2 weights, one token
                rows.append(Lc.row_e5m2w(1, st, args.warmup))
            del Lc
            torch.cuda.empty_cache()
        out["configs_columns"] = ["llama*", "T", "us_graph", "us_eager", "bound", "TFLOPs|GBps", "frac"]  # of the peak
        out["configs"] = rows

    if args.extras:
        torch.cuda.empty_cache()
        out["extras"] = {
            "two_matrix_mlp": two_matrix_mlp("gpt2xl_b64_s80", args.steps, args.warmup, cpu),
            "backward": backward_products("llama1b_b64_s90", 2048, args.steps, args.warmup, cpu),
            "e5m2": e5m2_product("llama1b_b64_s90", (16, 2048), args.steps, args.warmup, cpu),
            "pack": pack_times(api, torch, synth, cpu),
            "block16": block16_rows(api, torch, synth, args.steps, args.warmup),
            "dense_context": dense_context(api, torch, synth),
        }

    print(json.dumps(out, separators=(",", ":")))


def dense_context(api, torch, synth):
    """Context only (the paper quotes its MLP results as speedups over dense library GEMMs, Sec. 5.2): the dense
    MLP of the same shape - three torch.matmul calls (hipBLASLt) and the activation on random bf16 weights - timed on
    the same GPU next to the block-sparse pass.  Not part of the product path and not a target."""
    out = []
    for name, T in (("llama405b_b128_s95_zipf", 2048), ("llama3b_b64_s70", 4096), ("llama1b_b64_s90", 2048)):
        wl = synth.WORKLOADS[name]
        E, I = wl.hidden, wl.inter
        Lc = Layer(name, api, torch, synth)
        graph, eager = Lc.time(T, 20, 10)
        sparse_ms = graph if graph is not None else eager
        del Lc
        torch.cuda.empty_cache()
        wg, wu = (torch.randn((I, E), device="cuda:0", dtype=torch.bfloat16) * 0.02 for _ in range(2))
        wd = torch.randn((E, I), device="cuda:0", dtype=torch.bfloat16) * 0.02
        x = torch.randn((T, E), device="cuda:0", dtype=torch.bfloat16)

        def dense():
            return (torch.nn.functional.silu(x @ wg.t()) * (x @ wu.t())) @ wd.t()

        for _ in range(3):
            dense()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 10
        e0.record()
        for _ in range(reps):
            dense()
        e1.record()
        torch.cuda.synchronize()
        dense_ms = e0.elapsed_time(e1) / reps
        out.append({"workload": name, "T": T, "sparse_ms": sig(sparse_ms), "dense_torch_matmul_ms": sig(dense_ms),
                    "dense_TFLOPs": sig(6.0 * E * I * T / (dense_ms * 1e-3) / 1e12),
                    "speedup_over_dense": sig(dense_ms / sparse_ms, 3)})
        del wg, wu, wd, x
        torch.cuda.empty_cache()
    # the single product at the shape of the paper's largest kernel comparison (Sec. 5.2: Seq 1024, Emb 32768,
    # N = 4 Emb, 95 % sparsity), 128-wide blocks, uniform mask
    import numpy as np

    b, T, K, N = 128, 1024, 32768, 131072
    W = torch.randn((N, K), device="cuda:0", dtype=torch.bfloat16) * 0.02
    mask = torch.from_numpy(synth.uniform_mask(np.random.default_rng(synth.BASE_SEED + 9), N // b, K // b, 0.95)).to("cuda:0")
    p = api.bsr_pack(W, b, mask=mask, nnz_cap=int(mask.sum().item()))
    x = torch.randn((T, K), device="cuda:0", dtype=torch.bfloat16)
    y = torch.empty((T, N), device="cuda:0", dtype=torch.bfloat16)

    def timed(fn, reps=10):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    sparse_ms = timed(lambda: api.bsr_spmm(p, x, out=y))
    dense_ms = timed(lambda: torch.matmul(x, W.t(), out=y))
    out.append({"workload": "spmm %dx%d b%d s95 uniform" % (N, K, b), "T": T, "sparse_ms": sig(sparse_ms),
                "sparse_TFLOPs": sig(2.0 * b * b * T * p.nnz / (sparse_ms * 1e-3) / 1e12),
                "dense_torch_matmul_ms": sig(dense_ms), "dense_TFLOPs": sig(2.0 * N * K * T / (dense_ms * 1e-3) / 1e12),
                "speedup_over_dense": sig(dense_ms / sparse_ms, 3)})
    del W, p, x, y, mask
    torch.cuda.empty_cache()
    return out


def block16_rows(api, torch, synth, steps, warmup):
    """The 1B-shaped layer with 16 x 16 blocks (the smallest block size of the paper's block-size sweeps), same dense
    weights and sparsity as the 64-wide configuration: rows as in `configs`."""
    Lc = Layer("llama1b_b16_s90", api, torch, synth)
    rows = [Lc.row(Tc, max(steps, 100) if Tc < 512 else steps, warmup) for Tc in (1, 16, 128, 2048)]
    del Lc
    torch.cuda.empty_cache()
    return rows


def pack_times(api, torch, synth, cpu):
    """Block-norm pruning + packing (three matrices of the 1B-shaped layer, scoring mode) and one mask update of
    blocked prune-and-grow on its gate matrix."""
    import numpy as np

    from tests.helpers import to_dev

    wl = synth.WORKLOADS["llama1b_b64_s90"]
    inp = synth.make_mlp(wl)
    b = wl.b
    dW = [to_dev(l.W) for l in (inp.gate, inp.up, inp.down)]
    reps = 5
    for w_ in dW:
        api.bsr_pack(w_, b, sparsity=wl.sparsity)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        for w_ in dW:
            api.bsr_pack(w_, b, sparsity=wl.sparsity)  # the scoring mode: reads every dense weight once
    torch.cuda.synchronize()
    pack_ms = (time.perf_counter() - t0) * 1e3 / reps
    # the same three matrices enqueued back to back, one synchronisation (blast_bsr_pack_enqueue); wall clock and,
    # between two events on the stream, the device's share of it
    reps = 20
    api.bsr_pack_many(dW, b, sparsity=wl.sparsity)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        api.bsr_pack_many(dW, b, sparsity=wl.sparsity)
    many_ms = (time.perf_counter() - t0) * 1e3 / reps
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    dev_ms = []
    for _ in range(reps):
        e0.record()
        api.bsr_pack_many(dW, b, sparsity=wl.sparsity)
        e1.record()
        torch.cuda.synchronize()
        dev_ms.append(e0.elapsed_time(e1))
    reps = 5
    dense_bytes = sum(int(w_.numel()) * 2 for w_ in dW)
    g_h = synth.gauss_bf16(np.random.default_rng(synth.BASE_SEED + 5), inp.gate.W.shape, 1e-3)
    dG = to_dev(g_h)
    api.generate_masks(dW[0], dG, b, wl.sparsity)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        api.generate_masks(dW[0], dG, b, wl.sparsity)
    torch.cuda.synchronize()
    masks_ms = (time.perf_counter() - t0) * 1e3 / reps
    rec = {"ms_three_matrices_topk": pack_ms, "ms_three_matrices_topk_one_sync": many_ms,
           "ms_three_matrices_topk_on_stream": sorted(dev_ms)[len(dev_ms) // 2],
           "dense_GBps": dense_bytes / (many_ms * 1e-3) / 1e9,
           "frac_hbm": dense_bytes / (many_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
           "generate_masks_ms_gate_matrix": masks_ms}
    if cpu:
        from oracle import oracle as orc

        t0 = time.perf_counter()
        m_or = orc.generate_masks(inp.gate.W, g_h, b, wl.sparsity)
        rec["generate_masks_cpu_baseline"] = {
            "seconds": time.perf_counter() - t0, "kind": "oracle", "cores": 1, "sample": "the whole gate matrix and gradient",
            "identical_to_device": bool(np.array_equal(m_or, api.generate_masks(dW[0], dG, b, wl.sparsity).cpu().numpy()))}
    return rec


if __name__ == "__main__":
    main()
