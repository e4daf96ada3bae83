#!/usr/bin/env python3
"""Benchmark of the fused block-sparse SwiGLU MLP on one MI355X.

A step = one pass of the MLP of Eq. (1) (gate/up products, activation, down
product; output written) through the C ABI over one synthetic batch already
resident in HBM.  Packing is done once before the timed region, like loading a
checkpoint; its throughput is reported separately in "pack".

Workload (benchmark configs[1]): Llama-3.2-1B-shaped MLP, hidden 2048,
intermediate 8192, 64x64 blocks, 90 % uniform-random block sparsity.  The
headline `value` is the prefill case T = 2048 (effective TFLOP/s on stored
blocks); the decode token counts 1, 16, 128 are timed the same way and reported
under "decode" as algorithmic HBM GB/s.

Timing: the K steps are timed twice.  Eagerly: the loop calls blast_sparse_mlp, every tenth
step instrumented with HIP events (blast_sparse_mlp_events) for the per-phase and roofline
figures.  And as one replay of a HIP graph that holds the same K calls; the headline `value`
is the faster of the two ("config.launch" says which; normally the graph), both are reported
in "launch_modes".

Cold-HBM protocol: every step uses a different copy of the packed block values
(>= 768 MB in rotation), so no step re-reads weights still sitting in the
256 MB last-level cache.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # dense bf16 MFMA, MI355X
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch sequence from rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE), scaled by the
# factor a plain copy kernel of known size reads on the same counters.  Filled from profiles/*.txt.
# Source: profiles/bench_llama1b_b64_s90_hbm_traffic.txt (read x2.0, write x1.0; counters sit between each XCD's
# L2 and the fabric).  Keys: (kernel, tokens) of the default workload.
MEASURED_TRAFFIC_BYTES = {
    ("gate_up", 2048): 62.96e6 + 34.49e6,
    ("mlp", 1): 10.50e6 + 0.03e6,
    ("mlp", 16): 12.56e6 + 0.41e6,
    ("llama405b_b128_s95_zipf", 1): (175.63e6 + 0.12e6) + (88.61e6 + 0.13e6),
    ("llama405b_b128_s95_zipf", 8): (178.13e6 + 0.96e6) + (97.70e6 + 1.00e6),
    ("llama405b_b128_s95_zipf", 16): (181.38e6 + 1.92e6) + (112.39e6 + 2.01e6),
}


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


EVENT_EVERY = 10  # steps between two instrumented steps of the timed loop


def time_mlp(api, torch, sets, x, T, steps, warmup, ws):
    """Returns (wall ms per step, mean ms of phase 1, mean ms of phase 2, mean ms of the pass from events).

    The timed loop calls blast_sparse_mlp; every EVENT_EVERY-th step goes through blast_sparse_mlp_events
    instead, which records three hipEvents on the launch stream (each record costs the stream about 2.5 us,
    so instrumenting every step would inflate the per-step wall time by more than a tenth at these sizes)."""
    E = sets[0][2].rows
    y = torch.empty((T, E), dtype=torch.float32, device="cuda:0")
    marked = list(range(0, steps, EVENT_EVERY))
    ev = Events(len(marked))
    n = len(sets)
    # arguments marshalled once per (weight set, event triple): the timed loop is one foreign call per step
    plain = [api.prepare_sparse_mlp(g, u, d, x, y, ws) for g, u, d in sets]
    calls = []
    for i in range(steps):
        if i % EVENT_EVERY == 0:
            g, u, d = sets[(warmup + i) % n]
            calls.append(api.prepare_sparse_mlp(g, u, d, x, y, ws, events=ev.triples[i // EVENT_EVERY]))
        else:
            calls.append(plain[(warmup + i) % n])
    for i in range(warmup):
        plain[i % n]()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for call in calls:
        call()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    k = len(marked)
    p1 = sum(ev.elapsed(t[0], t[1]) for t in ev.triples) / k
    p2 = sum(ev.elapsed(t[1], t[2]) for t in ev.triples) / k
    tot = sum(ev.elapsed(t[0], t[2]) for t in ev.triples) / k
    ev.destroy()
    return wall_ms, p1, p2, tot


def time_gated_kernel(api, torch, sets, x, T, steps, warmup):
    """Mean duration of the dominant kernel on its own: `steps` launches of the gate/up product + activation
    (blast_bsr_gated_spmm, rotating weight copies) back to back between two hipEvents on the launch stream.
    The interval per launch is the kernel plus the dispatch gap to the next one, without the event records
    that the per-pass brackets of blast_sparse_mlp_events add around every phase."""
    I = sets[0][0].rows
    H = torch.empty((T, I), dtype=torch.bfloat16, device="cuda:0")
    n = len(sets)
    for i in range(warmup):
        api.bsr_gated_spmm(sets[i % n][0], sets[i % n][1], x, out=H)
    ev = Events(1)
    hip, stream = ev.hip, C.c_void_p(torch.cuda.current_stream().cuda_stream)
    hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
    torch.cuda.synchronize()
    hip.hipEventRecord(ev.triples[0][0], stream)
    for i in range(steps):
        g, u, _ = sets[(warmup + i) % n]
        api.bsr_gated_spmm(g, u, x, out=H)
    hip.hipEventRecord(ev.triples[0][1], stream)
    torch.cuda.synchronize()
    ms = ev.elapsed(ev.triples[0][0], ev.triples[0][1]) / steps
    ev.destroy()
    return ms


def graph_time_mlp(api, torch, sets, x, T, steps, warmup):
    """The same K steps recorded once into a HIP graph (rotating weight copies, fixed activation, output and
    workspace buffers) and replayed: wall ms per step of one timed replay, after one untimed replay (K >= W
    warm steps).  None if the capture is refused."""
    try:
        E = sets[0][2].rows
        n = len(sets)
        st = torch.cuda.Stream()  # default priority
        torch.cuda.synchronize()
        with torch.cuda.stream(st):
            y = torch.empty((T, E), dtype=torch.float32, device="cuda:0")
            ws = torch.empty(max(api.mlp_workspace_bytes(*sets[0], T), 256), dtype=torch.uint8, device="cuda:0")
            calls = [api.prepare_sparse_mlp(g, u, d, x, y, ws) for g, u, d in sets]
            st.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=st):
                for i in range(steps):
                    calls[(warmup + i) % n]()
            graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            graph.replay()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / steps
        del graph
        return ms
    except Exception as e:  # the eager figure stands
        print("graph replay not measured: %r" % (e,), file=sys.stderr)
        return None


def decode_sweep(workload: str, tokens, steps: int, warmup: int, time_pack: bool = False):
    """Decode-sized passes of another workload, packed here: list of per-token-count records.
    time_pack: also time block-norm pruning + packing of the gate matrix at the workload's sparsity (on a
    matrix of this size the packer is bound by reading the dense weight once)."""
    import torch

    from paper_2507_03117_amd import api, synth
    from tests.helpers import mask_dev, to_dev

    wl = synth.WORKLOADS[workload]
    inp = synth.make_mlp(wl)
    b = wl.b
    packed = []
    pack_rec = None
    for l in (inp.gate, inp.up, inp.down):
        w_ = to_dev(l.W)
        if time_pack and pack_rec is None:
            for _ in range(2):
                api.bsr_pack(w_, b, sparsity=wl.sparsity)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(5):
                api.bsr_pack(w_, b, sparsity=wl.sparsity)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) / 5 * 1e3
            dense = w_.numel() * 2
            pack_rec = {"ms_gate_matrix_topk": ms, "dense_MB": dense / 1e6, "dense_GBps": dense / ms / 1e6,
                        "frac_hbm": dense / ms / 1e6 / PEAK_HBM_GBS}
        packed.append(api.bsr_pack(w_, b, mask=mask_dev(l.mask), nnz_cap=int(l.mask.sum())) if l.mask is not None
                      else api.bsr_pack(w_, b, sparsity=l.sparsity))
        del w_
    del inp
    g, u, d = packed
    g = api.with_joint_row_order(g, u)
    nnz = g.nnz + u.nnz + d.nnz
    w_bytes = nnz * b * b * 2
    n_copies = max(2, -(-768 * 1024 * 1024 // w_bytes))
    sets = list(zip(rotated_copies(g, n_copies), rotated_copies(u, n_copies), rotated_copies(d, n_copies)))
    out = []
    for T in tokens:
        x = to_dev(synth.make_x(wl, T))
        ws = torch.empty(max(api.mlp_workspace_bytes(g, u, d, T), 256), dtype=torch.uint8, device="cuda:0")
        wall_ms, p1, p2, tot = time_mlp(api, torch, sets, x, T, steps, warmup, ws)
        alg_bytes = w_bytes + 4 * nnz + 2 * wl.hidden * T + 4 * wl.hidden * T
        gbs = alg_bytes / (wall_ms * 1e-3) / 1e9  # wall clock of the timed loop
        out.append({"T": T, "ms_per_step": wall_ms, "ms_events": tot, "ms_gate_up": p1, "ms_down": p2,
                    "alg_MB": alg_bytes / 1e6, "GBps": gbs, "frac_hbm": gbs / PEAK_HBM_GBS,
                    "GBps_events": alg_bytes / (tot * 1e-3) / 1e9,
                    "traffic": MEASURED_TRAFFIC_BYTES.get((wl.name, T))})
    rec = {"workload": wl.name, "hidden": wl.hidden, "intermediate": wl.inter, "block": b, "sparsity": wl.sparsity,
           "mask": wl.mask_kind, "nnz_blocks": nnz, "weight_copies_in_rotation": n_copies, "passes": out}
    if pack_rec is not None:
        rec["pack"] = pack_rec
    return rec


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
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="llama1b_b64_s90")
    ap.add_argument("--tokens", type=int, default=2048, help="token count of the headline step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-large-decode", action="store_true",
                    help="skip the decode passes of the 405B-class layer (the case where weight bytes, not launch "
                         "latency, set the time)")
    ap.add_argument("--no-mlp2", action="store_true", help="skip the two-matrix MLP (GPT-2-shaped) passes")
    ap.add_argument("--no-e5m2", action="store_true", help="skip the E5M2 product of the gate matrix")
    ap.add_argument("--no-backward", action="store_true", help="skip the backward-pass products of the gate matrix")
    ap.add_argument("--decode-tokens", default="", help="comma-separated decode token counts (default: the workload's)")
    ap.add_argument("--cpu-sample-tokens", type=int, default=2048)
    ap.add_argument("--copies", type=int, default=0,
                    help="weight copies in rotation (0 = enough for 768 MB: cold HBM; 1 = warm caches)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2507_03117_amd import api, synth
    from tests.helpers import mask_dev, to_dev

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    from paper_2507_03117_amd import build as hip_build

    hip_build.ensure_built()
    api.lib()
    wl = synth.WORKLOADS[args.workload]
    assert wl.kind == "mlp"
    inp = synth.make_mlp(wl)
    b = wl.b

    # ---- pack once (timed separately) ------------------------------------------------------
    def pack(lin):
        if lin.mask is not None:
            return api.bsr_pack(to_dev(lin.W), b, mask=mask_dev(lin.mask))
        return api.bsr_pack(to_dev(lin.W), b, sparsity=lin.sparsity)

    dW = [to_dev(l.W) for l in (inp.gate, inp.up, inp.down)]
    dM = [mask_dev(l.mask) if l.mask is not None else None for l in (inp.gate, inp.up, inp.down)]
    packed = []
    for w_, m_, l in zip(dW, dM, (inp.gate, inp.up, inp.down)):
        packed.append(api.bsr_pack(w_, b, mask=m_, nnz_cap=int(l.mask.sum())) if m_ is not None
                      else api.bsr_pack(w_, b, sparsity=l.sparsity))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    reps = 5
    for _ in range(reps):
        for w_, l in zip(dW, (inp.gate, inp.up, inp.down)):
            api.bsr_pack(w_, b, sparsity=l.sparsity)  # the scoring mode: reads every dense weight once
    torch.cuda.synchronize()
    pack_ms = (time.perf_counter() - t0) * 1e3 / reps
    dense_bytes = sum(int(w_.numel()) * 2 for w_ in dW)
    # one prune-and-grow mask update of the gate matrix (reads W and a gradient-shaped tensor once each)
    g_h = synth.gauss_bf16(np.random.default_rng(synth.BASE_SEED + 5), inp.gate.W.shape, 1e-3)
    dG = to_dev(g_h)
    api.generate_masks(dW[0], dG, b, wl.sparsity)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        api.generate_masks(dW[0], dG, b, wl.sparsity)
    torch.cuda.synchronize()
    masks_ms = (time.perf_counter() - t0) * 1e3 / reps
    masks_bytes = 2 * int(dW[0].numel()) * 2
    masks_cpu = None
    if not args.no_cpu_baseline:
        from oracle import oracle as orc

        t0 = time.perf_counter()
        m_or = orc.generate_masks(inp.gate.W, g_h, b, wl.sparsity)
        masks_cpu = {"seconds": time.perf_counter() - t0, "kind": "oracle", "cores": 1,
                     "sample": "the whole gate matrix and gradient",
                     "identical_to_device": bool(np.array_equal(m_or, api.generate_masks(dW[0], dG, b, wl.sparsity).cpu().numpy()))}
    del dW, dG
    g, u, d = packed
    g = api.with_joint_row_order(g, u)
    nnz = g.nnz + u.nnz + d.nnz
    w_bytes = nnz * b * b * 2
    n_copies = args.copies if args.copies > 0 else max(2, -(-768 * 1024 * 1024 // w_bytes))
    sets = list(zip(rotated_copies(g, n_copies), rotated_copies(u, n_copies), rotated_copies(d, n_copies)))

    def run_T(T, steps, warmup, warm_caches=False):
        x = to_dev(synth.make_x(wl, T))
        ws = torch.empty(max(api.mlp_workspace_bytes(g, u, d, T), 256), dtype=torch.uint8, device="cuda:0")
        # warm_caches: one copy of the weights, re-read from the caches by every pass (a cache-bandwidth figure)
        wall_ms, p1, p2, tot = time_mlp(api, torch, sets[:1] if warm_caches else sets, x, T, steps, warmup, ws)
        flops = 2.0 * b * b * T * nnz
        alg_bytes = w_bytes + 4 * nnz + 2 * wl.hidden * T + 4 * wl.hidden * T
        return dict(T=T, ms_per_step=wall_ms, ms_events=tot, ms_gate_up=p1, ms_down=p2, flops=flops,
                    alg_bytes=alg_bytes)

    T = args.tokens
    head = run_T(T, args.steps, args.warmup)
    eager_ms = head["ms_per_step"]
    # The headline step time: the K steps replayed from one HIP graph (launch-bound loops belong in graphs on
    # this hardware: the two kernels of a pass then follow each other without the host in between) or the eager
    # loop's, whichever way of launching the same K steps is faster here.  Both are reported.
    graph_ms = graph_time_mlp(api, torch, sets, to_dev(synth.make_x(wl, T)), T, args.steps, args.warmup) if T > 256 else None
    use_graph = graph_ms is not None and graph_ms <= eager_ms
    step_ms = graph_ms if use_graph else eager_ms
    tflops = head["flops"] / (step_ms * 1e-3) / 1e12

    # roofline of the dominant kernel (gate/up product + activation: 2/3 of the stored blocks)
    gu_flops = 2.0 * b * b * T * (g.nnz + u.nnz)
    mfma_bound = T >= 512
    if mfma_bound:
        # the kernel's own duration: back-to-back launches between two events (the bracket of a phase inside a
        # pass, phases_ms, also holds two event records and reads about 4 us more)
        gu_ms = time_gated_kernel(api, torch, sets, to_dev(synth.make_x(wl, T)), T, args.steps, args.warmup)
        gu_tflops = gu_flops / (gu_ms * 1e-3) / 1e12
        roofline = dict(bound="mfma", kernel="k_spmm_stream<%d,dual> (gate/up + activation)" % b, achieved=gu_tflops,
                        peak=PEAK_BF16_TFLOPS, unit="TFLOP/s", frac=gu_tflops / PEAK_BF16_TFLOPS,
                        avg_kernel_ms=gu_ms, avg_ms_inside_a_pass=head["ms_gate_up"], traffic=MEASURED_TRAFFIC_BYTES.get(("gate_up", T)) if args.workload == "llama1b_b64_s90" else None)
    else:
        gbs = head["alg_bytes"] / (head["ms_events"] * 1e-3) / 1e9
        roofline = dict(bound="hbm", kernel="whole MLP pass (event interval)", achieved=gbs, peak=PEAK_HBM_GBS, unit="GB/s",
                        frac=gbs / PEAK_HBM_GBS, avg_kernel_ms=head["ms_events"],
                        traffic=MEASURED_TRAFFIC_BYTES.get(("mlp", T)))

    out = {
        "metric": "fused BSR MLP effective TFLOP/s (stored blocks only), prefill T=%d" % T,
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": step_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "hidden": wl.hidden, "intermediate": wl.inter, "block": b,
                   "sparsity": wl.sparsity, "mask": wl.mask_kind, "tokens": T, "nnz_blocks": nnz,
                   "x_layout": "token_major", "y_dtype": "f32", "weight_copies_in_rotation": n_copies,
                   "launch": "hip_graph_replay" if use_graph else "eager"},
        "launch_modes": {"eager_ms_per_step": eager_ms, "eager_TFLOPs": head["flops"] / (eager_ms * 1e-3) / 1e12,
                         "graph_replay_ms_per_step": graph_ms},
        "frac_of_mfma_peak": tflops / PEAK_BF16_TFLOPS,
        "phases_ms": {"gate_up_act": head["ms_gate_up"], "down": head["ms_down"], "pass_events": head["ms_events"]},
        "roofline": roofline,
        "pack": {"ms_three_matrices_topk": pack_ms, "dense_GBps": dense_bytes / (pack_ms * 1e-3) / 1e9,
                 "frac_hbm": dense_bytes / (pack_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                 "generate_masks": {"ms_gate_matrix": masks_ms, "GBps": masks_bytes / (masks_ms * 1e-3) / 1e9,
                                    "frac_hbm": masks_bytes / (masks_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                    "cpu_baseline": masks_cpu}},
    }

    if not args.no_decode:
        dec = []
        dec_T = [int(t) for t in args.decode_tokens.split(",") if t] or [t for t in wl.tokens if t <= 128]
        for Td in dec_T:
            r = run_T(Td, max(args.steps, 100), args.warmup)
            gbs = r["alg_bytes"] / (r["ms_per_step"] * 1e-3) / 1e9  # wall clock of the timed loop
            warm = run_T(Td, max(args.steps, 100), args.warmup, warm_caches=True)
            dec.append({"T": Td, "ms_per_step": r["ms_per_step"], "ms_events": r["ms_events"],
                        "ms_gate_up": r["ms_gate_up"], "ms_down": r["ms_down"], "alg_MB": r["alg_bytes"] / 1e6,
                        "GBps": gbs, "frac_hbm": gbs / PEAK_HBM_GBS,
                        "GBps_events": r["alg_bytes"] / (r["ms_events"] * 1e-3) / 1e9,
                        "warm_caches": {"ms_per_step": warm["ms_per_step"], "ms_events": warm["ms_events"],
                                        "GBps_cache": r["alg_bytes"] / (warm["ms_per_step"] * 1e-3) / 1e9},
                        "traffic": MEASURED_TRAFFIC_BYTES.get(("mlp", Td)) if args.workload == "llama1b_b64_s90" else None,
                        "TFLOPs": r["flops"] / (r["ms_events"] * 1e-3) / 1e12})
        out["decode"] = dec

    if not args.no_cpu_baseline:
        from oracle import oracle as orc

        Ts = min(args.cpu_sample_tokens, T)
        rg = orc.pack(inp.gate.W, b, inp.gate.mask) if inp.gate.mask is not None else orc.pack_topk(inp.gate.W, b, wl.sparsity)[0]
        ru = orc.pack(inp.up.W, b, inp.up.mask) if inp.up.mask is not None else orc.pack_topk(inp.up.W, b, wl.sparsity)[0]
        rd = orc.pack(inp.down.W, b, inp.down.mask) if inp.down.mask is not None else orc.pack_topk(inp.down.W, b, wl.sparsity)[0]
        xs = synth.make_x(wl, T)[:Ts]
        t0 = time.perf_counter()
        y_or = orc.mlp(rg, ru, rd, np.ascontiguousarray(xs))
        sec = time.perf_counter() - t0
        out["cpu_baseline"] = {
            "value": 2.0 * b * b * Ts * nnz / sec / 1e12, "unit": "TFLOP/s", "cores": orc.num_threads(),
            "kind": "oracle", "seconds": sec,
            "sample": "first %d of %d tokens, all rows; dense masked fp64 triple loop (it also multiplies the zeros)" % (Ts, T),
        }
        # the same sample doubles as a parity check of the timed launch configuration
        x = to_dev(synth.make_x(wl, T))
        y = api.sparse_mlp(g, u, d, x)
        torch.cuda.synchronize()
        yh = y[:Ts].cpu().numpy().astype(np.float64).T
        out["parity_on_sample"] = {
            "rel_fro": float(np.linalg.norm(yh - y_or) / np.linalg.norm(y_or)),
            "max_abs_over_rms": float(np.abs(yh - y_or).max() / np.sqrt((y_or ** 2).mean())),
        }

    if not args.no_large_decode and args.workload == "llama1b_b64_s90":
        del sets
        torch.cuda.empty_cache()
        out["decode_hbm_bound"] = decode_sweep("llama405b_b128_s95_zipf", (1, 8, 16), 30, 5, time_pack=True)

    if not args.no_mlp2 and args.workload == "llama1b_b64_s90":
        torch.cuda.empty_cache()
        out["two_matrix_mlp"] = two_matrix_mlp("gpt2xl_b64_s80", args.steps, args.warmup, not args.no_cpu_baseline)

    if not args.no_backward and args.workload == "llama1b_b64_s90":
        torch.cuda.empty_cache()
        out["backward"] = backward_products(args.workload, T, args.steps, args.warmup, not args.no_cpu_baseline)

    if not args.no_e5m2 and args.workload == "llama1b_b64_s90":
        torch.cuda.empty_cache()
        out["e5m2"] = e5m2_product(args.workload, (16, T), args.steps, args.warmup, not args.no_cpu_baseline)

    print(json.dumps(out))


if __name__ == "__main__":
    main()
