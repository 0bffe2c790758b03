#!/usr/bin/env python3
"""Benchmark of the CDL quantized layer step on one MI355X.

A "step" is one pass of the whole hot path over one layer-shaped batch of
seeded synthetic input, in the order of Algorithm 1 of the paper:

    quantize W (indices, soft values, marginal PMF + entropy)
    quantize X (same)
    forward product over the indices            Y = dx*dw * Xi . Wi^T
    backward products                           dL/dQ(X), dL/dQ(W)   (fp32 upstream gradient)
    quantizer backward for X and for W          dX, dW, d(step), d(sharpness)

All inputs are resident in HBM before the timed region.  The timed step runs on the
largest of the five workloads (transformer-MLP-shaped, 8-bit levels).  One JSON line
is printed.  Its metric has two halves, and the line carries both:
  value                the quantizer's forward + backward rate in Gelem/s on the flat 25.6 M-entry weight
                       tensor (workload 4), from a cold cache, with its fraction of the 8 TB/s HBM peak beside it;
  index_gemm_fwd_TOPS  the forward index product on the timed workload, with its fractions of the int8 peak
                       and of its own roofline beside it.
ms_per_step is the whole step on the timed workload (step_gelem_per_s: entries of W and X per second of it).
Per-kernel times come from HIP events the library records around each of its kernels on the launch stream.
Cache state of every figure: "cold" = a 1 GiB scrub buffer is written right before the timed call (the chip's
last-level cache holds 256 MB); "warm" = calls back to back.  A step of workload 5 moves about 3.8 GB and is
cold by its size.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload {1,2,3,4,5}]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from collections import OrderedDict

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import cdl_inputs  # noqa: E402

METRIC = "quantizer fwd+bwd Gelem/s (% HBM peak); index-GEMM int8 TOPS (% MFMA peak)"
HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
INT8_PEAK_TOPS = 5000.0      # MI355X dense int8 MFMA


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def ensure_built():
    """The library must have been built from the sources in the tree: a missing or stale binary ends the run."""
    import paper_2501_09849_amd.build as b
    if b.is_stale():
        log("bench.py: %s is missing or was not built from the sources now in the tree; "
            "run `python -m paper_2501_09849_amd.build` (or __graft_entry__.build()) first" % b.LIB_PATH)
        sys.exit(4)
    import oracle
    oracle.build(force=False)


class Step:
    """Device buffers and the sequence of library calls of one layer step."""

    def __init__(self, wl, seed=0, fused=False):
        import torch
        self.fused = fused if (fused and wl.has_gemm and wl.N > 32 and wl.K % 4 == 0) else None
        import paper_2501_09849_amd as cdl
        self.torch, self.cdl, self.wl = torch, cdl, wl
        dev = "cuda:0"
        t0 = time.time()
        self.W_host = cdl_inputs.draw_w(wl, seed)
        self.G_host = cdl_inputs.draw_g(wl, seed)
        self.X_host = cdl_inputs.draw_x(wl, seed) if wl.has_gemm else None
        log("[bench] drew inputs in %.1fs" % (time.time() - t0))
        f32, i8 = torch.float32, torch.int8
        self.W = torch.from_numpy(self.W_host).to(dev)
        self.G = torch.from_numpy(self.G_host).to(dev)
        self.nW = self.W.numel()
        self.Wi = torch.empty(self.nW, dtype=i8, device=dev)
        self.Wsoft = torch.empty(self.nW, dtype=f32, device=dev)
        self.dW = torch.empty(self.nW, dtype=f32, device=dev)
        self.margW = torch.empty(wl.w_spec.n_levels, dtype=f32, device=dev)
        self.scal = torch.zeros(8, dtype=f32, device=dev)   # H_w, H_x, d_delta_w, d_alpha_w, d_delta_x, d_alpha_x
        ws_bytes = cdl.quantize_workspace_bytes(self.nW, wl.w_spec.n_levels)
        self.nX = 0
        if wl.has_gemm:
            M, N, K = wl.M, wl.N, wl.K
            self.X = torch.from_numpy(self.X_host).to(dev)
            self.nX = self.X.numel()
            self.Xi = torch.empty(self.nX, dtype=i8, device=dev)
            self.Xsoft = torch.empty(self.nX, dtype=f32, device=dev)
            self.dX = torch.empty(self.nX, dtype=f32, device=dev)
            self.margX = torch.empty(wl.x_spec.n_levels, dtype=f32, device=dev)
            self.Y = torch.empty((M, N), dtype=f32, device=dev)
            self.dXh = torch.empty((M, K), dtype=f32, device=dev)
            self.dWh = torch.empty((N, K), dtype=f32, device=dev)
            ws_bytes = max(ws_bytes, cdl.quantize_workspace_bytes(self.nX, wl.x_spec.n_levels),
                           cdl.qgemm_fwd_workspace_bytes(M, N, K), cdl.qgemm_bwd_workspace_bytes(M, N, K))
        self.ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
        torch.cuda.synchronize()

    def run(self):
        cdl, wl, s = self.cdl, self.wl, self.scal
        w, x = wl.w_spec, wl.x_spec
        wa = (w.lo, w.n_levels, w.delta, w.alpha)
        cdl.cdl_quantize_fwd(self.W, self.nW, *wa, self.Wi, self.Wsoft, self.margW, s[0:1], self.ws)
        if not wl.has_gemm:
            cdl.cdl_quantize_bwd(self.W, self.G, self.nW, *wa, self.dW, s[2:3], s[3:4], self.ws)
            return
        xa = (x.lo, x.n_levels, x.delta, x.alpha)
        M, N, K = wl.M, wl.N, wl.K
        cdl.cdl_quantize_fwd(self.X, self.nX, *xa, self.Xi, self.Xsoft, self.margX, s[1:2], self.ws)
        cdl.cdl_qgemm_fwd(self.Xi, self.Wi, M, N, K, x.delta, w.delta, None, self.Y, self.ws)
        if self.fused == "both":
            # the whole backward step in one call: neither dL/dQ(X) nor dL/dQ(W) is written
            cdl.cdl_qgemm_bwd_quantize_bwd(self.G, self.Xi, self.Wi, M, N, K, self.X, *xa, w.delta, self.dX, s[4:5], s[5:6],
                                           None, self.ws, theta_b=self.W, qparams_b=wa, d_theta_b=self.dW, d_delta_b=s[2:3],
                                           d_alpha_b=s[3:4])
            return
        if self.fused:
            # the activation-gradient product applies the quantizer's backward pass in its epilogue: dL/dQ(X) is never written
            cdl.cdl_qgemm_bwd_quantize_bwd(self.G, self.Xi, self.Wi, M, N, K, self.X, *xa, w.delta, self.dX, s[4:5], s[5:6],
                                           self.dWh, self.ws)
        else:
            cdl.cdl_qgemm_bwd(self.G, self.Xi, self.Wi, M, N, K, x.delta, w.delta, self.dXh, self.dWh, self.ws)
            cdl.cdl_quantize_bwd(self.X, self.dXh, self.nX, *xa, self.dX, s[4:5], s[5:6], self.ws)
        cdl.cdl_quantize_bwd(self.W, self.dWh, self.nW, *wa, self.dW, s[2:3], s[3:4], self.ws)


def kernel_model(wl, name, occurrence):
    """Algorithmic work of one launch: (bound, amount, unit of rate) - bytes for HBM-bound kernels, int8 ops for GEMMs.

    Quantizer forward: reads theta (4 B), writes index (1 B) and soft value (4 B) = 9 B per entry.
    Quantizer backward: reads theta and g (8 B), writes dtheta (4 B) = 12 B per entry.
    Index GEMMs: 2*M*N*K integer operations of the product being formed (for the limb kernels this is the
    product the caller asked for, not the limbs issued).
    """
    nW = wl.flat_n if wl.flat_n else wl.N * wl.K
    nX = wl.M * wl.K
    # per step the quantizer kernels run first on W, then on X (forward) and first on X, then on W (backward)
    if name == "quantize_fwd_kernel":
        n = nW if occurrence == 0 else nX
        return "hbm", 9.0 * n, n
    if name == "quantize_bwd_kernel":
        n = (nX if occurrence == 0 else nW) if wl.has_gemm else nW
        return "hbm", 12.0 * n, n
    if name == "limb_gemm_kernel(d_a_hat + quantize_bwd)":
        return "mfma", 2.0 * wl.M * wl.N * wl.K, 0
    if name.startswith("qgemm_kernel") or name.startswith("limb_gemm_kernel"):
        return "mfma", 2.0 * wl.M * wl.N * wl.K, 0
    if name == "absmax_kernel":
        return "hbm", 4.0 * wl.M * wl.N, 0          # reads g once
    if name == "da_direct_kernel":
        return "hbm", 4.0 * wl.M * wl.N + 1.0 * wl.N * wl.K + 4.0 * wl.M * wl.K, 0   # reads g and b_idx, writes d_a_hat
    if name == "transpose_i8_kernel":
        n = wl.N * wl.K if occurrence == 0 else wl.M * wl.K
        return "hbm", 2.0 * n, 0                    # reads and writes an index matrix
    return None, 0.0, 0


def cpu_baseline(wl, step):
    """Times the oracle, as it is, on a bounded sample of the same workload and scales to one step.  The hard
    indices the oracle produces on the way are compared with the GPU's on the same entries: the count of entries
    that differ where the oracle's two best level scores are closer than 1e-6 (exempt near-ties), and of any
    other difference (must be 0)."""
    import oracle
    parts = []
    t_all = time.time()

    def timed(f):
        t = time.perf_counter()
        r = f()
        return time.perf_counter() - t, r

    est = 0.0
    w, x = wl.w_spec, wl.x_spec
    index_check = {"sampled": 0, "exempt_near_ties": 0, "other_differences": 0}
    for name, host, spec, n_full, idx_dev in ((("W", step.W_host, w, step.nW, step.Wi),)
                                              + ((("X", step.X_host, x, step.nX, step.Xi),) if wl.has_gemm else ())):
        flat = host.reshape(-1)
        n_s = int(min(n_full, max(4096, 400_000_000 // spec.n_levels)))
        th = flat[:n_s]
        g = np.resize(step.G_host.reshape(-1), n_s)       # (repeated where the gradient tensor is the smaller one: timing only)
        a = (spec.lo, spec.n_levels, spec.delta, spec.alpha)
        dt_f, (r_idx, _, gap) = timed(lambda: oracle.quantize_fwd(th, *a))
        dt_m, _ = timed(lambda: oracle.marginal_entropy(th, *a))
        dt_b, _ = timed(lambda: oracle.quantize_bwd(th, g, *a))
        dt = dt_f + dt_m + dt_b
        est += dt * n_full / n_s
        parts.append("quantizer %s: %d of %d entries %.2fs" % (name, n_s, n_full, dt))
        diff = idx_dev[:n_s].cpu().numpy().astype(np.int64) != r_idx
        index_check["sampled"] += n_s
        index_check["exempt_near_ties"] += int((diff & (gap < 1e-6)).sum())
        index_check["other_differences"] += int((diff & (gap >= 1e-6)).sum())
    if wl.has_gemm:
        M, N, K = wl.M, wl.N, wl.K
        rows = int(max(1, min(M, 6.0e9 // (3.0 * N * K))))
        xi = cdl_inputs.draw_indices((rows, K), x.lo, x.hi, seed=1)   # timing does not depend on the index values
        wi = cdl_inputs.draw_indices((N, K), w.lo, w.hi, seed=2)
        g = step.G_host[:rows]
        dt = timed(lambda: oracle.qgemm_fwd(xi, wi, x.delta, w.delta))[0] + timed(lambda: oracle.qgemm_bwd(g, xi, wi, x.delta, w.delta))[0]
        est += dt * M / rows
        parts.append("GEMM fwd+bwd: %d of %d rows %.2fs" % (rows, M, dt))
    n_total = step.nW + step.nX
    # the headline metric itself: quantizer forward (indices, soft values, marginal PMF, entropy) + backward on the flat
    # 25.6 M-entry weight tensor of workload 4, on a sample of it
    wl4 = cdl_inputs.workload(4)
    s4 = wl4.w_spec
    n4 = int(min(wl4.flat_n, 1_000_000_000 // s4.n_levels))
    th4 = cdl_inputs.draw_w(wl4).reshape(-1)[:n4]
    g4 = np.random.default_rng(7).standard_normal(n4).astype(np.float32)
    a4 = (s4.lo, s4.n_levels, s4.delta, s4.alpha)
    dt4 = (timed(lambda: oracle.quantize_fwd(th4, *a4))[0] + timed(lambda: oracle.marginal_entropy(th4, *a4))[0]
           + timed(lambda: oracle.quantize_bwd(th4, g4, *a4))[0])
    return {
        "value": n4 / dt4 / 1e9, "unit": "Gelem/s (quantizer forward + backward on workload 4: the metric of `value`)",
        "cores": oracle.num_threads(), "kind": "oracle",
        "sample": "%d of %d entries of the flat weight tensor (31 levels) in %.2fs" % (n4, wl4.flat_n, dt4),
        "whole_step": {"value": n_total / est / 1e9, "unit": "Gelem/s (entries of W and X per second of one whole step of the timed workload)",
                       "sample": "; ".join(parts) + "; scaled linearly to one full step (%.0fs estimated)" % est},
        "measured_in_s": time.time() - t_all,
    }, index_check


SCRUB_BYTES = 1 << 30


class Scrub:
    """The cold-cache protocol: a 1 GiB buffer written right before a timed call, outside the library's events."""

    def __init__(self):
        import torch
        self.buf = torch.empty(SCRUB_BYTES // 4, dtype=torch.float32, device="cuda:0")
        self.n = 0

    def __call__(self):
        self.n += 1
        self.buf.fill_(float(self.n))


def timed_calls(calls, iters, scrub=None):
    """Runs every call of `calls` (name -> function that enqueues library kernels) `iters` times with the library's
    per-kernel events on; `scrub`, if given, runs before every call.  Returns name -> list of per-call kernel
    time sums in us (one per iteration)."""
    import torch
    import paper_2501_09849_amd as cdl
    out = {k: [] for k in calls}
    for k, f in calls.items():
        for _ in range(2):
            f()
        torch.cuda.synchronize()
        for _ in range(iters):
            if scrub is not None:
                scrub()
            cdl.cdl_profile_enable(True)
            f()
            torch.cuda.synchronize()
            recs = cdl.cdl_profile_collect()
            cdl.cdl_profile_enable(False)
            out[k].append(sum(ms for _, ms in recs) * 1e3)
    return out


def bracketed_calls(calls, iters, scrub=None):
    """Stream time of every call of `calls` between one pair of HIP events on the launch stream (the kernels of the
    call and the gaps between them, no per-kernel events); `scrub`, if given, runs before the first event."""
    import torch
    out = {k: [] for k in calls}
    for k, f in calls.items():
        for _ in range(2):
            f()
        torch.cuda.synchronize()
        for _ in range(iters):
            if scrub is not None:
                scrub()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            f()
            e1.record()
            torch.cuda.synchronize()
            out[k].append(e0.elapsed_time(e1) * 1e3)
    return out


def med_min(v):
    return {"median_us": float(np.median(v)), "min_us": float(np.min(v))}


def quantizer_only(scrub, seed=0, iters=10):
    """Quantizer forward (index, soft value, marginal PMF, entropy) + backward (dtheta, d step, d sharpness) on the
    25.6 M-entry flat weight tensor (31 levels), cold and warm, at kappa = 4 and at the paper's alpha = 500."""
    import torch
    import paper_2501_09849_amd as cdl
    wl = cdl_inputs.workload(4)
    st = Step(wl, seed)
    n = wl.flat_n
    out = {"workload": "%d:%s" % (wl.number, wl.name), "n": n, "levels": wl.w_spec.n_levels,
           "algorithmic_bytes_per_entry": {"fwd": 9, "bwd": 12}}
    for tag, spec in (("kappa_4", wl.w_spec), ("alpha_500", wl.w_spec.with_alpha(cdl_inputs.ALPHA_PAPER))):
        a = (spec.lo, spec.n_levels, spec.delta, spec.alpha)
        calls = {
            "fwd": lambda: cdl.cdl_quantize_fwd(st.W, n, *a, st.Wi, st.Wsoft, st.margW, st.scal[0:1], st.ws),
            "bwd": lambda: cdl.cdl_quantize_bwd(st.W, st.G, n, *a, st.dW, st.scal[2:3], st.scal[3:4], st.ws),
        }
        calls["fwd_then_bwd"] = lambda: (calls["fwd"](), calls["bwd"]())
        row = {"kappa": spec.alpha * spec.delta ** 2}
        for state, sc in (("cold", scrub), ("warm", None)):
            # the figure of merit: the two calls one after the other between one pair of events (their four kernels and
            # the gaps between them); beside it each call alone, and the sums of the kernel times from per-kernel events
            b = bracketed_calls(calls, iters, sc)
            t = timed_calls({"fwd": calls["fwd"], "bwd": calls["bwd"]}, iters, sc)
            med = float(np.median(b["fwd_then_bwd"]))
            row[state] = {"fwd_plus_bwd": med_min(b["fwd_then_bwd"]), "fwd": med_min(b["fwd"]), "bwd": med_min(b["bwd"]),
                          "sum_of_kernel_times": {"fwd": med_min(t["fwd"]), "bwd": med_min(t["bwd"])},
                          "gelem_per_s": n / med / 1e3, "algorithmic_GBps": 21.0 * n / med / 1e3,
                          "hbm_frac": 21.0 * n / med / 1e3 / HBM_PEAK_GBS}
        out[tag] = row
    del st
    torch.cuda.empty_cache()
    return out


def load_traffic(wl_number):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary (FETCH_SIZE + WRITE_SIZE, calibrated there)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_workload%d.txt" % wl_number)
    table = {}
    if not os.path.exists(path):
        return table
    for line in open(path):
        if line.startswith("#") or line.startswith("kernel") or not line.strip():
            continue
        name, _, fetch_mb, write_mb = line.rstrip("\n").split("\t")
        table.setdefault(name, []).append((float(fetch_mb) + float(write_mb)) * 1e6)
    return table


def traffic_of(table, kernel, occurrence):
    """Maps a name of the library's event records to the kernel name rocprofv3 prints (template arguments vary)."""
    if kernel == "limb_gemm_kernel(d_b_hat)":
        prefix, occ = "limb_gemm_kernel<true", 0
    elif kernel == "limb_gemm_kernel(d_a_hat)":
        prefix, occ = "limb_gemm_kernel<false", 0
    elif kernel == "qgemm_kernel(fwd)":
        prefix, occ = ("qgemm_dma_kernel" if any(n.startswith("qgemm_dma_kernel") for n in table) else "qgemm_kernel"), 0
    else:
        prefix, occ = kernel, occurrence
    for name, rows in table.items():
        if name == prefix or name.startswith(prefix + "<") or name.startswith(prefix + ",") or name.startswith(prefix + ">"):
            return rows[occ] if occ < len(rows) else None
    return None


def graph_replay(st, steps):
    """The same step captured once into a HIP graph and replayed: what a caller gains who removes the launch
    gaps (the library only enqueues kernels, so a step is capturable as it is).  Not the headline number:
    the timed region above launches eagerly, with the per-kernel events in it."""
    import torch
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        st.run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        st.run()
    for _ in range(2):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    n_total = st.nW + st.nX
    return {"ms_per_step": ms, "gelem_per_s": n_total / (ms * 1e-3) / 1e9, "replays": steps}


def machine_probes():
    """What the box itself sustains: a plain device copy (HBM) and register-resident int8 MFMAs (matrix cores)."""
    import torch
    import paper_2501_09849_amd as cdl
    out = {}
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").normal_()
    dst = torch.empty_like(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(2):
        dst.copy_(src)
    e0.record()
    for _ in range(5):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    out["copy_1GiB_GBps_read_plus_write"] = 2.0 * src.numel() * 4 / (e0.elapsed_time(e1) / 5 * 1e-3) / 1e9
    del src, dst
    sink = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    for rnd, key in ((False, "int8_mfma_probe_TOPS_constant_operands"), (True, "int8_mfma_probe_TOPS_random_operands")):
        cdl.cdl_probe_mfma_int8(2000, rnd, 256, sink)
        torch.cuda.synchronize()
        cdl.cdl_profile_enable(True)
        ops = cdl.cdl_probe_mfma_int8(20000, rnd, 256, sink)
        torch.cuda.synchronize()
        recs = cdl.cdl_profile_collect()
        cdl.cdl_profile_enable(False)
        out[key] = ops / (recs[0][1] * 1e-3) / 1e12
    # For scale only (no part of the path): the vendor library's int8 product, int32 output, on the shapes of the
    # forward product and of one limb of dL/dQ(x) of workload 5, uniformly random index bytes.
    try:
        for key, (m, n, k) in (("library_int8_gemm_TOPS_65536x3072x768", (65536, 3072, 768)),
                               ("library_int8_gemm_TOPS_65536x768x3072", (65536, 768, 3072))):
            a = torch.randint(-128, 128, (m, k), dtype=torch.int8, device="cuda:0")
            b = torch.randint(-128, 128, (k, n), dtype=torch.int8, device="cuda:0")
            for _ in range(2):
                torch._int_mm(a, b)
            e0.record()
            for _ in range(5):
                torch._int_mm(a, b)
            e1.record()
            torch.cuda.synchronize()
            out[key] = 2.0 * m * n * k / (e0.elapsed_time(e1) / 5 * 1e-3) / 1e12
            del a, b
    except Exception as ex:   # the probe is context, not a requirement
        out["library_int8_gemm"] = "unavailable: " + repr(ex)[:120]
    return out


def extensions_bench(seed=0, iters=5):
    """The rows next to the core path, on the flat 25.6 M-entry tensor: the probabilistic draw, the entropy-term
    gradient, and the truncated (top-5) CPMF in the soft regime of the paper's initial sharpness."""
    import torch
    import paper_2501_09849_amd as cdl
    wl = cdl_inputs.workload(4)
    spec = wl.w_spec
    n = wl.flat_n
    dev = "cuda:0"
    th = torch.from_numpy(cdl_inputs.draw_w(wl, seed)).to(dev)
    g = torch.from_numpy(cdl_inputs.draw_g(wl, seed)).to(dev)
    u = torch.rand(n, device=dev)
    idx = torch.empty(n, dtype=torch.int8, device=dev)
    soft = torch.empty(n, device=dev)
    dth = torch.empty(n, device=dev)
    marg = torch.empty(spec.n_levels, device=dev)
    sc = torch.zeros(4, device=dev)
    ws = torch.empty(cdl.quantize_workspace_bytes(n, spec.n_levels), dtype=torch.uint8, device=dev)
    a = (spec.lo, spec.n_levels, spec.delta, spec.alpha)
    soft_a = (spec.lo, spec.n_levels, spec.delta, cdl_inputs.ALPHA_PAPER)
    cdl.cdl_marginal_entropy(th, n, *a, marg, sc[0:1], ws)

    def timed(f):
        for _ in range(2):
            f()
        torch.cuda.synchronize()
        cdl.cdl_profile_enable(True)
        for _ in range(iters):
            f()
        torch.cuda.synchronize()
        recs = cdl.cdl_profile_collect()
        cdl.cdl_profile_enable(False)
        return sum(ms for _, ms in recs) / iters * 1e3

    out = {"workload": wl.name, "n": n, "levels": spec.n_levels}
    t = timed(lambda: cdl.cdl_quantize_draw(th, u, n, *a, idx))
    out["draw_us"], out["draw_GBps"] = t, 9.0 * n / t / 1e3                      # reads theta, u; writes one byte
    t = timed(lambda: cdl.cdl_entropy_bwd(th, marg, n, *a, 1.0, g, dth, sc[1:2], sc[2:3], ws))
    out["entropy_bwd_us"], out["entropy_bwd_GBps"] = t, 12.0 * n / t / 1e3        # reads theta, g; writes dtheta
    cdl.cdl_quantize_fwd(th, n, *a, idx)
    hws = torch.empty(cdl.huffman_workspace_bytes(n), dtype=torch.uint8, device=dev)
    hc = torch.empty(spec.n_levels, dtype=torch.int64, device=dev)
    hb = torch.zeros(1, device=dev)
    t = timed(lambda: cdl.cdl_huffman_bits(idx, n, spec.lo, spec.n_levels, hc, None, hb, hws))
    out["huffman_bits_us"], out["huffman_bits_GBps"], out["huffman_bits_per_weight"] = t, 1.0 * n / t / 1e3, float(hb.item())
    for key, k in (("full_cpmf", 0), ("top5", 5)):
        t = timed(lambda: (cdl.cdl_quantize_fwd(th, n, *soft_a, idx, soft, marg, sc[0:1], ws, top_k=k),
                           cdl.cdl_quantize_bwd(th, g, n, *soft_a, dth, sc[1:2], sc[2:3], ws, top_k=k)))
        out["soft_regime_fwd_bwd_us_" + key] = t
    out["soft_regime_kappa"] = cdl_inputs.ALPHA_PAPER * spec.delta ** 2
    return out


def gemm_only(number, scrub, seed=0, iters=5):
    """The three index products alone on another workload's shape, cold and warm, uniform random indices."""
    import torch
    import paper_2501_09849_amd as cdl
    wl = cdl_inputs.workload(number)
    M, N, K = wl.M, wl.N, wl.K
    w, x = wl.w_spec, wl.x_spec
    dev = "cuda:0"
    Xi = torch.from_numpy(cdl_inputs.draw_indices((M, K), x.lo, x.hi, seed=seed + 1)).to(dev)
    Wi = torch.from_numpy(cdl_inputs.draw_indices((N, K), w.lo, w.hi, seed=seed + 2)).to(dev)
    G = torch.from_numpy(cdl_inputs.draw_g(wl, seed)).to(dev)
    Y = torch.empty((M, N), dtype=torch.float32, device=dev)
    dXh = torch.empty((M, K), dtype=torch.float32, device=dev)
    dWh = torch.empty((N, K), dtype=torch.float32, device=dev)
    ws = torch.empty(max(256, cdl.qgemm_fwd_workspace_bytes(M, N, K), cdl.qgemm_bwd_workspace_bytes(M, N, K)),
                     dtype=torch.uint8, device=dev)
    calls = {
        "fwd": lambda: cdl.cdl_qgemm_fwd(Xi, Wi, M, N, K, x.delta, w.delta, None, Y, ws),
        "d_a_hat": lambda: cdl.cdl_qgemm_bwd(G, Xi, Wi, M, N, K, x.delta, w.delta, dXh, None, ws),
        "d_b_hat": lambda: cdl.cdl_qgemm_bwd(G, Xi, Wi, M, N, K, x.delta, w.delta, None, dWh, ws),
    }
    ops = 2.0 * M * N * K
    t_hbm = (4.0 * M * N + 1.0 * (M + N) * K) / (HBM_PEAK_GBS * 1e9)
    t_mfma = ops / (INT8_PEAK_TOPS * 1e12)
    out = {"workload": "%d:%s" % (wl.number, wl.name), "M": M, "N": N, "K": K, "index_values": "uniform over the level sets",
           "note": "d_a_hat / d_b_hat: one backward call each, helper kernels (max|g|, transposition, plan, reduction) included"}
    for state, sc in (("cold", scrub), ("warm", None)):
        t = timed_calls(calls, iters, sc)
        row = {}
        for key in calls:
            mm = med_min(t[key])
            mm["TOPS"] = ops / mm["median_us"] / 1e6
            mm["frac_of_int8_peak"] = mm["TOPS"] / INT8_PEAK_TOPS
            row[key] = mm
        row["fwd"]["frac_of_roofline"] = max(t_hbm, t_mfma) * 1e6 / row["fwd"]["median_us"]
        row["fwd"]["roofline_bound"] = "hbm" if t_hbm > t_mfma else "mfma"
        out[state] = row
    del Xi, Wi, G, Y, dXh, dWh, ws
    torch.cuda.empty_cache()
    return out


def conv_forward(scrub, seed=0, iters=5):
    """The forward product of the convolution that workload 3 stands for (ResNet-18 layer 3: 256 images of 14 x 14 x 256,
    256 kernels of 3 x 3, padding 1), read where the activations lie (cdl_qconv_fwd), against the index product on the
    matrix of input windows, which somebody has to write first (9 times the activations)."""
    import torch
    import paper_2501_09849_amd as cdl
    wl = cdl_inputs.workload(3)
    w, x = wl.w_spec, wl.x_spec
    B, H, W, C, N, R, S, stride, pad = 256, 14, 14, 256, 256, 3, 3, 1, 1
    dev = "cuda:0"
    M, K = B * H * W, R * S * C
    assert (M, N, K) == (wl.M, wl.N, wl.K)
    # operands as the layer has them: the workload's distributions on the un-expanded tensors, quantized by the library
    # (uniformly drawn indices would be larger on average and cost the gradient products a limb more)
    Xf = torch.from_numpy(cdl_inputs.draw_x(wl, seed, rows=(M * C + K - 1) // K).reshape(-1)[:M * C].copy()).to(dev)
    Wf = torch.from_numpy(cdl_inputs.draw_w(wl, seed).reshape(-1)).to(dev)
    Xi = torch.empty((B, H, W, C), dtype=torch.int8, device=dev)
    Wi = torch.empty((N, R, S, C), dtype=torch.int8, device=dev)
    cdl.cdl_quantize_fwd(Xf, Xf.numel(), x.lo, x.n_levels, x.delta, x.alpha, Xi)
    cdl.cdl_quantize_fwd(Wf, Wf.numel(), w.lo, w.n_levels, w.delta, w.alpha, Wi)
    del Xf, Wf
    Y = torch.empty((M, N), dtype=torch.float32, device=dev)
    Y2 = torch.empty((M, N), dtype=torch.float32, device=dev)
    # the matrix of windows, for the comparison only (torch is plumbing here; its time is reported, not counted)
    xp = torch.zeros((B, H + 2 * pad, W + 2 * pad, C), dtype=torch.int8, device=dev)
    xp[:, pad:pad + H, pad:pad + W, :] = Xi
    st_b, st_h, st_w, st_c = xp.stride()
    cols = torch.empty((M, K), dtype=torch.int8, device=dev)
    def expand():
        cols.view(B, H, W, R, S, C).copy_(torch.as_strided(xp, (B, H, W, R, S, C), (st_b, st_h * stride, st_w * stride, st_h, st_w, st_c)))
    expand()
    ws = torch.empty(max(256, cdl.qgemm_fwd_workspace_bytes(M, N, K)), dtype=torch.uint8, device=dev)
    G = torch.from_numpy(cdl_inputs.draw_g(wl, seed)).to(dev)           # [M, N] = [B, P, Q, N]
    dW, dW2 = torch.empty((N, K), dtype=torch.float32, device=dev), torch.empty((N, K), dtype=torch.float32, device=dev)
    dX = torch.empty((B, H, W, C), dtype=torch.float32, device=dev)
    dcols = torch.empty((M, K), dtype=torch.float32, device=dev)
    wsb = torch.empty(max(256, cdl.qgemm_bwd_workspace_bytes(M, N, K), cdl.qconv_bwd_weights_workspace_bytes(B, H, W, C, N, R, S, stride, pad),
                          cdl.qconv_bwd_activations_workspace_bytes(B, H, W, C, N, R, S, stride, pad)), dtype=torch.uint8, device=dev)
    calls = {"conv": lambda: cdl.cdl_qconv_fwd(Xi, Wi, B, H, W, C, N, R, S, stride, pad, x.delta, w.delta, None, Y, None),
             "product_on_windows": lambda: cdl.cdl_qgemm_fwd(cols, Wi.view(N, K), M, N, K, x.delta, w.delta, None, Y2, ws),
             "conv_weight_gradient": lambda: cdl.cdl_qconv_bwd_weights(G, Xi, B, H, W, C, N, R, S, stride, pad, x.delta, dW, wsb),
             "weight_gradient_on_windows": lambda: cdl.cdl_qgemm_bwd(G, cols, Wi.view(N, K), M, N, K, x.delta, w.delta, None, dW2, wsb),
             "conv_activation_gradient": lambda: cdl.cdl_qconv_bwd_activations(G, Wi, B, H, W, C, N, R, S, stride, pad, w.delta, dX, wsb),
             "activation_gradient_on_windows (before the sum over windows)": lambda: cdl.cdl_qgemm_bwd(G, cols, Wi.view(N, K), M, N, K, x.delta, w.delta, dcols, None, wsb)}
    out = {"layer": "B=256, 14x14x256 -> 256, 3x3, stride 1, padding 1 (M=%d, N=%d, K=%d)" % (M, N, K),
           "activation_bytes": int(Xi.numel()), "window_matrix_bytes": int(cols.numel())}
    ops = 2.0 * M * N * K
    for state, sc in (("cold", scrub), ("warm", None)):
        t = timed_calls(calls, iters, sc)
        row = {}
        for key in calls:
            mm = med_min(t[key])
            mm["TOPS"] = ops / mm["median_us"] / 1e6
            row[key] = mm
        out[state] = row
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        expand()
    e1.record()
    torch.cuda.synchronize()
    out["forming_the_window_matrix_us (a strided device copy, not a kernel of this library)"] = e0.elapsed_time(e1) / iters * 1e3
    out["outputs_equal"] = bool(torch.equal(Y, Y2) and torch.equal(dW, dW2))
    del Xi, Wi, Y, Y2, xp, cols, ws, G, dW, dW2, dX, dcols, wsb
    torch.cuda.empty_cache()
    return out


def conv_stage_shapes(batch=128, iters=5):
    """The three convolution calls on the 3 x 3 layers of a ResNet-18's four stages and its two stride-2 transitions
    (batch 128; activations |N(0,1)| on 16 unsigned levels, weights N(0, 2/fan-in) on 15 signed levels, the recipe of
    workload 3; g ~ N(0,1)): sums of kernel times per call, warm, median of `iters`."""
    import torch
    import paper_2501_09849_amd as cdl
    x, w = cdl_inputs.workload(3).x_spec, cdl_inputs.workload(3).w_spec
    dev = "cuda:0"
    rows = []
    for (H, C, N, stride) in ((56, 64, 64, 1), (28, 128, 128, 1), (14, 256, 256, 1), (7, 512, 512, 1), (56, 64, 128, 2), (28, 128, 256, 2)):
        B, W, R, S, pad = batch, H, 3, 3, 1
        P = (H + 2 * pad - R) // stride + 1
        gen = torch.Generator(device=dev)
        gen.manual_seed(H + C)
        Xf = torch.randn((B, H, W, C), device=dev, generator=gen).abs_()
        sigma_w = (2.0 / (R * S * C)) ** 0.5
        Wf = torch.randn((N, R, S, C), device=dev, generator=gen) * sigma_w
        delta_w = 2.0 * 0.79788 * sigma_w / 8.0 ** 0.5          # the step rule of Sec. V-B on N(0, sigma_w^2), 4 bits
        Xi = torch.empty((B, H, W, C), dtype=torch.int8, device=dev)
        Wi = torch.empty((N, R, S, C), dtype=torch.int8, device=dev)
        cdl.cdl_quantize_fwd(Xf, Xf.numel(), x.lo, x.n_levels, x.delta, x.alpha, Xi)
        cdl.cdl_quantize_fwd(Wf, Wf.numel(), w.lo, w.n_levels, delta_w, 4.0 / delta_w ** 2, Wi)
        G = torch.randn((B, P, P, N), device=dev, generator=gen)
        Y = torch.empty((B, P, P, N), device=dev)
        dW = torch.empty((N, R, S, C), device=dev)
        dX = torch.empty((B, H, W, C), device=dev)
        ws = torch.empty(max(256, cdl.qconv_bwd_weights_workspace_bytes(B, H, W, C, N, R, S, stride, pad),
                             cdl.qconv_bwd_activations_workspace_bytes(B, H, W, C, N, R, S, stride, pad)), dtype=torch.uint8, device=dev)
        calls = {"forward": lambda: cdl.cdl_qconv_fwd(Xi, Wi, B, H, W, C, N, R, S, stride, pad, x.delta, delta_w, None, Y, None),
                 "weight_gradient": lambda: cdl.cdl_qconv_bwd_weights(G, Xi, B, H, W, C, N, R, S, stride, pad, x.delta, dW, ws),
                 "activation_gradient": lambda: cdl.cdl_qconv_bwd_activations(G, Wi, B, H, W, C, N, R, S, stride, pad, delta_w, dX, ws)}
        t = timed_calls(calls, iters)
        gop = 2.0 * B * P * P * N * R * S * C / 1e9
        row = {"layer": "%dx%dx%d -> %d, stride %d" % (H, W, C, N, stride), "Gop_per_product": gop}
        for k in calls:
            us = float(np.median(t[k]))
            row[k] = {"us": us, "TOPS": gop / us * 1e3}
        rows.append(row)
        del Xf, Wf, Xi, Wi, G, Y, dW, dX, ws
        torch.cuda.empty_cache()
    return rows


def small_step(number, steps=20, warmup=3):
    """One whole layer step on a small workload (1: the tiny linear layer, 2: the CIFAR conv as an im2col GEMM)."""
    import torch
    wl = cdl_inputs.workload(number)
    st = Step(wl)
    for _ in range(warmup):
        st.run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        st.run()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    t = timed_calls({"step": st.run}, 5)
    n_total = st.nW + st.nX
    out = {"workload": "%d:%s" % (wl.number, wl.name), "M": wl.M, "N": wl.N, "K": wl.K, "ms_per_step": ms,
           "step_gelem_per_s": n_total / (ms * 1e-3) / 1e9, "sum_of_kernel_times": med_min(t["step"]), "cache": "warm (steps back to back)"}
    del st
    torch.cuda.empty_cache()
    return out


def conv_layer_step(number=3, geom=(256, 14, 14, 256, 256, 3, 3, 1, 1), steps=10, warmup=3):
    """The layer that workload 3 stands for as what it is - a convolution on [B,H,W,C] activations (ResNet-18 layer 3: 256
    images of 14 x 14 x 256, 256 kernels of 3 x 3, padding 1) - against the same layer as an index product on its matrix
    of input windows (workload 3 as the list gives it: the quantizer then runs on the 9 times larger window matrix).
    Conv form: quantize W and X (indices, soft values, marginal PMF, entropy), cdl_qconv_fwd, cdl_qconv_bwd_weights,
    cdl_qconv_bwd_activations, quantizer backward for X and W."""
    import torch
    import paper_2501_09849_amd as cdl
    wl = cdl_inputs.workload(number)
    w, x = wl.w_spec, wl.x_spec
    wa, xa = (w.lo, w.n_levels, w.delta, w.alpha), (x.lo, x.n_levels, x.delta, x.alpha)
    B, H, W, C, N, R, S, stride, pad = geom
    assert (B * H * W, N, R * S * C) == (wl.M, wl.N, wl.K) and stride == 1
    dev = "cuda:0"
    f32, i8 = torch.float32, torch.int8
    nX, nW = B * H * W * C, N * R * S * C
    X = torch.from_numpy(cdl_inputs.draw_x(wl).reshape(-1)[:nX].copy()).to(dev)     # same distribution, the un-expanded tensor
    Wt = torch.from_numpy(cdl_inputs.draw_w(wl).reshape(-1)).to(dev)
    G = torch.from_numpy(cdl_inputs.draw_g(wl)).to(dev)                              # [B*H*W, N]
    Xi, Wi = torch.empty(nX, dtype=i8, device=dev), torch.empty(nW, dtype=i8, device=dev)
    Xs, Ws = torch.empty(nX, dtype=f32, device=dev), torch.empty(nW, dtype=f32, device=dev)
    mX, mW = torch.empty(x.n_levels, dtype=f32, device=dev), torch.empty(w.n_levels, dtype=f32, device=dev)
    sc = torch.zeros(8, dtype=f32, device=dev)
    Y = torch.empty((B * H * W, N), dtype=f32, device=dev)
    dXh, dWh = torch.empty(nX, dtype=f32, device=dev), torch.empty(nW, dtype=f32, device=dev)
    dX, dW = torch.empty(nX, dtype=f32, device=dev), torch.empty(nW, dtype=f32, device=dev)
    ws = torch.empty(max(256, cdl.quantize_workspace_bytes(nX, x.n_levels), cdl.quantize_workspace_bytes(nW, w.n_levels),
                         cdl.qconv_bwd_weights_workspace_bytes(B, H, W, C, N, R, S, stride, pad),
                         cdl.qconv_bwd_activations_workspace_bytes(B, H, W, C, N, R, S, stride, pad)), dtype=torch.uint8, device=dev)

    def run():
        cdl.cdl_quantize_fwd(Wt, nW, *wa, Wi, Ws, mW, sc[0:1], ws)
        cdl.cdl_quantize_fwd(X, nX, *xa, Xi, Xs, mX, sc[1:2], ws)
        cdl.cdl_qconv_fwd(Xi, Wi, B, H, W, C, N, R, S, stride, pad, x.delta, w.delta, None, Y, None)
        cdl.cdl_qconv_bwd_weights(G, Xi, B, H, W, C, N, R, S, stride, pad, x.delta, dWh, ws)
        cdl.cdl_qconv_bwd_activations(G, Wi, B, H, W, C, N, R, S, stride, pad, w.delta, dXh, ws)
        cdl.cdl_quantize_bwd(X, dXh, nX, *xa, dX, sc[4:5], sc[5:6], ws)
        cdl.cdl_quantize_bwd(Wt, dWh, nW, *wa, dW, sc[2:3], sc[3:4], ws)

    def eager(f):
        for _ in range(warmup):
            f()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            f()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    ms_conv = eager(run)
    del X, Wt, G, Xi, Wi, Xs, Ws, Y, dXh, dWh, dX, dW, ws
    torch.cuda.empty_cache()
    st = Step(wl)
    ms_gemm = eager(st.run)
    n_gemm = st.nW + st.nX
    del st
    torch.cuda.empty_cache()
    return {"layer": "workload %d: B=%d, %dx%dx%d -> %d, %dx%d, stride %d, padding %d" % (number, B, H, W, C, N, R, S, stride, pad),
            "as_convolution": {"ms_per_step": ms_conv, "entries_quantized": nX + nW},
            "as_index_product_on_windows (the workload as listed; forming the window matrix not included)":
                {"ms_per_step": ms_gemm, "entries_quantized": n_gemm},
            "cache": "warm (steps back to back)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true")
    ap.add_argument("--fused", nargs="?", const="both", default=None, choices=["activations", "both"],
                    help="backward step through cdl_qgemm_bwd_quantize_bwd (the quantizer's backward pass applied where the products "
                         "finish: dL/dQ(X), and with 'both' also dL/dQ(W), never written) instead of cdl_qgemm_bwd followed by "
                         "cdl_quantize_bwd; measured slower by about 1 %% on workload 5, so the separate calls are the default")
    ap.add_argument("--step-only", action="store_true",
                    help="time the step and nothing else (for profiler runs): no quantizer-only legs, so `value` is null")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB device copy (a kernel of known HBM traffic, to calibrate rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only (no sharding, no collectives); --gpus %d is not supported" % args.gpus)
        sys.exit(2)

    ensure_built()
    import torch
    import paper_2501_09849_amd as cdl
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(3)
    cdl.load()
    wl = cdl_inputs.workload(args.workload)
    st = Step(wl, fused=args.fused)

    if args.copy_probe:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        st.run()
    torch.cuda.synchronize()

    # Per-kernel table: K steps with HIP events around every kernel.  An event pair costs a few microseconds of
    # stream time per launch (about 0.2 ms per step of workload 5), so these steps are not the timed ones.
    cdl.cdl_profile_enable(True)
    for _ in range(args.steps):
        st.run()
    torch.cuda.synchronize()
    recs = cdl.cdl_profile_collect()
    per_step0 = len(recs) // args.steps
    by_name = {}
    for name, ms in recs:
        by_name.setdefault(name, []).append(ms)
    # the kernel with the largest average duration: in the timed region only its launches are bracketed by events
    dom_name = max(by_name, key=lambda k: max(np.mean(by_name[k][i::max(1, len(by_name[k]) // args.steps)])
                                                   for i in range(max(1, len(by_name[k]) // args.steps))))
    cdl.cdl_profile_only(dom_name)

    # The timed region: exactly K steps between two synchronisations.
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        st.run()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    recs_timed = cdl.cdl_profile_collect()
    cdl.cdl_profile_only(None)
    cdl.cdl_profile_enable(False)
    assert per_step0 * args.steps == len(recs)

    ms_per_step = elapsed * 1e3 / args.steps
    n_total = st.nW + st.nX
    step_rate = n_total / (elapsed / args.steps) / 1e9

    # per-kernel table: launches are grouped by (name, position among same-named launches within a step)
    per_step = len(recs) // args.steps
    table = OrderedDict()
    for s in range(args.steps):
        seen = {}
        for name, ms in recs[s * per_step:(s + 1) * per_step]:
            occ = seen.get(name, 0)
            seen[name] = occ + 1
            table.setdefault((name, occ), []).append(ms)
    kernels = []
    for (name, occ), v in table.items():
        avg = float(np.mean(v))
        bound, amount, n_el = kernel_model(wl, name, occ)
        row = {"kernel": name, "launch": occ, "avg_us": avg * 1e3, "median_us": float(np.median(v)) * 1e3,
               "min_us": float(np.min(v)) * 1e3}
        if bound == "hbm":
            row.update(bound="hbm", algorithmic_GBps=amount / (avg * 1e-3) / 1e9,
                       frac=amount / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS)
        elif bound == "mfma":
            row.update(bound="mfma", algorithmic_TOPS=amount / (avg * 1e-3) / 1e12,
                       frac=amount / (avg * 1e-3) / 1e12 / INT8_PEAK_TOPS)
        kernels.append(row)
    dom = max(kernels, key=lambda r: r["avg_us"])
    # the dominant kernel's duration as measured inside the timed region (its launches only were bracketed there)
    if dom["kernel"] == dom_name and recs_timed:
        per = max(1, len(recs_timed) // args.steps)
        v = [ms for i, (name, ms) in enumerate(recs_timed) if i % per == dom["launch"]]
        if v:
            avg = float(np.mean(v))
            dom = dict(dom, avg_us=avg * 1e3, median_us=float(np.median(v)) * 1e3, min_us=float(np.min(v)) * 1e3)
            bound, amount, _ = kernel_model(wl, dom["kernel"], dom["launch"])
            if bound == "hbm":
                dom.update(algorithmic_GBps=amount / (avg * 1e-3) / 1e9, frac=amount / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS)
            elif bound == "mfma":
                dom.update(algorithmic_TOPS=amount / (avg * 1e-3) / 1e12, frac=amount / (avg * 1e-3) / 1e12 / INT8_PEAK_TOPS)
    traffic = traffic_of(load_traffic(wl.number), dom["kernel"], dom["launch"])
    traffic_source = ("profiles/hbm_traffic_workload%d.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this "
                      "command, not measured by this run)" % wl.number) if traffic is not None else None
    if dom.get("bound") == "mfma":
        roofline = {"kernel": "%s #%d" % (dom["kernel"], dom["launch"]), "bound": "mfma", "achieved": dom["algorithmic_TOPS"],
                    "peak": INT8_PEAK_TOPS, "unit": "TOP/s", "frac": dom["frac"], "traffic": traffic,
                    "traffic_source": traffic_source, "avg_launch_us": dom["avg_us"]}
    else:
        roofline = {"kernel": "%s #%d" % (dom["kernel"], dom["launch"]), "bound": "hbm", "achieved": dom.get("algorithmic_GBps"),
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": dom.get("frac"), "traffic": traffic,
                    "traffic_source": traffic_source, "avg_launch_us": dom["avg_us"]}

    out = OrderedDict()
    out["metric"] = METRIC
    out["value"] = None          # set below: the quantizer's rate on workload 4 from a cold cache
    out["unit"] = "Gelem/s"
    out["n_gpus"] = 1
    out["steps"] = args.steps
    out["warmup"] = args.warmup
    out["ms_per_step"] = ms_per_step
    out["higher_is_better"] = True
    out["scaling"] = "weak"
    out["vs_baseline"] = None
    out["dtype"] = "f32 quantizer (f64 in its soft-regime kernels), int8 x int8 -> int32 products"
    out["data"] = "synthetic"
    cfg = {"workload": "%d:%s" % (wl.number, wl.name), "entries_per_step": n_total,
           "w_levels": wl.w_spec.n_levels, "kappa": wl.w_spec.alpha * wl.w_spec.delta ** 2,
           "cache": "cold by size: a step moves about 3.8 GB, the last-level cache holds 256 MB" if wl.number == 5 else "steps back to back",
           "backward_step": ("cdl_qgemm_bwd_quantize_bwd (%s)" % st.fused) if st.fused else "cdl_qgemm_bwd + cdl_quantize_bwd"}
    if wl.has_gemm:
        cfg.update(M=wl.M, N=wl.N, K=wl.K, x_levels=wl.x_spec.n_levels)
    out["config"] = cfg
    out["step_gelem_per_s"] = step_rate
    out["roofline"] = roofline
    if not args.no_cpu_baseline:
        out["cpu_baseline"], out["hard_index_check"] = cpu_baseline(wl, st)
    if wl.has_gemm:
        # limb counts of the two backward products (diagnostic words at the start of the workspace): the int8 work
        # actually issued is that many times the product's own 2*M*N*K
        w_, x_ = wl.w_spec, wl.x_spec
        cdl.cdl_qgemm_bwd(st.G, st.Xi, st.Wi, wl.M, wl.N, wl.K, x_.delta, w_.delta, st.dXh, st.dWh, st.ws)   # (untimed: the words are overwritten by the calls that follow it in a step)
        torch.cuda.synchronize()
        limbs = st.ws[:8].view(torch.int32).cpu().tolist()
        for r in kernels:
            which = {"limb_gemm_kernel(d_a_hat)": 0, "limb_gemm_kernel(d_a_hat + quantize_bwd)": 0, "limb_gemm_kernel(d_b_hat)": 1}.get(r["kernel"])
            if which is not None and "algorithmic_TOPS" in r:
                r["limbs"] = limbs[which]
                r["issued_TOPS"] = r["algorithmic_TOPS"] * limbs[which]
                r["issued_frac_of_int8_peak"] = r["issued_TOPS"] / INT8_PEAK_TOPS
    roofline["avg_launch_us_measured"] = ("HIP events on the launch stream inside the timed steps; only this kernel's launches are "
                                          "bracketed there, every other kernel runs without events")
    out["kernels"] = kernels
    out["kernels_measured"] = ("%d further steps with HIP events around every kernel, run right before the timed steps "
                               "(the events themselves cost about 0.1 ms per 10 launches, so those steps are not the timed ones)" % args.steps)
    q_us = sum(r["avg_us"] for r in kernels if r["kernel"] in ("quantize_fwd_kernel", "quantize_bwd_kernel",
                                                                 "marginal_finalize_kernel", "scalar_finalize_kernel"))
    if q_us and not st.fused:
        out["quantizer_in_step"] = {"gelem_per_s": n_total / (q_us * 1e-6) / 1e9, "hbm_frac": 21.0 * n_total / (q_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                                    "us": q_us, "cache": "cold by size"}
    gf = [r for r in kernels if r["kernel"] == "qgemm_kernel(fwd)"]
    if gf:
        out["index_gemm_fwd_TOPS"] = gf[0]["algorithmic_TOPS"]
        out["index_gemm_fwd_frac_of_int8_peak"] = gf[0]["frac"]
        # the forward product writes M*N fp32 and reads both index matrices once: what HBM alone allows
        # (8 TB/s), and the smaller of the two ceilings as the launch's roofline
        t_hbm = (4.0 * wl.M * wl.N + 1.0 * (wl.M + wl.N) * wl.K) / (HBM_PEAK_GBS * 1e9)
        t_mfma = 2.0 * wl.M * wl.N * wl.K / (INT8_PEAK_TOPS * 1e12)
        out["index_gemm_fwd_frac_of_roofline"] = max(t_hbm, t_mfma) / (gf[0]["avg_us"] * 1e-6)
        out["index_gemm_fwd_roofline_bound"] = "hbm" if t_hbm > t_mfma else "mfma"
    if not args.no_extra and not args.step_only:
        out["step_as_hip_graph"] = graph_replay(st, args.steps)
        if wl.has_gemm and wl.N > 32 and wl.K % 4 == 0 and not st.fused:
            # the same step with the backward pass of both quantizers applied where the backward products finish
            # (cdl_qgemm_bwd_quantize_bwd), against the separate calls: same buffers, same box, right after the timed
            # steps, both without the per-kernel events of the timed region
            def eager(mode):
                st.fused = mode
                for _ in range(2):
                    st.run()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(args.steps):
                    st.run()
                torch.cuda.synchronize()
                st.fused = None
                return (time.perf_counter() - t0) * 1e3 / args.steps
            ms_s, ms_f = eager(None), eager("both")
            # the same step at the paper's initial sharpness alpha = beta = 500 (Sec. V-B) instead of kappa = 4: with
            # this workload's steps that is the weights of this workload are deep in the soft regime (kappa_w in the line: every level live, the generic loop)
            import dataclasses
            wl_k4 = st.wl
            st.wl = dataclasses.replace(wl_k4, w_spec=wl_k4.w_spec.with_alpha(cdl_inputs.ALPHA_PAPER),
                                        x_spec=wl_k4.x_spec.with_alpha(cdl_inputs.ALPHA_PAPER))
            ms_500 = eager(None)
            t500 = timed_calls({"step": st.run}, 3)
            out["step_at_alpha_500"] = {"ms_per_step": ms_500, "gelem_per_s": n_total / (ms_500 * 1e-3) / 1e9,
                                        "kappa_w": st.wl.w_spec.alpha * st.wl.w_spec.delta ** 2,
                                        "kappa_x": st.wl.x_spec.alpha * st.wl.x_spec.delta ** 2,
                                        "sum_of_kernel_times": med_min(t500["step"])}
            st.wl = wl_k4
            out["step_without_kernel_events"] = {
                "separate_calls": {"ms_per_step": ms_s, "gelem_per_s": n_total / (ms_s * 1e-3) / 1e9},
                "fused_backward": {"ms_per_step": ms_f, "gelem_per_s": n_total / (ms_f * 1e-3) / 1e9,
                                   "calls": "cdl_qgemm_bwd_quantize_bwd for both operands instead of cdl_qgemm_bwd + 2 x cdl_quantize_bwd"},
                "fused_over_separate": ms_f / ms_s}
    if not args.no_extra and not args.step_only and wl.has_gemm and wl.K % 128 == 0 and wl.x_spec.hi <= 127:
        # the forward product with the activation quantizer in its prologue (the indices of X are never written),
        # against the hard-index quantizer followed by the forward product; same buffers
        x_, w_ = wl.x_spec, wl.w_spec
        xa_ = (x_.lo, x_.n_levels, x_.delta, x_.alpha)
        t = timed_calls({"quantizer_in_prologue": lambda: cdl.cdl_qgemm_fwd_quantize(st.X, *xa_, st.Wi, wl.M, wl.N, wl.K, w_.delta, st.Y),
                         "index_only_quantizer_then_product": lambda: (cdl.cdl_quantize_fwd(st.X, st.nX, *xa_, st.Xi),
                                                                       cdl.cdl_qgemm_fwd(st.Xi, st.Wi, wl.M, wl.N, wl.K, x_.delta, w_.delta, None, st.Y, st.ws))}, 5)
        out["forward_with_quantizer_in_prologue"] = {k: med_min(v) for k, v in t.items()}
    del st
    torch.cuda.empty_cache()
    if args.step_only:
        print(json.dumps(out), flush=True)
        return
    scrub = Scrub()
    qo = quantizer_only(scrub)
    out["quantizer_only_flat_25M"] = qo
    out["value"] = qo["kappa_4"]["cold"]["gelem_per_s"]
    out["value_is"] = ("quantizer forward (index, soft value, marginal PMF, entropy) + backward (dtheta, d step, d sharpness) on "
                       "workload 4 (25.6 M entries, 31 levels, kappa 4), cache cold (1 GiB written before), the two calls between one pair of "
                       "HIP events on the launch stream, median of 10; hbm_frac beside it")
    out["value_hbm_frac"] = qo["kappa_4"]["cold"]["hbm_frac"]
    out["targets"] = {
        "quantizer_fwd_bwd_hbm_frac": {"target": 0.70, "achieved_cold": qo["kappa_4"]["cold"]["hbm_frac"],
                                       "achieved_warm": qo["kappa_4"]["warm"]["hbm_frac"],
                                       "met": bool(qo["kappa_4"]["cold"]["hbm_frac"] >= 0.70)},
    }
    if gf:
        out["targets"]["index_gemm_frac_of_int8_peak"] = {"target": 0.60, "achieved": gf[0]["frac"], "met": bool(gf[0]["frac"] >= 0.60),
                                                          "hbm_limited_ceiling": min(1.0, t_mfma / max(t_hbm, t_mfma))}
    if not args.no_extra:
        out["small_workloads"] = [small_step(1), small_step(2)]
        out["conv_layer_step"] = [conv_layer_step(3, (256, 14, 14, 256, 256, 3, 3, 1, 1)), conv_layer_step(2, (128, 32, 32, 16, 16, 3, 3, 1, 1))]
        out["index_gemms_alone"] = [gemm_only(n_, scrub) for n_ in (2, 3) if n_ != wl.number]
        out["conv_layer_without_window_matrix"] = conv_forward(scrub)
        out["conv_calls_on_resnet18_stage_shapes_batch128"] = conv_stage_shapes()
        del scrub
        torch.cuda.empty_cache()
        out["extensions_flat_25M"] = extensions_bench()
        out["machine"] = machine_probes()
        # the quantizer's traffic against what a plain device copy moves on this machine (half reads, half writes, as the
        # quantizer's own mix nearly is): the practical ceiling of an HBM-bound kernel here, next to the nameplate one
        copy = out["machine"].get("copy_1GiB_GBps_read_plus_write")
        if copy:
            out["value_frac_of_measured_copy_rate"] = qo["kappa_4"]["cold"]["algorithmic_GBps"] / copy
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
