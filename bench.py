#!/usr/bin/env python3
"""Benchmark of the Monarch multiply hot path (forward + backward) on one MI355X.

Headline ("step"): the GPT-2-medium-style MLP pair 1024 -> 4096 -> 1024 on 16384 tokens, the largest
of the five stated configurations: forward of both layers, then backward of both (no nonlinearity
between the two multiplies, the hidden activation stored in bf16 in HBM between the calls):
    h = fwd(x; fc1)   y = fwd(h; fc2)   (dh, dR2, dL2) = bwd(dy, h; fc2)   (dx, dR1, dL1) = bwd(dh, x; fc1)
`--workload NAME` times one layer's forward + backward as the step instead.

Prints ONE JSON line.  Besides the headline it carries, under detail.configs, one block for every
stated configuration (and the n = 256 fp32 shape at 2^20 rows): forward and backward time per call
(median and minimum over >= 100 timed calls), TFLOP/s, GB/s, fraction of the nominal roofline and of the
measured copy rate, HBM traffic from the committed counter profiles, the vendor dense GEMM of the same
(B, n_in, n_out), and the kernels the dispatcher picked.  `--gpus N` with N > 1 is refused: the library is
a single-GPU kernel library.

Timing: the K steps are bracketed by torch.cuda.synchronize(); per-call durations come from HIP events
recorded on the stream the kernels are launched on (torch's current stream) around runs of consecutive
calls of one entry point, so that the events (3-10 us each) sit outside the timed launches.  Buffers
rotate through enough distinct sets that the footprint exceeds the 256 MB Infinity Cache, so repeats are
served from HBM; the weights stay hot, as they would in training.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}
ROTATE_BYTES = 1 << 30
COPY_BYTES = 1 << 30           # size of the plain copy timed as the empirical HBM roof
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "traffic.json")
PAIR = "gpt2m_pair"
CONFIGS = ("sq256_f32", "sq256_f32_big", "vitb_proj", "gpt2s_fc1", "sq4096", "gpt2m_fc1", "gpt2m_fc2")
TIMED_CALLS = 100              # per entry point and configuration, split into RUNS runs
RUNS = 10


def _events(n):
    import torch
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


def timed_runs(fn, calls: int = TIMED_CALLS, runs: int = RUNS, untimed: int = 3):
    """`runs` runs of calls/runs consecutive calls of fn(i), each run between two events on the launch
    stream; returns (median, min, mean) over the runs of the time per call, in ms, and the calls timed."""
    import numpy as np
    import torch
    per = max(1, -(-calls // runs))
    for i in range(untimed):   # first launches of a kernel pay for loading it
        fn(i)
    out = []
    n = untimed
    for _ in range(runs):
        e0, e1 = _events(2)
        e0.record()
        for _ in range(per):
            fn(n)
            n += 1
        e1.record()
        torch.cuda.synchronize()
        out.append(e0.elapsed_time(e1) / per)
    return float(np.median(out)), float(np.min(out)), float(np.mean(out)), per * runs


def graph_time(fn, calls_per_graph: int = 50, replays: int = 10):
    """Time per call (ms) of fn(i) when `calls_per_graph` consecutive calls are captured into one HIP graph and the
    graph is replayed: the host's share of a launch (interpreter, binding, runtime) is paid at capture, not at
    replay, so for microsecond kernels this is the GPU's own time per call.  Median and min over the replays."""
    import numpy as np
    import torch
    for i in range(3):
        fn(i)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for i in range(calls_per_graph):
            fn(i)
    g.replay()
    torch.cuda.synchronize()
    out = []
    for _ in range(replays):
        e0, e1 = _events(2)
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        out.append(e0.elapsed_time(e1) / calls_per_graph)
    del g
    return float(np.median(out)), float(np.min(out))


def copy_roof(reps: int = 5):
    """GB/s (read + write) of the library's plain streaming copy over COPY_BYTES: the empirical HBM roof.
    A profiler run of this script also uses this kernel's known traffic to calibrate its counters."""
    import torch
    from paper_2204_00595_amd import binding
    src = torch.empty(COPY_BYTES, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    src.zero_()
    best = None
    for _ in range(reps):
        e0, e1 = _events(2)
        e0.record()
        binding.monarch_stream_copy(dst, src)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        best = ms if best is None or ms < best else best
    del src, dst
    return 2.0 * COPY_BYTES / (best * 1e-3) / 1e9


def launch_floor():
    """Time per launch of a run of empty kernels on the launch stream, in us (median and min of 10 runs of 200)."""
    from paper_2204_00595_amd import binding
    med, mn, _, _ = timed_runs(lambda i: binding.monarch_launch_probe(), calls=2000, runs=10)
    return {"median_us": med * 1e3, "min_us": mn * 1e3}


def mfma_roof(n: int = 8192, reps: int = 10):
    """TFLOP/s of the vendor library's dense GEMM at a large square shape: the empirical matrix-core roof."""
    import torch
    res = {}
    for name, dt in (("bf16", torch.bfloat16), ("f32", torch.float32)):
        a = torch.randn(n, n, device="cuda", dtype=dt)
        b = torch.randn(n, n, device="cuda", dtype=dt)
        for _ in range(2):
            a @ b
        torch.cuda.synchronize()
        e0, e1 = _events(2)
        e0.record()
        for _ in range(reps):
            a @ b
        e1.record()
        torch.cuda.synchronize()
        res[name] = 2.0 * n ** 3 * reps / (e0.elapsed_time(e1) * 1e-3) / 1e12
    return res


def traffic_of(workload: str, call: str):
    """HBM bytes per call from the committed rocprofv3 counter profile of the workload, or None."""
    if not os.path.exists(TRAFFIC_JSON):
        return None
    t = json.load(open(TRAFFIC_JSON)).get(workload, {}).get(call)
    return (t["fetch_bytes"] + t["write_bytes"]) if t else None


def roofline_of(sh, ps: str, ms: float):
    """Nominal roofline of one call: max(T_hbm, T_mfma) / measured, and which of the two bounds it."""
    flops = sh.fwd_flops() if ps == "fwd" else sh.bwd_flops()
    nbytes = sh.fwd_bytes() if ps == "fwd" else sh.bwd_bytes()
    t_hbm = nbytes / (HBM_PEAK_GBS * 1e9)
    t_mfma = flops / (MFMA_PEAK_TFLOPS[sh.dtype] * 1e12)
    return max(t_hbm, t_mfma) / (ms * 1e-3), ("hbm" if t_hbm >= t_mfma else "mfma")


def _gen_rows(B: int, cap: int = 2048) -> int:
    """Largest divisor of B that is <= cap: rows drawn from the generator; the rest of the batch repeats them
    (the kernels' time does not depend on the values, and generating 10^8 normals on the host takes minutes)."""
    return max(d for d in range(1, min(B, cap) + 1) if B % d == 0)


class Layer:
    """Device tensors of one workload: weights, gradients, workspaces, and rotating activation sets."""

    def __init__(self, name: str, rotate_bytes: int = ROTATE_BYTES):
        import torch
        from paper_2204_00595_amd import binding, synth
        self.name = name
        self.sh = sh = synth.workload(name)
        self.dt = torch.float32 if sh.dtype == "f32" else torch.bfloat16
        self.code = 0 if sh.dtype == "f32" else 1
        dev = torch.device("cuda:0")
        gen_rows = _gen_rows(sh.B)  # the batch repeats a generated block of rows (timing only)
        x, R, L, dy = synth.make_inputs(sh, rows=gen_rows)
        self.R, self.L = (torch.from_numpy(a).to(dev).to(self.dt) for a in (R, L))
        x0 = torch.from_numpy(x).to(dev).to(self.dt).repeat(sh.B // gen_rows, 1)
        dy0 = torch.from_numpy(dy).to(dev).to(self.dt).repeat(sh.B // gen_rows, 1)
        per_set = sh.esize * sh.B * (2 * sh.n_in + 2 * sh.n_out)
        self.nsets = max(2, min(64, -(-rotate_bytes // per_set)))
        self.sets = []
        for i in range(self.nsets):
            xs = x0 if i == 0 else x0.roll(i, 0).contiguous()
            dys = dy0 if i == 0 else dy0.roll(i, 0).contiguous()
            self.sets.append((xs, dys, torch.empty((sh.B, sh.n_out), dtype=self.dt, device=dev), torch.empty_like(xs)))
        self.dR = torch.empty_like(self.R)
        self.dL = torch.empty_like(self.L)
        need = binding.monarch_bwd_workspace_bytes(sh.B, sh.n_in, sh.k, sh.q, sh.s, self.code, 0)
        self.ws = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
        self.fneed = binding.monarch_fwd_workspace_bytes(sh.B, sh.n_in, sh.k, sh.q, sh.s, self.code, 0)
        self.fws = torch.empty(max(self.fneed, 256), dtype=torch.uint8, device=dev)

    def fwd(self, i):
        from paper_2204_00595_amd import binding
        xs, _, y, _ = self.sets[i % self.nsets]
        binding.monarch_fwd(xs, self.R, self.L, y)

    def bwd(self, i):
        from paper_2204_00595_amd import binding
        xs, dys, _, dx = self.sets[i % self.nsets]
        binding.monarch_bwd(dys, xs, self.R, self.L, dx, self.dR, self.dL, workspace=self.ws)

    def step(self, i):
        self.fwd(i)
        self.bwd(i)


def measure_layer(name: str, with_dense: bool = True, with_extras: bool = False, layer: Layer | None = None,
                  calls: int = TIMED_CALLS, copy_gbs: float | None = None, variants: bool = True):
    """One configuration's block: per-call times of monarch_fwd and monarch_bwd (and of the variants with a
    workspace / a saved intermediate), rooflines, counter traffic, dense comparator."""
    import numpy as np
    import torch
    from paper_2204_00595_amd import binding

    ly = layer or Layer(name)
    sh, code, dev, dt = ly.sh, ly.code, torch.device("cuda:0"), ly.dt
    nsets, sets, Rd, Ld, dR, dL, ws, fws, fneed = ly.nsets, ly.sets, ly.R, ly.L, ly.dR, ly.dL, ly.ws, ly.fws, ly.fneed
    small = sh.fwd_bytes() < (8 << 20)
    if small:
        calls = max(calls, 500)  # microsecond calls: longer runs
    fwd_med, fwd_min, fwd_mean, ncalls = timed_runs(ly.fwd, calls)
    bwd_med, bwd_min, bwd_mean, _ = timed_runs(ly.bwd, calls)
    # the same calls on one buffer set ("warm": repeats can be served by the 256 MB Infinity Cache)
    fwd_warm = timed_runs(lambda i: ly.fwd(0), calls // 2)[0] if variants else None
    bwd_warm = timed_runs(lambda i: ly.bwd(0), calls // 2)[0] if variants else None

    def fwd_ws_only(i):
        xs, _, y, _ = sets[i % nsets]
        binding.monarch_fwd_ws(xs, Rd, Ld, y, workspace=fws)

    def fwd_ws_packed(i):
        xs, _, y, _ = sets[i % nsets]
        binding.monarch_fwd_ws(xs, Rd, Ld, y, workspace=fws, flags=binding.MONARCH_FLAG_WS_PACKED)

    fwd_ws_ms = timed_runs(fwd_ws_only, calls // 2)[0] if fneed else None
    fwd_ws_packed_ms = timed_runs(fwd_ws_packed, calls // 2)[0] if fneed else None

    # forward that saves the vector between the factors + backward that reads it instead of recomputing
    sneed = binding.monarch_saved_bytes(sh.B, sh.n_in, sh.k, sh.q, sh.s, code, 0) if variants else 0
    fwd_save_ms = bwd_saved_ms = None
    if sneed:
        svs = [torch.empty(sneed, dtype=torch.uint8, device=dev) for _ in range(nsets)]

        def fwd_save_only(i):
            xs, _, y, _ = sets[i % nsets]
            binding.monarch_fwd_save(xs, Rd, Ld, y, svs[i % nsets])

        def bwd_saved_only(i):
            xs, dys, _, dx = sets[i % nsets]
            binding.monarch_bwd_saved(dys, xs, svs[i % nsets], Rd, Ld, dx, dR, dL, workspace=ws)

        fwd_save_ms = timed_runs(fwd_save_only, calls // 2)[0]
        bwd_saved_ms = timed_runs(bwd_saved_only, calls // 2)[0]
        del svs

    out = {
        "workload": name, "shape": "k=%d p=%d q=%d s=%d (%d->%d), B=%d, %s" % (sh.k, sh.p, sh.q, sh.s, sh.n_in, sh.n_out, sh.B, sh.dtype),
        "timed_calls": ncalls, "statistic": "median / min over %d runs of %d consecutive calls (time per call of a run)" % (RUNS, ncalls // RUNS),
        "fwd_us": fwd_med * 1e3, "fwd_us_min": fwd_min * 1e3, "bwd_us": bwd_med * 1e3, "bwd_us_min": bwd_min * 1e3,
        "fwd_us_warm": fwd_warm and fwd_warm * 1e3, "bwd_us_warm": bwd_warm and bwd_warm * 1e3,  # one buffer set instead of the rotation: cache-assisted
        "fwd_kernel": binding.monarch_kernel_name(0, sh.n_in, sh.k, sh.q, sh.s, code),
        "bwd_kernel": binding.monarch_kernel_name(1, sh.n_in, sh.k, sh.q, sh.s, code),
        # monarch_fwd_ws (weights packed into a caller workspace, pack included / pack skipped); null without such a kernel
        "fwd_ws_us": fwd_ws_ms and fwd_ws_ms * 1e3, "fwd_ws_packed_us": fwd_ws_packed_ms and fwd_ws_packed_ms * 1e3,
        "fwd_ws_kernel": binding.monarch_kernel_name(2, sh.n_in, sh.k, sh.q, sh.s, code),
        # monarch_fwd_save / monarch_bwd_saved (the intermediate goes through HBM once instead of being recomputed)
        "fwd_save_us": fwd_save_ms and fwd_save_ms * 1e3, "bwd_saved_us": bwd_saved_ms and bwd_saved_ms * 1e3,
        "fwd_tflops": sh.fwd_flops() / (fwd_med * 1e-3) / 1e12, "bwd_tflops": sh.bwd_flops() / (bwd_med * 1e-3) / 1e12,
        "fwd_gbs": sh.fwd_bytes() / (fwd_med * 1e-3) / 1e9, "bwd_gbs": sh.bwd_bytes() / (bwd_med * 1e-3) / 1e9,
        "fwd_algorithmic_bytes": sh.fwd_bytes(), "bwd_algorithmic_bytes": sh.bwd_bytes(),
        "rotating_sets": nsets,
    }
    for ps, ms in (("fwd", fwd_med), ("bwd", bwd_med)):
        frac, bound = roofline_of(sh, ps, ms)
        out[ps + "_roofline_frac"] = frac
        out[ps + "_bound"] = bound
        if copy_gbs:
            # the same fraction with the measured copy rate in place of the nominal 8 TB/s
            out[ps + "_frac_of_copy_roof"] = out[ps + "_gbs"] / copy_gbs if bound == "hbm" else None
        t = traffic_of(name, "monarch_" + ps)
        out[ps + "_traffic_bytes"] = t  # rocprofv3 FETCH_SIZE + WRITE_SIZE per call (profiles/), null if not profiled
        out[ps + "_traffic_ratio"] = (t / out[ps + "_algorithmic_bytes"]) if t else None
    if small and variants:
        out["note"] = ("launch-latency bound: %d KB and %.1f MFLOP per forward; the eager per-call times above include the host's "
                       "cost of issuing a launch from Python (see launch_floor_us); *_us_graph are the same calls replayed from a "
                       "captured HIP graph" % (sh.fwd_bytes() // 1000, sh.fwd_flops() / 1e6))
        out["fwd_us_graph"], out["fwd_us_graph_min"] = (v * 1e3 for v in graph_time(ly.fwd))
        out["bwd_us_graph"], out["bwd_us_graph_min"] = (v * 1e3 for v in graph_time(ly.bwd))

    if with_dense:
        # vendor dense GEMM of the same (B, n_in, n_out): 1 GEMM forward, 2 GEMMs backward
        W = torch.randn(sh.n_out, sh.n_in, device=dev, dtype=dt)

        def dense_fwd(i):
            sets[i % nsets][0] @ W.t()

        def dense_bwd(i):
            xs, dys, _, _ = sets[i % nsets]
            dys @ W
            dys.t() @ xs

        out["dense_fwd_us"] = timed_runs(dense_fwd, calls // 2)[0] * 1e3
        out["dense_bwd_us"] = timed_runs(dense_bwd, calls // 2)[0] * 1e3
        out["speedup_vs_dense"] = (out["dense_fwd_us"] + out["dense_bwd_us"]) / (out["fwd_us"] + out["bwd_us"])
    if with_extras:
        out["extras"] = measure_extras(ly, calls // 2)
    return out


def measure_extras(ly: Layer, calls: int):
    """Per-call times of the other entry points on the workload's shape (ms): affine layer, transposed multiply,
    dense form, and for square shapes the complex multiply and the projection."""
    import torch
    from paper_2204_00595_amd import binding, synth
    sh, code, dev, dt = ly.sh, ly.code, torch.device("cuda:0"), ly.dt
    nsets, sets, Rd, Ld, dR, dL, ws, fws, fneed = ly.nsets, ly.sets, ly.R, ly.L, ly.dR, ly.dL, ly.ws, ly.fws, ly.fneed
    ex = {}
    biasd = torch.from_numpy(synth.quantize(synth.normal(4242, (sh.n_out,)), sh.dtype)).to(dev).to(dt)
    dbias = torch.empty_like(biasd)

    def fwd_bias_only(i):
        xs, _, y, _ = sets[i % nsets]
        binding.monarch_fwd_bias(xs, Rd, Ld, biasd, y, workspace=fws if fneed else None)

    def fwd_then_add(i):
        xs, _, y, _ = sets[i % nsets]
        if fneed:
            binding.monarch_fwd_ws(xs, Rd, Ld, y, workspace=fws)
        else:
            binding.monarch_fwd(xs, Rd, Ld, y)
        y.add_(biasd)

    def bwd_bias_only(i):
        xs, dys, _, dx = sets[i % nsets]
        binding.monarch_bwd_bias(dys, xs, Rd, Ld, dx, dR, dL, dbias, workspace=ws)

    # the layer with the block's nonlinearity: forward writing pre-activation and activation, backward taking both
    hbuf = [torch.empty_like(st[2]) for st in sets[:min(nsets, 2)]]
    xpre = [torch.empty_like(st[0]).normal_() for st in sets[:min(nsets, 2)]]

    def fwd_gelu_only(i):
        xs, _, y, _ = sets[i % nsets]
        binding.monarch_fwd_bias_gelu(xs, Rd, Ld, biasd, hbuf[i % len(hbuf)], y, workspace=fws if fneed else None)

    def bwd_gelu_in_only(i):
        xs, dys, _, dx = sets[i % nsets]
        binding.monarch_bwd_bias_gelu_in(dys, xs, xpre[i % len(xpre)], Rd, Ld, dx, dR, dL, dbias, workspace=ws)

    ex["fwd_bias_gelu_ms"] = timed_runs(fwd_gelu_only, calls)[0]
    ex["bwd_bias_gelu_in_ms"] = timed_runs(bwd_gelu_in_only, calls)[0]
    del hbuf, xpre
    ex["fwd_bias_ms"] = timed_runs(fwd_bias_only, calls)[0]
    ex["fwd_then_add_ms"] = timed_runs(fwd_then_add, calls)[0]   # forward with workspace + a separate framework add
    ex["bwd_bias_ms"] = timed_runs(bwd_bias_only, calls)[0]
    tneed = binding.monarch_fwd_t_workspace_bytes(sh.B, sh.n_in, sh.k, sh.q, sh.s, code, 0)
    tws = torch.empty(max(tneed, 256), dtype=torch.uint8, device=dev)

    def fwd_t_only(i):
        _, dys, _, dx = sets[i % nsets]
        binding.monarch_fwd_t(dys, Rd, Ld, dx, workspace=tws if tneed else None)

    ex["fwd_t_ms"] = timed_runs(fwd_t_only, calls)[0]
    ex["fwd_t_kernel"] = binding.monarch_kernel_name(3, sh.n_in, sh.k, sh.q, sh.s, code)
    Mdense = torch.empty((sh.n_out, sh.n_in), dtype=Rd.dtype, device="cuda")
    ex["to_dense_ms"] = timed_runs(lambda i: binding.monarch_to_dense(Rd, Ld, Mdense), calls)[0]
    dense_bytes = (sh.k * sh.q * sh.p + sh.k * sh.s * sh.q + sh.n_out * sh.n_in) * sh.esize
    ex["to_dense_gbs"] = dense_bytes / (ex["to_dense_ms"] * 1e-3) / 1e9
    if sh.k == sh.p == sh.q == sh.s:
        # complex64 multiply with the DFT factors on the first rows of the batch
        crow = min(sh.B, 2048)
        cx = torch.randn((crow, sh.n_in), dtype=torch.complex64, device=dev, generator=torch.Generator(device=dev).manual_seed(7))
        cR, cL = binding.monarch_dft_factors(sh.k, False, device=dev)
        cy = torch.empty_like(cx)
        cdx, cdR, cdL = torch.empty_like(cx), torch.empty_like(cR), torch.empty_like(cL)
        cneed = binding.monarch_c64_workspace_bytes(binding.C64_BWD, crow, sh.n_in, sh.k, sh.q, sh.s)
        cws = torch.empty(max(cneed, 256), dtype=torch.uint8, device=dev)
        ex["c64_fwd_ms"] = timed_runs(lambda i: binding.monarch_fwd_c64_ws(cx, cR, cL, cy, workspace=cws), 20, 2)[0]
        ex["c64_fwd_h_ms"] = timed_runs(lambda i: binding.monarch_fwd_h_c64_ws(cx, cR, cL, cy, workspace=cws), 20, 2)[0]
        ex["c64_bwd_ms"] = timed_runs(lambda i: binding.monarch_bwd_c64_ws(cy, cx, cR, cL, cdx, cdR, cdL, workspace=cws), 20, 2)[0]
        # the calls without a workspace (shape-generic fp32 kernels, weight gradients through atomics)
        ex["c64_fwd_noworkspace_ms"] = timed_runs(lambda i: binding.monarch_fwd_c64(cx, cR, cL, cy), 5, 2)[0]
        ex["c64_bwd_noworkspace_ms"] = timed_runs(lambda i: binding.monarch_bwd_c64(cy, cx, cR, cL), 5, 2)[0]
        ex["c64_rows"] = crow
        # 8 real flops per complex multiply-add, two factors forward, six block products backward
        cflops = 8.0 * crow * sh.k * (sh.q * sh.p + sh.s * sh.q)
        ex["c64_fwd_tflops"] = cflops / (ex["c64_fwd_ms"] * 1e-3) / 1e12
        ex["c64_bwd_tflops"] = 2.5 * cflops / (ex["c64_bwd_ms"] * 1e-3) / 1e12
        del cws, cdx
        if sh.p in (32, 64):
            # the same layer in fp32 (fp32 matrix-core stage kernels), whole batch
            fx = torch.randn((sh.B, sh.n_in), dtype=torch.float32, device=dev, generator=torch.Generator(device=dev).manual_seed(8))
            fR, fL = Rd.float(), Ld.float()
            fy, fdx, fdR, fdL = torch.empty_like(fx), torch.empty_like(fx), torch.empty_like(fR), torch.empty_like(fL)
            fwn = binding.monarch_fwd_workspace_bytes(sh.B, sh.n_in, sh.k, sh.q, sh.s, 0, 0)
            bwn = binding.monarch_bwd_workspace_bytes(sh.B, sh.n_in, sh.k, sh.q, sh.s, 0, 0)
            fws2 = torch.empty(max(fwn, bwn, 256), dtype=torch.uint8, device=dev)
            ex["f32_fwd_ms"] = timed_runs(lambda i: binding.monarch_fwd_ws(fx, fR, fL, fy, workspace=fws2), 10, 2)[0]
            ex["f32_bwd_ms"] = timed_runs(lambda i: binding.monarch_bwd(fy, fx, fR, fL, fdx, fdR, fdL, workspace=fws2), 10, 2)[0]
            ex["f32_fwd_kernel"] = binding.monarch_kernel_name(2, sh.n_in, sh.k, sh.q, sh.s, 0)
            ex["f32_fwd_tflops"] = sh.fwd_flops() / (ex["f32_fwd_ms"] * 1e-3) / 1e12
            del fx, fy, fdx, fws2
        # Algorithm 1 on a dense Gaussian n x n matrix: one Jacobi SVD per slice
        Adense = torch.from_numpy(synth.quantize(synth.normal(4343, (sh.n_in, sh.n_in)), sh.dtype)).to(dev).to(dt)
        Rp, Lp = torch.empty_like(Rd), torch.empty_like(Ld)
        ex["project_ms"] = timed_runs(lambda i: binding.monarch_project(Adense, Rp, Lp), 20, 2)[0]
    return ex


class Pair:
    """The MLP pair: fc1 and fc2 chained through the hidden activation, with rotating buffer sets."""

    def __init__(self):
        import torch
        from paper_2204_00595_amd import binding, synth
        s1, s2 = synth.WORKLOADS["gpt2m_fc1"], synth.WORKLOADS["gpt2m_fc2"]
        self.s1, self.s2 = s1, s2
        dev, dt = torch.device("cuda:0"), torch.bfloat16
        B = s1.B
        g = _gen_rows(B)
        x, R1, L1, _ = synth.make_inputs(s1, rows=g)
        _, R2, L2, dy = synth.make_inputs(s2, rows=g)
        self.R1, self.L1, self.R2, self.L2 = (torch.from_numpy(a).to(dev).to(dt) for a in (R1, L1, R2, L2))
        x0, dy0 = (torch.from_numpy(a).to(dev).to(dt).repeat(B // g, 1) for a in (x, dy))
        per_set = 2 * B * (3 * s1.n_in + 2 * s1.n_out + 0) + 2 * B * s2.n_out
        self.nsets = max(2, -(-ROTATE_BYTES // per_set))
        self.sets = []
        for i in range(self.nsets):
            xs = x0 if i == 0 else x0.roll(i, 0).contiguous()
            dys = dy0 if i == 0 else dy0.roll(i, 0).contiguous()
            h = torch.empty((B, s1.n_out), dtype=dt, device=dev)
            self.sets.append((xs, dys, h, torch.empty((B, s2.n_out), dtype=dt, device=dev), torch.empty_like(h), torch.empty_like(xs)))
        self.g = [torch.empty_like(t) for t in (self.R1, self.L1, self.R2, self.L2)]
        need = max(binding.monarch_bwd_workspace_bytes(B, s.n_in, s.k, s.q, s.s, 1, 0) for s in (s1, s2))
        self.ws = torch.empty(need, dtype=torch.uint8, device=dev)

    def flops(self):
        return sum(s.fwd_flops() + s.bwd_flops() for s in (self.s1, self.s2))

    def nbytes(self):
        return sum(s.fwd_bytes() + s.bwd_bytes() for s in (self.s1, self.s2))

    def calls(self, i):
        """The four calls of step i as (label, shape, pass, thunk)."""
        from paper_2204_00595_amd import binding
        xs, dys, h, y, dh, dx = self.sets[i % self.nsets]
        dR1, dL1, dR2, dL2 = self.g
        return (
            # the forward with a workspace: the weights are re-packed inside every call (they change every step)
            ("fwd_fc1", self.s1, "fwd", lambda: binding.monarch_fwd_ws(xs, self.R1, self.L1, h, workspace=self.ws)),
            ("fwd_fc2", self.s2, "fwd", lambda: binding.monarch_fwd_ws(h, self.R2, self.L2, y, workspace=self.ws)),
            ("bwd_fc2", self.s2, "bwd", lambda: binding.monarch_bwd(dys, h, self.R2, self.L2, dh, dR2, dL2, workspace=self.ws)),
            ("bwd_fc1", self.s1, "bwd", lambda: binding.monarch_bwd(dh, xs, self.R1, self.L1, dx, dR1, dL1, workspace=self.ws)),
        )

    def step(self, i):
        for _, _, _, fn in self.calls(i):
            fn()


def measure_ffn_block():
    """The feed-forward block of GPT-2 medium around the pair: biases and the nonlinearity (tanh-form GELU) between
    the layers, forward and backward, 16384 rows.  `fused`: the nonlinearity runs in the layers' own epilogues
    (monarch_fwd_bias_gelu, monarch_bwd_bias_gelu_in); `separate_passes`: the plain layer calls with the
    framework's elementwise gelu / gelu_backward kernels between them."""
    import torch
    from paper_2204_00595_amd import binding, synth
    s1, s2 = synth.WORKLOADS["gpt2m_fc1"], synth.WORKLOADS["gpt2m_fc2"]
    dev, dt = torch.device("cuda:0"), torch.bfloat16
    B = s1.B
    g = _gen_rows(B)
    x, R1, L1, _ = synth.make_inputs(s1, rows=g)
    _, R2, L2, dy = synth.make_inputs(s2, rows=g)
    R1, L1, R2, L2 = (torch.from_numpy(a).to(dev).to(dt) for a in (R1, L1, R2, L2))
    b1 = torch.from_numpy(synth.quantize(synth.normal(811, (s1.n_out,)), "bf16")).to(dev).to(dt)
    b2 = torch.from_numpy(synth.quantize(synth.normal(812, (s2.n_out,)), "bf16")).to(dev).to(dt)
    x0, dy0 = (torch.from_numpy(a).to(dev).to(dt).repeat(B // g, 1) for a in (x, dy))
    sets = []
    for i in range(2):
        xs = x0 if i == 0 else x0.roll(i, 0).contiguous()
        dys = dy0 if i == 0 else dy0.roll(i, 0).contiguous()
        hid = lambda: torch.empty((B, s1.n_out), dtype=dt, device=dev)
        sets.append((xs, dys, hid(), hid(), torch.empty((B, s2.n_out), dtype=dt, device=dev), hid(), torch.empty_like(xs)))
    gR1, gL1, gR2, gL2, gb1, gb2 = (torch.empty_like(t) for t in (R1, L1, R2, L2, b1, b2))
    fneed = max(binding.monarch_fwd_workspace_bytes(B, s.n_in, s.k, s.q, s.s, 1, 0) for s in (s1, s2))
    bneed = max(binding.monarch_bwd_workspace_bytes(B, s.n_in, s.k, s.q, s.s, 1, 0) for s in (s1, s2))
    ws = torch.empty(max(fneed, bneed), dtype=torch.uint8, device=dev)

    def fused(i):
        xs, dys, h, a, y, dh, dx = sets[i % 2]
        binding.monarch_fwd_bias_gelu(xs, R1, L1, b1, h, a, workspace=ws)
        binding.monarch_fwd_bias(a, R2, L2, b2, y, workspace=ws)
        binding.monarch_bwd_bias_gelu_in(dys, a, h, R2, L2, dh, gR2, gL2, gb2, workspace=ws)
        binding.monarch_bwd_bias(dh, xs, R1, L1, dx, gR1, gL1, gb1, workspace=ws)

    def separate(i):
        xs, dys, h, a, y, dh, dx = sets[i % 2]
        binding.monarch_fwd_bias(xs, R1, L1, b1, h, workspace=ws)
        torch.ops.aten.gelu.out(h, approximate="tanh", out=a)
        binding.monarch_fwd_bias(a, R2, L2, b2, y, workspace=ws)
        binding.monarch_bwd_bias(dys, a, R2, L2, dh, gR2, gL2, gb2, workspace=ws)
        torch.ops.aten.gelu_backward.grad_input(dh, h, approximate="tanh", grad_input=dh)
        binding.monarch_bwd_bias(dh, xs, R1, L1, dx, gR1, gL1, gb1, workspace=ws)

    fmed, fmin, _, n = timed_runs(fused, 50)
    smed, smin, _, _ = timed_runs(separate, 50)
    flops = sum(s.fwd_flops() + s.bwd_flops() for s in (s1, s2))
    return {"workload": "gpt2m feed-forward block 1024->4096->gelu->1024 with biases, B=%d, bf16, fwd+bwd" % B,
            "fused_epilogues_us": fmed * 1e3, "fused_epilogues_us_min": fmin * 1e3,
            "separate_passes_us": smed * 1e3, "separate_passes_us_min": smin * 1e3,
            "timed_steps": n, "fused_tflops": flops / (fmed * 1e-3) / 1e12,
            "note": "separate_passes = the same layer calls with the framework's elementwise gelu and gelu_backward "
                    "kernels between them (one more read and one more write of the hidden activation forward, "
                    "two reads and a write backward)"}


def cpu_baseline(workload: str, cpu_seconds: float = 20.0):
    """The CPU oracle as it stands, timed on this host: the same step (for the pair: both layers, forward and
    backward, chained in fp64) over the first rows of the workload, sized to about `cpu_seconds` core-seconds."""
    import oracle
    from paper_2204_00595_amd import synth

    cores = oracle.num_threads()
    if workload == PAIR:
        shapes = [synth.WORKLOADS["gpt2m_fc1"], synth.WORKLOADS["gpt2m_fc2"]]
    else:
        shapes = [synth.workload(workload)]
    Bfull = shapes[0].B

    def make(rows):
        ins = [synth.make_inputs(s, rows=rows) for s in shapes]
        return ins

    def run(ins):
        if len(ins) == 1:
            x, R, L, dy = ins[0]
            oracle.fwd(x, R, L)
            oracle.bwd(dy, x, R, L)
        else:
            (x, R1, L1, _), (_, R2, L2, dy) = ins
            h = oracle.fwd(x, R1, L1)
            oracle.fwd(h, R2, L2)
            dh = oracle.bwd(dy, h, R2, L2)[0]
            oracle.bwd(dh, x, R1, L1)

    rows = min(Bfull, 256 if workload == PAIR else 2048)
    ins = make(rows)
    t0 = time.perf_counter()
    run(ins)
    probe = time.perf_counter() - t0
    wall_budget = cpu_seconds / max(cores, 1)
    rows2 = max(rows, min(Bfull, min(65536, int(rows * wall_budget / max(probe, 1e-4)))))
    if rows2 != rows:
        ins = make(rows2)
    reps, dt_s = 0, 0.0
    while reps == 0 or (dt_s < wall_budget and reps < 200):
        t0 = time.perf_counter()
        run(ins)
        dt_s += time.perf_counter() - t0
        reps += 1
    flops = sum(s.fwd_flops() + s.bwd_flops() for s in shapes) * rows2 / Bfull * reps
    return {"value": flops / dt_s / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": "fwd+bwd (%s) of the first %d of %d rows of %s, fp64, %d repetition(s), %.2f s wall on %d threads"
                      % ("both layers chained" if len(shapes) == 2 else "one layer", rows2, Bfull, workload, reps, dt_s, cores)}


def progress(msg: str):
    """One line on stderr per stage (flushed): if a run dies, the last line names the stage."""
    sys.stderr.write("[bench] %s\n" % msg)
    sys.stderr.flush()


def main():
    try:
        _main()
    finally:
        # never leave the process with kernels still queued (an exception above included): the library's code
        # objects are unloaded at exit
        try:
            import torch
            if torch.cuda.is_available():
                torch.cuda.synchronize()
        except Exception as e:  # the original error, if any, is the one to report
            sys.stderr.write("[bench] synchronize at exit failed: %r\n" % (e,))


def _main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=PAIR, help="the step: %s (default) or one of %s" % (PAIR, ", ".join(CONFIGS)))
    ap.add_argument("--only", action="store_true", help="measure the step's workload only, not every configuration")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--extras", action="store_true", help="also time the other entry points (bias, transposed, dense form, complex, projection)")
    ap.add_argument("--no-variants", action="store_true",
                    help="time monarch_fwd, monarch_fwd_ws and monarch_bwd only (profiler runs: one kernel set per call)")
    ap.add_argument("--layers", action="store_true", help="also time the other layer shapes of the same models (extra keys)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.stderr.write("bench.py: this library runs on ONE GPU; --gpus N with N > 1 is not supported "
                         "(a multi-GPU run would shard the batch rows and all-reduce dR, dL; nothing of that is built).\n")
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2204_00595_amd import binding, synth
    if not torch.cuda.is_available():
        sys.stderr.write("bench.py needs a GPU\n")
        sys.exit(2)
    binding.lib()
    progress("copy roof")
    copy_gbs = copy_roof()
    detail = {}
    progress("building inputs of %s" % args.workload)

    if args.workload == PAIR:
        job = Pair()
        step, flops, nbytes, dtype = job.step, job.flops(), job.nbytes(), "bf16"
        s1, s2 = job.s1, job.s2
        wl_text = ("%s: MLP pair 1024->4096->1024 (fc1 k=4 p=q=256 s=1024; fc2 k=4 p=1024 q=s=256), B=%d rows, bf16, "
                   "monarch_fwd_ws fc1 + monarch_fwd_ws fc2 + monarch_bwd fc2 + monarch_bwd fc1 (weights re-packed in every call), "
                   "no nonlinearity between the multiplies" % (PAIR, s1.B))
    else:
        job = Layer(args.workload)
        step, sh = job.step, job.sh
        flops, nbytes, dtype = sh.fwd_flops() + sh.bwd_flops(), sh.fwd_bytes() + sh.bwd_bytes(), sh.dtype
        wl_text = "%s: k=%d p=%d q=%d s=%d (%d->%d), B=%d rows, fwd+bwd" % (sh.name, sh.k, sh.p, sh.q, sh.s, sh.n_in, sh.n_out, sh.B)

    progress("warm-up: %d steps" % args.warmup)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    progress("timed: %d steps" % args.steps)
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3
    progress("%.4f ms per step; per-call timings" % ms_per_step)

    # per-call durations of the step's calls: runs of consecutive calls of one entry point between two events
    if args.workload == PAIR:
        # the hidden activation and its gradient must exist before the backward calls are timed alone
        for i in range(job.nsets):
            job.step(i)
        per_call = {}
        for idx in range(4):
            label, shp, ps, _ = job.calls(0)[idx]
            med, mn, _, n = timed_runs(lambda i, idx=idx: job.calls(i)[idx][3](), TIMED_CALLS)
            frac, bound = roofline_of(shp, ps, med)
            per_call[label] = {"us": med * 1e3, "us_min": mn * 1e3, "timed_calls": n, "roofline_frac": frac, "bound": bound,
                               "workload": shp.name, "pass": ps,
                               "flops": shp.fwd_flops() if ps == "fwd" else shp.bwd_flops(),
                               "bytes": shp.fwd_bytes() if ps == "fwd" else shp.bwd_bytes()}
        detail["step_calls"] = per_call
        dom_label = max(per_call, key=lambda k_: per_call[k_]["us"])
        dom = per_call[dom_label]
        dom_sh, dom_ps = (s2 if dom["workload"] == "gpt2m_fc2" else s1), dom["pass"]
    else:
        fmed, fmin, _, n = timed_runs(job.fwd, TIMED_CALLS)
        bmed, bmin, _, _ = timed_runs(job.bwd, TIMED_CALLS)
        per_call = {}
        for label, ps, med, mn in (("fwd", "fwd", fmed, fmin), ("bwd", "bwd", bmed, bmin)):
            frac, bound = roofline_of(sh, ps, med)
            per_call[label] = {"us": med * 1e3, "us_min": mn * 1e3, "timed_calls": n, "roofline_frac": frac, "bound": bound,
                               "workload": sh.name, "pass": ps,
                               "flops": sh.fwd_flops() if ps == "fwd" else sh.bwd_flops(),
                               "bytes": sh.fwd_bytes() if ps == "fwd" else sh.bwd_bytes()}
        detail["step_calls"] = per_call
        dom_label = max(per_call, key=lambda k_: per_call[k_]["us"])
        dom = per_call[dom_label]
        dom_sh, dom_ps = sh, dom["pass"]

    # roofline of the dominant call (the one with the largest duration)
    dom_ms = dom["us"] * 1e-3
    if dom["bound"] == "hbm":
        roof = {"bound": "hbm", "achieved": dom["bytes"] / (dom_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    else:
        roof = {"bound": "mfma", "achieved": dom["flops"] / (dom_ms * 1e-3) / 1e12, "peak": MFMA_PEAK_TFLOPS[dom_sh.dtype], "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    # HBM bytes per call measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (calibrated on the copy kernel)
    # by the committed profile of this workload; null when no such profile has been taken
    dom_entry = "monarch_bwd" if dom_ps == "bwd" else ("monarch_fwd_ws" if args.workload == PAIR else "monarch_fwd")
    roof["traffic"] = traffic_of(dom_sh.name, dom_entry)
    roof["traffic_unit"] = "bytes per call"
    roof["algorithmic_bytes"] = dom["bytes"]
    roof["algorithmic_flops"] = dom["flops"]
    code = 0 if dom_sh.dtype == "f32" else 1
    roof["kernel"] = binding.monarch_kernel_name(0 if dom_ps == "fwd" else 1, dom_sh.n_in, dom_sh.k, dom_sh.q, dom_sh.s, code)
    roof["call"] = "%s on %s" % (dom_entry, dom_sh.name)
    roof["avg_ms"] = dom_ms
    roof["frac_of_copy_roof"] = (roof["achieved"] / copy_gbs) if roof["bound"] == "hbm" else None
    del job
    torch.cuda.empty_cache()

    progress("launch floor")
    floor = launch_floor()
    detail["launch_floor_us"] = floor
    names = [args.workload] if (args.only and args.workload != PAIR) else ([] if args.only else list(CONFIGS))
    configs = {}
    for name in names:
        progress("configuration %s" % name)
        configs[name] = measure_layer(name, with_dense=not args.no_dense, with_extras=args.extras, copy_gbs=copy_gbs,
                                      variants=not args.no_variants)
        if name == "sq256_f32":
            configs[name]["launch_floor_us"] = floor["median_us"]
        torch.cuda.empty_cache()
    detail["configs"] = configs
    if not args.only and not args.no_variants:
        progress("feed-forward block with the nonlinearity")
        detail["ffn_block"] = measure_ffn_block()
        torch.cuda.empty_cache()
    if args.layers:
        detail["model_layers"] = {}
        for name in synth.MODEL_LAYERS:
            detail["model_layers"][name] = measure_layer(name, with_dense=not args.no_dense, with_extras=args.extras, copy_gbs=copy_gbs)
            torch.cuda.empty_cache()

    step_s = ms_per_step * 1e-3
    line = {
        "metric": "monarch_fwd_bwd_tflops", "value": flops / step_s / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "config": {"workload": wl_text},
        "gb_per_s": nbytes / step_s / 1e9,
        "roofline": roof,
        "hbm_copy_gbs": copy_gbs,
        "detail": detail,
    }
    if not args.no_dense:
        # empirical matrix-core roof (vendor GEMM, n = 8192) and the step's share of it
        progress("dense GEMM roof")
        line["dense_gemm_roof_tflops"] = mfma_roof()
        line["frac_of_dense_gemm_roof"] = line["value"] / line["dense_gemm_roof_tflops"][dtype]
    if not args.no_cpu:
        torch.cuda.synchronize()
        progress("CPU oracle baseline")
        line["cpu_baseline"] = cpu_baseline(args.workload)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
