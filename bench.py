#!/usr/bin/env python3
"""Benchmark of the Monarch multiply hot path (forward + backward) on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input:
monarch_fwd followed by monarch_bwd on the workload's shape, inputs resident in HBM.
Prints ONE JSON line (see the keys below).  `--gpus N` with N > 1 is refused: the
library is a single-GPU kernel library.

Timing: K steps bracketed by torch.cuda.synchronize(); per-call durations come from HIP
events recorded on the stream the kernels are launched on (torch's current stream) around a
run of K consecutive calls of one entry point.
Buffers rotate through enough distinct (x, y, dy, dx) sets that the footprint exceeds the
256 MB Infinity Cache, so repeats are served from HBM; the weights stay hot, as they would
in training.
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


def _events(n):
    import torch
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


def run_workload(name: str, steps: int, warmup: int, with_dense: bool = True, with_extras: bool = True):
    import numpy as np
    import torch
    from paper_2204_00595_amd import binding, synth

    sh = synth.workload(name)
    dt = torch.float32 if sh.dtype == "f32" else torch.bfloat16
    code = 0 if sh.dtype == "f32" else 1
    dev = torch.device("cuda:0")
    gen_rows = min(sh.B, 65536)  # larger batches repeat a generated block (timing only)
    x, R, L, dy = synth.make_inputs(sh, rows=gen_rows)
    Rd, Ld = (torch.from_numpy(a).to(dev).to(dt) for a in (R, L))
    x0 = torch.from_numpy(x).to(dev).to(dt).repeat(sh.B // gen_rows, 1)
    dy0 = torch.from_numpy(dy).to(dev).to(dt).repeat(sh.B // gen_rows, 1)
    per_set = sh.esize * sh.B * (2 * sh.n_in + 2 * sh.n_out)
    nsets = max(2, min(64, -(-ROTATE_BYTES // per_set)))
    sets = []
    for i in range(nsets):
        xs = x0 if i == 0 else x0.roll(i, 0).contiguous()
        dys = dy0 if i == 0 else dy0.roll(i, 0).contiguous()
        sets.append((xs, dys, torch.empty((sh.B, sh.n_out), dtype=dt, device=dev), torch.empty_like(xs)))
    dR = torch.empty_like(Rd)
    dL = torch.empty_like(Ld)
    need = binding.monarch_bwd_workspace_bytes(sh.B, sh.n_in, sh.k, sh.q, sh.s, code, 0)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)

    def step(i, ev=None):
        xs, dys, y, dx = sets[i % nsets]
        if ev:
            ev[0].record()
        binding.monarch_fwd(xs, Rd, Ld, y)
        if ev:
            ev[1].record()
        binding.monarch_bwd(dys, xs, Rd, Ld, dx, dR, dL, workspace=ws)
        if ev:
            ev[2].record()

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    # per-call durations: HIP events on the launch stream around a run of `steps` consecutive calls of
    # one entry point (same rotation), so that the events themselves sit outside the timed launches;
    # a single step with an event after every call is kept as the "evented" figure
    def run_of(fn):
        for i in range(3):  # untimed: first launches of a kernel pay for loading it
            fn(i)
        e0, e1 = _events(2)
        e0.record()
        for i in range(steps):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps

    def fwd_only(i):
        xs, _, y, _ = sets[i % nsets]
        binding.monarch_fwd(xs, Rd, Ld, y)

    def bwd_only(i):
        xs, dys, _, dx = sets[i % nsets]
        binding.monarch_bwd(dys, xs, Rd, Ld, dx, dR, dL, workspace=ws)

    # the same calls on one buffer set ("warm": repeats can be served by the 256 MB Infinity Cache)
    fwd_warm = run_of(lambda i: fwd_only(0))
    bwd_warm = run_of(lambda i: bwd_only(0))

    fneed = binding.monarch_fwd_workspace_bytes(sh.B, sh.n_in, sh.k, sh.q, sh.s, code, 0)
    fws = torch.empty(max(fneed, 256), dtype=torch.uint8, device=dev)

    def fwd_ws_only(i):
        xs, _, y, _ = sets[i % nsets]
        binding.monarch_fwd_ws(xs, Rd, Ld, y, workspace=fws)

    def fwd_ws_packed(i):
        xs, _, y, _ = sets[i % nsets]
        binding.monarch_fwd_ws(xs, Rd, Ld, y, workspace=fws, flags=binding.MONARCH_FLAG_WS_PACKED)

    fwd_ws_ms = float(np.mean([run_of(fwd_ws_only) for _ in range(3)])) if fneed else None
    fwd_ws_packed_ms = float(np.mean([run_of(fwd_ws_packed) for _ in range(3)])) if fneed else None
    fwd_bias_ms = fwd_then_add_ms = bwd_bias_ms = to_dense_ms = to_dense_gbs = project_ms = fwd_t_ms = c64_fwd_ms = c64_bwd_ms = c64_rows = None
    fwd_save_ms = bwd_saved_ms = step_saved_ms = None
    if with_extras:
        # forward that saves the vector between the factors + backward that reads it instead of recomputing
        sneed = binding.monarch_saved_bytes(sh.B, sh.n_in, sh.k, sh.q, sh.s, code, 0)
        svs = [torch.empty(sneed, dtype=torch.uint8, device=dev) for _ in range(nsets)] if sneed else None

        def fwd_save_only(i):
            xs, _, y, _ = sets[i % nsets]
            binding.monarch_fwd_save(xs, Rd, Ld, y, svs[i % nsets])

        def bwd_saved_only(i):
            xs, dys, _, dx = sets[i % nsets]
            binding.monarch_bwd_saved(dys, xs, svs[i % nsets], Rd, Ld, dx, dR, dL, workspace=ws)

        def step_saved(i):
            fwd_save_only(i)
            bwd_saved_only(i)

        fwd_save_ms = float(np.mean([run_of(fwd_save_only) for _ in range(3)])) if sneed else None
        bwd_saved_ms = float(np.mean([run_of(bwd_saved_only) for _ in range(3)])) if sneed else None
        step_saved_ms = float(np.mean([run_of(step_saved) for _ in range(3)])) if sneed else None
        # affine layer: bias fused into the forward (where the kernel has the epilogue), bias gradient with the backward;
        # beside them the unfused forms (the plain call, then a separate elementwise add / column sum by the framework)
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

        fwd_bias_ms = float(np.mean([run_of(fwd_bias_only) for _ in range(3)]))
        fwd_then_add_ms = float(np.mean([run_of(fwd_then_add) for _ in range(3)]))
        bwd_bias_ms = float(np.mean([run_of(bwd_bias_only) for _ in range(3)]))
        # transposed multiply x M (monarch_fwd_t): input of the output's shape, result of the input's shape
        tneed = binding.monarch_fwd_t_workspace_bytes(sh.B, sh.n_in, sh.k, sh.q, sh.s, code, 0)
        tws = torch.empty(max(tneed, 256), dtype=torch.uint8, device=dev)

        def fwd_t_only(i):
            _, dys, _, dx = sets[i % nsets]
            binding.monarch_fwd_t(dys, Rd, Ld, dx, workspace=tws if tneed else None)

        fwd_t_ms = float(np.mean([run_of(fwd_t_only) for _ in range(3)]))
        Mdense = torch.empty((sh.n_out, sh.n_in), dtype=Rd.dtype, device="cuda")
        to_dense_ms = float(np.mean([run_of(lambda i: binding.monarch_to_dense(Rd, Ld, Mdense)) for _ in range(3)]))
        dense_bytes = (sh.k * sh.q * sh.p + sh.k * sh.s * sh.q + sh.n_out * sh.n_in) * sh.esize
        to_dense_gbs = dense_bytes / (to_dense_ms * 1e-3) / 1e9
        if sh.k == sh.p == sh.q == sh.s:
            # complex64 multiply with the DFT factors (shape-generic SIMT kernels) on the first rows of the batch
            crow = min(sh.B, 2048)
            cx = torch.randn((crow, sh.n_in), dtype=torch.complex64, device=dev, generator=torch.Generator(device=dev).manual_seed(7))
            cR, cL = binding.monarch_dft_factors(sh.k, False, device=dev)
            cy = torch.empty_like(cx)
            c64_fwd_ms = float(np.mean([run_of(lambda i: binding.monarch_fwd_c64(cx, cR, cL, cy)) for _ in range(2)]))
            c64_bwd_ms = float(np.mean([run_of(lambda i: binding.monarch_bwd_c64(cy, cx, cR, cL)) for _ in range(2)]))
            c64_rows = crow
            # Algorithm 1 on a dense Gaussian n x n matrix (square shapes only): one Jacobi SVD per slice
            Adense = torch.from_numpy(synth.quantize(synth.normal(4343, (sh.n_in, sh.n_in)), sh.dtype)).to(dev).to(dt)
            Rp, Lp = torch.empty_like(Rd), torch.empty_like(Ld)
            project_ms = float(np.mean([run_of(lambda i: binding.monarch_project(Adense, Rp, Lp)) for _ in range(2)]))
    fwd_runs = [run_of(fwd_only) for _ in range(3)]
    bwd_runs = [run_of(bwd_only) for _ in range(3)]
    fwd_ms, bwd_ms = float(np.mean(fwd_runs)), float(np.mean(bwd_runs))
    fwd_min, bwd_min = float(np.min(fwd_runs)), float(np.min(bwd_runs))
    evs = [_events(3) for _ in range(steps)]
    for i in range(steps):
        step(i, evs[i])
    torch.cuda.synchronize()
    fwd_ev = float(np.mean([e[0].elapsed_time(e[1]) for e in evs]))
    bwd_ev = float(np.mean([e[1].elapsed_time(e[2]) for e in evs]))

    out = {
        "workload": name, "ms_per_step": wall / steps * 1e3,
        "fwd_ms": fwd_ms, "bwd_ms": bwd_ms, "fwd_ms_min": fwd_min, "bwd_ms_min": bwd_min,
        "fwd_ms_evented": fwd_ev, "bwd_ms_evented": bwd_ev,
        "fwd_ms_warm": fwd_warm, "bwd_ms_warm": bwd_warm,  # one buffer set instead of the rotation: cache-assisted, not the headline
        # monarch_fwd_ws (weights packed into a caller workspace, pack included); null when the shape has no such kernel
        "fwd_ws_ms": fwd_ws_ms, "fwd_ws_packed_ms": fwd_ws_packed_ms,  # the latter: pack pass skipped (weights unchanged)
        "fwd_ws_kernel": binding.monarch_kernel_name(2, sh.n_in, sh.k, sh.q, sh.s, code),
        # monarch_fwd_bias / monarch_bwd_bias (affine layer); fwd_then_add_ms = forward with workspace + a separate torch add
        "fwd_bias_ms": fwd_bias_ms, "fwd_then_add_ms": fwd_then_add_ms, "bwd_bias_ms": bwd_bias_ms,
        # monarch_to_dense: M written out as a dense (n_out, n_in) matrix; bytes = R + L read, M written
        "to_dense_ms": to_dense_ms, "to_dense_gbs": to_dense_gbs,
        "fwd_t_ms": fwd_t_ms, "fwd_t_kernel": binding.monarch_kernel_name(3, sh.n_in, sh.k, sh.q, sh.s, code),  # monarch_fwd_t
        "c64_fwd_ms": c64_fwd_ms, "c64_bwd_ms": c64_bwd_ms, "c64_rows": c64_rows,  # monarch_fwd_c64 / monarch_bwd_c64 on c64_rows rows
        "project_ms": project_ms,  # monarch_project of a dense n x n matrix (square shapes), else null
        # monarch_fwd_save / monarch_bwd_saved (the intermediate goes through HBM once instead of being recomputed); null without that path
        "fwd_save_ms": fwd_save_ms, "bwd_saved_ms": bwd_saved_ms, "step_saved_ms": step_saved_ms,
        "fwd_kernel": binding.monarch_kernel_name(0, sh.n_in, sh.k, sh.q, sh.s, code),
        "bwd_kernel": binding.monarch_kernel_name(1, sh.n_in, sh.k, sh.q, sh.s, code),
        "fwd_tflops": sh.fwd_flops() / (fwd_ms * 1e-3) / 1e12,
        "bwd_tflops": sh.bwd_flops() / (bwd_ms * 1e-3) / 1e12,
        "fwd_gbs": sh.fwd_bytes() / (fwd_ms * 1e-3) / 1e9,
        "bwd_gbs": sh.bwd_bytes() / (bwd_ms * 1e-3) / 1e9,
        "rotating_sets": nsets,
    }
    for ps, flops, nbytes, ms in (("fwd", sh.fwd_flops(), sh.fwd_bytes(), fwd_ms), ("bwd", sh.bwd_flops(), sh.bwd_bytes(), bwd_ms)):
        t_hbm = nbytes / (HBM_PEAK_GBS * 1e9)
        t_mfma = flops / (MFMA_PEAK_TFLOPS[sh.dtype] * 1e12)
        out[ps + "_roofline_frac"] = max(t_hbm, t_mfma) / (ms * 1e-3)
        out[ps + "_bound"] = "hbm" if t_hbm >= t_mfma else "mfma"

    if with_dense:
        # vendor dense GEMM of the same (B, n_in, n_out): 1 GEMM forward, 2 GEMMs backward
        W = torch.randn(sh.n_out, sh.n_in, device=dev, dtype=dt)
        for _ in range(3):
            sets[0][0] @ W.t()
        torch.cuda.synchronize()
        def dense_fwd(i):
            sets[i % nsets][0] @ W.t()

        def dense_bwd(i):
            xs, dys, _, _ = sets[i % nsets]
            dys @ W
            dys.t() @ xs

        out["dense_fwd_ms"] = float(np.mean([run_of(dense_fwd) for _ in range(2)]))
        out["dense_bwd_ms"] = float(np.mean([run_of(dense_bwd) for _ in range(2)]))
        out["speedup_vs_dense"] = (out["dense_fwd_ms"] + out["dense_bwd_ms"]) / (fwd_ms + bwd_ms)

        # The multiply as the paper runs it (Section 3.3): two framework batched matmuls with the reshapes and
        # transposes between them as separate passes, the intermediate in HBM.  Context for what the fusion buys.
        k, p, q, s_ = sh.k, sh.p, sh.q, sh.s
        Rt = torch.randn(k, q, p, device=dev, dtype=dt)
        Lt = torch.randn(k, s_, q, device=dev, dtype=dt)

        def unfused_fwd(i):
            xs = sets[i % nsets][0]
            y1 = torch.bmm(xs.view(-1, k, p).transpose(0, 1), Rt.transpose(1, 2))        # (k, B, q)
            u = y1.permute(1, 2, 0).reshape(-1, k, q).transpose(0, 1)                      # (q, k) grid, k chunks of q
            w = torch.bmm(u, Lt.transpose(1, 2))                                           # (k, B, s)
            return w.permute(1, 2, 0).reshape(-1, s_ * k)                                  # y[b, l*k + c]

        unfused_fwd(0)
        torch.cuda.synchronize()
        out["unfused_bmm_fwd_ms"] = float(np.mean([run_of(unfused_fwd) for _ in range(2)]))
    return sh, out


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


def cpu_baseline(name: str, cpu_seconds: float = 20.0):
    """The CPU oracle as it stands, timed on this host: forward + backward over the first rows of the
    workload (the whole batch when it is cheap enough, then repeated), sized to about `cpu_seconds`
    core-seconds of work in total."""
    import oracle
    from paper_2204_00595_amd import synth

    sh = synth.WORKLOADS[name]
    cores = oracle.num_threads()
    rows = min(sh.B, 2048)
    x, R, L, dy = synth.make_inputs(sh, rows=rows)
    t0 = time.perf_counter()
    oracle.fwd(x, R, L)
    oracle.bwd(dy, x, R, L)
    probe = time.perf_counter() - t0
    wall_budget = cpu_seconds / max(cores, 1)
    rows2 = max(rows, min(sh.B, min(65536, int(rows * wall_budget / max(probe, 1e-4)))))
    if rows2 != rows:
        x, R, L, dy = synth.make_inputs(sh, rows=rows2)
    reps, dt_s = 0, 0.0
    while reps == 0 or (dt_s < wall_budget and reps < 200):
        t0 = time.perf_counter()
        oracle.fwd(x, R, L)
        oracle.bwd(dy, x, R, L)
        dt_s += time.perf_counter() - t0
        reps += 1
    flops = (sh.fwd_flops() + sh.bwd_flops()) * rows2 / sh.B * reps
    return {"value": flops / dt_s / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": "fwd+bwd of the first %d of %d rows of %s, fp64, %d repetition(s), %.2f s wall on %d threads"
                      % (rows2, sh.B, name, reps, dt_s, cores)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="vitb_proj")
    ap.add_argument("--all", action="store_true", help="also time the other workloads (extra keys)")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--layers", action="store_true", help="also time the other layer shapes of the same models (extra keys)")
    ap.add_argument("--no-extras", action="store_true", help="skip the timings of monarch_to_dense and of the bias calls")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.stderr.write("bench.py: this library runs on ONE GPU; --gpus N with N > 1 is not supported "
                         "(a multi-GPU run would shard the batch rows and all-reduce dR, dL; nothing of that is built).\n")
        sys.exit(2)
    import torch
    from paper_2204_00595_amd import binding
    if not torch.cuda.is_available():
        sys.stderr.write("bench.py needs a GPU\n")
        sys.exit(2)
    binding.lib()

    sh, r = run_workload(args.workload, args.steps, args.warmup, with_dense=not args.no_dense, with_extras=not args.no_extras)
    flops = sh.fwd_flops() + sh.bwd_flops()
    nbytes = sh.fwd_bytes() + sh.bwd_bytes()
    step_s = r["ms_per_step"] * 1e-3
    # roofline of the dominant call (the one with the larger duration)
    dom = "bwd" if r["bwd_ms"] >= r["fwd_ms"] else "fwd"
    dom_bytes = sh.bwd_bytes() if dom == "bwd" else sh.fwd_bytes()
    dom_flops = sh.bwd_flops() if dom == "bwd" else sh.fwd_flops()
    dom_ms = r[dom + "_ms"]
    if r[dom + "_bound"] == "hbm":
        roof = {"bound": "hbm", "achieved": dom_bytes / (dom_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    else:
        roof = {"bound": "mfma", "achieved": dom_flops / (dom_ms * 1e-3) / 1e12,
                "peak": MFMA_PEAK_TFLOPS[sh.dtype], "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    # HBM bytes per call measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (calibrated on the copy
    # kernel) by the committed profile of this workload; null when no such profile has been taken
    roof["traffic"] = None
    if os.path.exists(TRAFFIC_JSON):
        t = json.load(open(TRAFFIC_JSON)).get(args.workload, {}).get("monarch_" + dom)
        if t:
            roof["traffic"] = t["fetch_bytes"] + t["write_bytes"]
            roof["traffic_unit"] = "bytes per call"
            roof["algorithmic_bytes"] = dom_bytes
    roof["kernel"] = r[dom + "_kernel"]
    roof["call"] = "monarch_" + dom
    roof["avg_ms"] = dom_ms
    line = {
        "metric": "monarch_fwd_bwd_tflops", "value": flops / step_s / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": r["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": sh.dtype, "data": "synthetic",
        "config": {"workload": "%s: k=%d p=%d q=%d s=%d (%d->%d), B=%d rows, fwd+bwd" % (
            sh.name, sh.k, sh.p, sh.q, sh.s, sh.n_in, sh.n_out, sh.B)},
        "gb_per_s": nbytes / step_s / 1e9,
        "roofline": roof,
        "detail": r,
    }
    if r.get("step_saved_ms"):
        # the same step through monarch_fwd_save + monarch_bwd_saved (intermediate kept in HBM, not recomputed);
        # same FLOP count as the headline (the recompute is not counted there either)
        line["step_with_saved_intermediate"] = {"ms_per_step": r["step_saved_ms"],
                                                "value": flops / (r["step_saved_ms"] * 1e-3) / 1e12, "unit": "TFLOP/s"}
    line["hbm_copy_gbs"] = copy_roof()
    roof["frac_of_copy_roof"] = (roof["achieved"] / line["hbm_copy_gbs"]) if roof["bound"] == "hbm" else None
    if not args.no_dense:
        # empirical matrix-core roof (vendor GEMM, n = 8192) and the step's share of it
        line["dense_gemm_roof_tflops"] = mfma_roof()
        line["frac_of_dense_gemm_roof"] = line["value"] / line["dense_gemm_roof_tflops"][sh.dtype]
    if args.all:
        others = {}
        for name in ("sq256_f32", "sq256_f32_big", "gpt2s_fc1", "sq4096", "gpt2m_fc1", "gpt2m_fc2"):
            if name != args.workload:
                others[name] = run_workload(name, max(5, args.steps // 2), max(2, args.warmup // 2),
                                            with_dense=not args.no_dense, with_extras=not args.no_extras)[1]
        line["other_workloads"] = others
    if args.layers:
        from paper_2204_00595_amd import synth as _synth
        line["model_layers"] = {name: run_workload(name, max(5, args.steps // 2), max(2, args.warmup // 2),
                                                   with_dense=not args.no_dense, with_extras=not args.no_extras)[1]
                                for name in _synth.MODEL_LAYERS}
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(args.workload)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
