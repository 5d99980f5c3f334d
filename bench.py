#!/usr/bin/env python3
"""Benchmark of the LLA hot path on one MI355X.

One "step" = one pass of the whole hot path (llla_forward, or llla_decode for the decode workload)
over one batch of seeded synthetic input that is already resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3|C3b|C3d32|C4|C2|C1|C5|C5s|C5d128|E2] [--path auto|valu|mfma]
                  [--ex | --cg T | --backward] [--no-secondary]

metric  : tokens/s of the causal forward (B*n / t)  -- or generated tokens/s for decode (B / t)
roofline: the dominant kernel's algorithmic flops (forward; d^2+11d per causal pair plus
          d^3/3+4d^2 per row) or bytes (decode; K and V read once) over its measured duration
cpu_baseline: the fp64 oracle as it stands, timed on the host cores on a bounded sample.
secondary: with no --workload, the line also carries the forward at the shape the matrix-core target is quoted
          for (d = 64, n = 8192), the long-context forward at d = 128 and the decode configuration at d = 64 and at
          d = 128, each with its own timing, roofline and parity summary.

`value` is timed on the production library.  The per-kernel durations behind `roofline` come from a second loop over
the same launches through the measurement build of the same sources (HIP events around every kernel, on the stream
the kernels run on).
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_16BIT = 2.5e15      # dense bf16/f16 MFMA, flop/s
PEAK_MFMA_FP32 = 157.3e12     # dense fp32 MFMA, flop/s
PEAK_FP32_VALU = 157.3e12     # fp32 vector, flop/s
PEAK_HBM = 8.0e12             # B/s

CSRC = os.path.join(ROOT, "paper_2510_01450_amd", "csrc")
# HBM bytes per launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this same command,
# scaled with a copy kernel of known size.  Each entry names the summary it was taken from and the hash of the kernel's
# source file at the time: when the source has changed since, the figure is not reported (traffic = null).
MEASURED_TRAFFIC = {
    ("C3_prefill_bf16_n4096_d64", "moments"): {"fetch_bytes": 1.043e+08, "write_bytes": 8.153e+07, "source": "profiles/forward_C3_C3b_moments_kernel_mfma_counters.md",
        "kernel_files": ["llla_mfma_fwd.hip", "llla_mfma_common.hpp", "llla_mfma_solve64.hpp"],
        "kernel_sha16": "cc9e278b1d26fd88,13fbb5de8c328a9c,1ab82f954063627c"},
    ("C3b_prefill_bf16_n8192_d64", "moments"): {"fetch_bytes": 1.064e+08, "write_bytes": 8.605e+07, "source": "profiles/forward_C3_C3b_moments_kernel_mfma_counters.md",
        "kernel_files": ["llla_mfma_fwd.hip", "llla_mfma_common.hpp", "llla_mfma_solve64.hpp"],
        "kernel_sha16": "cc9e278b1d26fd88,13fbb5de8c328a9c,1ab82f954063627c"},
    ("C5_decode_bf16_L32768_d64", "decode_partial"): {"fetch_bytes": 4.31e+09, "write_bytes": 5.564e+07, "source": "profiles/decode_C5_bf16_L32768_d64_hbm_traffic.md",
        "kernel_files": ["llla_mfma_decode.hip", "llla_mfma_common.hpp"],
        "kernel_sha16": "0e4506854346e98d,13fbb5de8c328a9c"},
    ("C5d128_decode_bf16_L32768_d128", "decode_partial"): {"fetch_bytes": 4.31e+09, "write_bytes": 5.297e+07, "source": "profiles/decode_C5d128_bf16_L32768_d128_hbm_traffic.md",
        "kernel_files": ["llla_mfma_decode128.hip", "llla_mfma_common.hpp"],
        "kernel_sha16": "43376581dc93a91c,13fbb5de8c328a9c"},
    ("C4_longctx_bf16_n8192_d128", "moments"): {"fetch_bytes": 9.259e+08, "write_bytes": 8.703e+07, "source": "profiles/forward_C4_bf16_n8192_d128_hbm_traffic.md",
        "kernel_files": ["llla_mfma_fwd.hip", "llla_mfma_common.hpp", "llla_mfma_solve128.hpp"],
        "kernel_sha16": "cc9e278b1d26fd88,13fbb5de8c328a9c,4d7e6e915f78b32e"},
    ("C2_f32_n1024_d64", "moments"): {"fetch_bytes": 9.069e+06, "write_bytes": 4.85e+06, "source": "profiles/forward_C2_f32_n1024_d64_counters.md",
        "kernel_files": ["llla_mfma_fwd_f32.hip", "llla_mfma_common.hpp", "llla_mfma_solve64.hpp"],
        "kernel_sha16": "931352b9d2528c92,13fbb5de8c328a9c,1ab82f954063627c"},
}


def _sha16(path):
    with open(path, "rb") as fh:
        return hashlib.sha256(fh.read()).hexdigest()[:16]


def measured_traffic(workload, kernel):
    """(bytes per launch or None, where the figure comes from)."""
    e = MEASURED_TRAFFIC.get((workload, kernel))
    if e is None:
        return None, "not measured for this workload and kernel"
    now = ",".join(_sha16(os.path.join(CSRC, f)) for f in e["kernel_files"])
    if now != e["kernel_sha16"]:
        return None, "%s is older than the kernel source (%s changed since)" % (e["source"], ", ".join(e["kernel_files"]))
    return e["fetch_bytes"] + e["write_bytes"], e["source"]


def forward_flops(B, H, n, d):
    """Algorithmic flops of a causal forward: symmetric half of the second moment and the solve."""
    pairs = n * (n + 1) // 2
    return B * H * (pairs * (d * d + 11 * d) + n * (d ** 3 / 3.0 + 4 * d * d))


def backward_flops(B, H, n, d):
    """Algorithmic flops of the backward: the forward's moments again, gamma, r, a, b, dV, dK (three terms), dQ per
    causal pair; the elimination with two right-hand sides per row."""
    pairs = n * (n + 1) // 2
    return B * H * (pairs * (d * d + 22 * d) + n * (d ** 3 / 3.0 + 6 * d * d))


def measure(w, args, steps, warmup, headline):
    """Times `steps` passes of the hot path over workload `w`, then the per-kernel durations and the roofline of the
    dominant kernel, then a parity check against the oracle (and, for the headline, the oracle's own speed)."""
    import numpy as np
    import torch

    import paper_2510_01450_amd as llla
    import workloads

    dev = "cuda:0"
    decode = w.kind == "decode"
    t0 = time.time()
    cpu_in = workloads.make_inputs(w)
    n_rot = 3 if decode else 1          # decode: rotate distinct caches, each >> the 256 MB infinity cache
    dev_in = [tuple(t.to(dev) for t in cpu_in)]
    for r in range(1, n_rot):
        g = torch.Generator(device=dev).manual_seed(workloads.SEED0 + 77 + r)
        dev_in.append((dev_in[0][0],) + tuple(
            torch.randn(t.shape, generator=g, device=dev, dtype=torch.float32).to(t.dtype) for t in cpu_in[1:]))
    gen_s = time.time() - t0
    dt = workloads.torch_dtype(w)
    cg = args.cg if (headline and not decode) else None
    ex = args.ex and headline and not decode
    bwd = args.backward and headline and not decode
    if decode:
        need = llla.decode_workspace_bytes(w.B, w.H, w.n, w.d, dt)
        out = torch.empty((w.B, w.H, w.d), dtype=torch.float32, device=dev)
    else:
        need = llla.forward_workspace_bytes(w.B, w.H, w.n, w.d, dt)
        if cg is not None:
            need = llla.forward_cg_workspace_bytes(w.B, w.H, w.n, w.d, dt)
        out = torch.empty((w.B, w.H, w.n, w.d), dtype=torch.float32, device=dev)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    if bwd:
        g = torch.Generator(device="cpu").manual_seed(workloads.SEED0 + 9000 + w.index)
        dO_cpu = torch.randn((w.B, w.H, w.n, w.d), generator=g, dtype=torch.float32).to(dt)
        dO = dO_cpu.to(dev)
        ws = torch.empty(max(llla.backward_workspace_bytes(w.B, w.H, w.n, w.d, dt), 256), dtype=torch.uint8, device=dev)
        grads = tuple(torch.empty((w.B, w.H, w.n, w.d), dtype=torch.float32, device=dev) for _ in range(3)) + (
            torch.empty((w.B, w.H, w.n), dtype=torch.float32, device=dev),)
    # the per-row ridge is the workload's lambda in every row, so that the outputs stay those of the plain call
    lam_rows = torch.full((w.B, w.H, w.n), w.lam, dtype=torch.float32, device=dev) if ex else None
    stats = {}

    def step(i):
        a, b, c = dev_in[i % n_rot]
        if decode:
            llla.llla_decode(a, b, c, w.lam, w.scale, path=args.path, workspace=ws, out=out)
        elif bwd:
            llla.llla_backward(a, b, c, dO, w.lam, w.scale, path=args.path, workspace=ws, out=grads)
        elif cg is not None:
            llla.llla_forward_cg(a, b, c, w.lam, w.scale, cg, 0.0, workspace=ws, out=out)
        elif ex:
            _, stats["rho"], stats["delta"] = llla.llla_forward(a, b, c, lam_rows, w.scale, path=args.path, workspace=ws,
                                                               out=out, return_stats=True)
        else:
            llla.llla_forward(a, b, c, w.lam, w.scale, path=args.path, workspace=ws, out=out)

    def timed(k):
        """k steps between two synchronisations: (wall ms per step, per-step device times)."""
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(k)]
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        for i in range(k):
            evs[i][0].record()
            step(i)
            evs[i][1].record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t_start
        return wall * 1e3 / k, np.array([a.elapsed_time(b) for a, b in evs])

    for i in range(warmup):
        step(i)
    ms, per = timed(steps)

    # the same K steps again after at least a second of continuous launches: under a sustained matrix-core load the
    # clock settles below where a cold start finds it
    t_hot = time.perf_counter()
    hot_steps = 0
    while time.perf_counter() - t_hot < (0.0 if args.no_sustained else 1.0):
        for i in range(8):
            step(i)
        hot_steps += 8
        torch.cuda.synchronize()
    ms_sustained, _ = timed(steps)

    # ---- per-kernel durations through the measurement build (HIP events around each kernel, same stream) ----
    llla.use_measure_library(True)
    llla.profile_enable(True)
    acc = {}
    for i in range(steps + 2):
        step(i)
        if i < 2:
            llla.profile_last()
            continue
        for k, v in llla.profile_last().items():
            acc.setdefault(k, []).append(v)
    llla.profile_enable(False)
    llla.use_measure_library(False)
    stages = {k: float(np.mean(v)) for k, v in acc.items()}
    dom = max(stages, key=stages.get) if stages else None

    d = w.d
    if decode:
        tokens = w.B
        algo_bytes = 2.0 * w.B * w.H * w.n * w.d * cpu_in[1].element_size()
        dom_ms = stages[dom] if dom else float(np.mean(per))
        roof = {"bound": "hbm", "achieved": algo_bytes / (dom_ms * 1e-3) / 1e9, "peak": PEAK_HBM / 1e9,
                "unit": "GB/s", "traffic": None, "kernel": dom or "llla_decode (whole call)",
                "algorithmic_bytes_per_launch": algo_bytes, "kernel_ms": dom_ms}
    else:
        tokens = w.B * w.n
        pairs = w.n * (w.n + 1) // 2
        if bwd:
            # rows kernel: half of the second moment, logits, mu~, gamma, r, a, b, dQ; keys kernel: logits, a, b,
            # gamma, dV, the three terms of dK; per row the elimination with two right-hand sides
            # matrix-core flow: r sweep (logits, gamma, r), moments with both solves, dQ sweep (logits, a, b, gamma, dQ)
            per_pair = {"backward_rows": d * d + 14 * d, "backward_keys": 16 * d, "backward_r": 6 * d,
                        "backward_dq": 10 * d, "moments_and_two_solves": d * d + 5 * d}.get(dom, d * d + 22 * d)
            per_row = (d ** 3 / 3.0 + 6 * d * d) if dom in ("backward_rows", "moments_and_two_solves") else 0.0
            flops = w.B * w.H * (pairs * float(per_pair) + w.n * per_row)
            bound, peak = ("mfma", PEAK_MFMA_16BIT) if dom == "moments_and_two_solves" else ("alu", PEAK_FP32_VALU)
        elif dom == "cg_steps":
            # per step and causal pair: logits (2d), k.p (2d), accumulate (2d); per row the vector updates (~12d)
            flops = cg * w.B * w.H * (pairs * 6.0 * d + w.n * 12.0 * d)
            bound, peak = "mfma", PEAK_MFMA_16BIT
        elif dom == "moments":
            # logits, weights, omega, mu~, symmetric half of Sigma~, and the per-row solve
            flops = w.B * w.H * (pairs * (d * d + 5 * d) + w.n * (d ** 3 / 3.0 + 4 * d * d))
            # fp32 inputs contract on v_mfma_f32_16x16x4_f32: the peak of that instruction, not the 16-bit one
            bound, peak = "mfma", (PEAK_MFMA_FP32 if w.dtype == "f32" else PEAK_MFMA_16BIT)
        else:
            flops = forward_flops(w.B, w.H, w.n, d)
            bound, peak = ("mfma", PEAK_MFMA_16BIT) if (w.dtype != "f32" or dom != "valu_forward") else ("alu", PEAK_FP32_VALU)
        dom_ms = stages[dom] if dom else float(np.mean(per))
        roof = {"bound": bound, "achieved": flops / (dom_ms * 1e-3) / 1e12, "peak": peak / 1e12,
                "unit": "TFLOP/s", "traffic": None, "kernel": dom or "llla_forward (whole call)",
                "algorithmic_flops_per_launch": flops, "kernel_ms": dom_ms,
                "whole_call_algorithmic_tflops": (backward_flops(w.B, w.H, w.n, d) if bwd else
                                                  forward_flops(w.B, w.H, w.n, d)) / (float(np.mean(per)) * 1e-3) / 1e12}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"], roof["traffic_source"] = measured_traffic(w.name, dom)
    if roof["bound"] == "mfma" and headline and w.dtype != "f32":
        # context for `peak`: the 16-bit MFMA rate this GPU sustains under a chip-wide matrix-core load (the
        # measurement library's probe: independent 16x16x32 f16 MFMAs and nothing else), measured here with HIP events
        sink = torch.zeros(64, dtype=torch.float32, device="cuda")
        llla.probe_mfma_f16(64, sink)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        probe_flops = sum(llla.probe_mfma_f16(512, sink) for _ in range(3))
        e1.record()
        torch.cuda.synchronize()
        roof["sustained_mfma_probe_tflops"] = probe_flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
        roof["frac_of_sustained_probe"] = roof["achieved"] / roof["sustained_mfma_probe_tflops"]

    if w.dtype == "f32":
        dtype = "f32 in, f32 accumulate"
    elif bwd:
        dtype = "bf16 in, bf16/f16/f32 MFMA, f32 accumulate"
    else:
        dtype = "bf16 in, f16/f32 MFMA, f32 accumulate"
    result = {
        "metric": "LLA decode generated tokens/s" if decode else
        ("LLA causal backward tokens/s" if bwd else "LLA causal forward tokens/s"),
        "value": tokens / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms, "ms_per_step_device_median": float(np.median(per)),
        "ms_per_step_device_min": float(per.min()),
        "ms_per_step_sustained": ms_sustained, "sustained_after_steps": hot_steps,
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": dtype,
        "data": "synthetic (seeded, %s)" % w.values,
        "config": {"workload": w.name, "B": w.B, "H": w.H, "n": w.n, "d": w.d, "lambda": w.lam,
                   "scale": w.scale, "path": args.path, "input_setup_s": round(gen_s, 2),
                   "entry": "llla_backward" if bwd else ("llla_forward_cg (approximate: %d conjugate-gradient steps)" % cg) if cg is not None
                   else "llla_forward_ex (ridge per row, rho and delta written)" if ex else
                   ("llla_decode" if decode else "llla_forward")},
        "roofline": roof,
    }
    if stages:
        result["stages_ms"] = {k: round(v, 4) for k, v in stages.items()}
    if not decode:
        result["tflops_algorithmic"] = roof["achieved"]
    if args.no_check and (args.no_cpu_baseline or not headline):
        return result

    # ---- self-check of the timed configuration against the oracle; for the headline the same oracle calls are the
    #      CPU baseline (a bounded sample of the workload, scaled to the whole) ------------------------------------
    import oracle
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from parity import check
    budget_s = 10.0 if (headline and not args.no_cpu_baseline) else 0.0
    torch.cuda.synchronize()
    baseline = None
    if decode:
        step(0)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        nh = w.B * w.H if headline else min(w.B * w.H, 64)
        q, Kc, Vc = cpu_in
        t1 = time.perf_counter()
        qf, Kf, Vf = (t.reshape((1, w.B * w.H) + tuple(t.shape[2:]))[:, :nh] for t in (q, Kc, Vc))
        ref = oracle.decode(qf, Kf, Vf, w.lam, w.scale)
        cpu_s = time.perf_counter() - t1
        summ = check(got.reshape(1, w.B * w.H, 1, w.d)[:, :nh], ref[:, :, None], np.array([w.n - 1]), w.d, w.tol,
                     "bench decode")
        summ["checked"] = "%d of %d (batch, head) outputs" % (nh, w.B * w.H)
        full = cpu_s * (w.B * w.H) / nh
        baseline = {"value": w.B / full, "unit": "tokens/s", "cores": oracle.threads(),
                    "kind": "oracle", "sample": "%d of %d (batch, head) pairs, %.1f s; scaled by count"
                    % (nh, w.B * w.H, cpu_s)}
    elif bwd:
        # the upstream gradient is kept on sampled rows only, so that the oracle can produce every gradient of a
        # head from those rows one by one; the kernels do the same work whatever dO holds
        from oracle import backward as ob
        from parity import check_grad
        Q, K, V = cpu_in
        rows = workloads.sample_rows(w, n_random=24)[::6] if w.n > 512 else list(range(w.n))
        keep = torch.zeros(w.n, dtype=torch.bool)
        keep[torch.as_tensor(rows)] = True
        dO_s = dO_cpu * keep[None, None, :, None]
        got = llla.llla_backward(dev_in[0][0], dev_in[0][1], dev_in[0][2], dO_s.to(dev), w.lam, w.scale, path=args.path,
                                 workspace=ws, return_dlambda=True)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ref = ob.backward_head(Q[0, 0], K[0, 0], V[0, 0], dO_s[0, 0], w.lam, w.scale, rows=rows)
        nrep = 1
        while time.perf_counter() - t1 < budget_s:          # bounded sample: the same rows of further heads
            hh = nrep % (w.B * w.H)
            ob.backward_head(Q[hh // w.H, hh % w.H], K[hh // w.H, hh % w.H], V[hh // w.H, hh % w.H],
                             dO_s[hh // w.H, hh % w.H], w.lam, w.scale, rows=rows)
            nrep += 1
        cpu_s = time.perf_counter() - t1
        tol = 1e-3 if w.dtype == "f32" else 2e-2
        floor = float(dO_s[0, 0].double().norm()) * float(V[0, 0].double().pow(2).mean().sqrt())
        summ = {}
        for name, gq, rf in zip(("dQ", "dK", "dV", "dlambda"), got, ref):
            summ[name] = check_grad(gq[0, 0].cpu().numpy()[None, None], rf[None, None], w.d, tol, "bench " + name,
                                    floor=floor / (w.lam if name == "dlambda" else 1.0))
        work_all = w.B * w.H * (w.n * (w.n + 1) / 2.0)
        work_s = nrep * float(np.sum(np.asarray(rows) + 1.0))
        full = cpu_s * work_all / work_s
        baseline = {"value": w.B * w.n / full, "unit": "tokens/s", "cores": torch.get_num_threads(),
                    "kind": "oracle",
                    "sample": "%d sampled rows x %d heads in %.1f s; scaled by causal pairs (x%.0f)"
                    % (len(rows), nrep, cpu_s, work_all / work_s)}
    else:
        step(0)
        torch.cuda.synchronize()
        Q, K, V = cpu_in
        rows = workloads.sample_rows(w, n_random=64) if w.n > 1024 else list(range(w.n))
        got = out[0, 0].cpu().numpy()[rows]
        t1 = time.perf_counter()
        nrep = 0
        while True:                         # bounded sample: a few heads' worth of sampled rows
            if cg is not None:
                ref = oracle.forward_head_cg(Q[0, nrep % w.H], K[0, nrep % w.H], V[0, nrep % w.H], w.lam, w.scale,
                                             cg, 0.0, rows=rows)[0]
            else:
                ref = oracle.forward_head(Q[0, nrep % w.H], K[0, nrep % w.H], V[0, nrep % w.H], w.lam, w.scale,
                                          rows=rows)
            if nrep == 0:
                ref0 = ref
            nrep += 1
            if time.perf_counter() - t1 > budget_s:
                break
        cpu_s = time.perf_counter() - t1
        if cg is not None:
            # later CG iterates are not comparable element-wise (they are unstable under rounding); report how far
            # the approximate outputs are from the exact forward of this library and from the fp64 CG oracle
            exact = llla.llla_forward(*dev_in[0], w.lam, w.scale)[0, 0].cpu().numpy()[rows]
            dist = np.linalg.norm(got - exact, axis=-1) / np.linalg.norm(exact, axis=-1)
            dor = np.linalg.norm(got - ref0, axis=-1) / np.linalg.norm(ref0, axis=-1)
            late = np.asarray(rows) >= 4 * w.d
            summ = {"steps": cg,
                    "distance_to_exact_forward": {"median": float(np.median(dist)), "p90": float(np.quantile(dist, 0.9)),
                                                  "median_rows_ge_4d": float(np.median(dist[late])),
                                                  "max_rows_ge_4d": float(dist[late].max())},
                    "distance_to_fp64_cg_oracle": {"median": float(np.median(dor)), "p90": float(np.quantile(dor, 0.9))}}
        else:
            summ = check(got[None, None], ref0[None, None], np.array(rows), w.d, w.tol, "bench forward")
            summ["checked"] = "%d rows of head (0, 0)" % len(rows)
        if ex:
            _, rref, dref = oracle.forward_head_ex(Q[0, 0], K[0, 0], V[0, 0], w.lam, w.scale, rows=rows)
            summ["rho"] = check(stats["rho"][0, 0].cpu().numpy()[rows][None, None], rref[None, None], np.array(rows),
                                w.d, w.tol, "bench rho")
            summ["delta"] = check(stats["delta"][0, 0].cpu().numpy()[rows][None, None, :, None],
                                  dref[None, None, :, None], np.array(rows), w.d, w.tol, "bench delta")
        work_all = w.B * w.H * (w.n * (w.n + 1) / 2.0)
        work_s = nrep * float(np.sum(np.asarray(rows) + 1.0))
        full = cpu_s * work_all / work_s
        baseline = {"value": w.B * w.n / full, "unit": "tokens/s", "cores": oracle.threads(),
                    "kind": "oracle",
                    "sample": "%d sampled rows x %d heads in %.1f s; scaled by causal pairs (x%.0f)"
                    % (len(rows), nrep, cpu_s, work_all / work_s)}
    if headline and not args.no_cpu_baseline:
        result["cpu_baseline"] = baseline
    result["parity_check"] = summ
    return result


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default=None)
    ap.add_argument("--path", default="auto", choices=["auto", "valu", "mfma"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-check", action="store_true")
    ap.add_argument("--no-sustained", action="store_true",
                    help="skip the second of continuous launches before ms_per_step_sustained (counter-collection runs, "
                         "where every dispatch is slow and logged)")
    ap.add_argument("--no-secondary", action="store_true",
                    help="default run only: leave out the C3b forward and the C5 decode measurements")
    ap.add_argument("--cg", type=int, default=None, metavar="T",
                    help="forward workloads: time llla_forward_cg, the paper's approximate mode with T conjugate-gradient steps")
    ap.add_argument("--backward", action="store_true",
                    help="forward workloads: time llla_backward (gradients w.r.t. Q, K, V and the ridge of every row)")
    ap.add_argument("--ex", action="store_true",
                    help="forward workloads: time llla_forward_ex with a ridge per row and the statistics rho, delta")
    ap.add_argument("--copy-probe", action="store_true",
                    help="run nothing but three plain copies of 1 GiB (measurement library): under rocprofv3 --pmc this is the "
                         "scale of the HBM counters, FETCH_SIZE or WRITE_SIZE units per byte")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures ONE GPU (one MI355X per box); --gpus %d is not run. "
              "How the path would shard over several GPUs is described in the design notes of this repository." % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import torch

    import workloads

    if not torch.cuda.is_available():
        print("bench.py needs a GPU (no CPU fallback exists)", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    if args.copy_probe:
        import paper_2510_01450_amd as llla
        src = torch.ones(1 << 28, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        copied = [llla.probe_copy(src, dst) for _ in range(3)]
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes_per_launch": copied[0], "launches": len(copied), "kernel": "copy_rate_kernel"}))
        return
    default_run = args.workload is None and not (args.cg is not None or args.backward or args.ex)
    name = args.workload or "C3"
    w = workloads.ALL[name.upper() if name.upper() in workloads.ALL else name]
    steps = args.steps if args.steps is not None else (20 if w.kind != "decode" else 30)
    warmup = args.warmup if args.warmup is not None else 3
    result = measure(w, args, steps, warmup, headline=True)
    if default_run and not args.no_secondary:
        # the same driver run witnesses the shape the 40 % matrix-core target is quoted for, the d = 128 forward and the
        # decode configuration at both head dimensions
        result["secondary"] = []
        for sw in (workloads.C3B, workloads.C4, workloads.C5, workloads.C5D128):
            torch.cuda.empty_cache()
            r = measure(sw, args, steps, warmup, headline=False)
            result["secondary"].append({k: r[k] for k in ("metric", "value", "unit", "ms_per_step", "ms_per_step_sustained",
                                                          "dtype", "config", "roofline", "stages_ms", "parity_check")
                                        if k in r})
    print(json.dumps(result))


if __name__ == "__main__":
    main()
