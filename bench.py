"""Benchmark of the TSR-Adam per-matrix optimizer hot path on one MI355X.

A "step" is one pass of the whole per-step path (project all blocks -> Adam on the cores ->
lift + apply) over one batch of synthetic LLaMA-shaped gradients already resident in HBM,
issued through the batched C-ABI call.  The workload at N=1 is the LLaMA-130M-shaped optimizer
step (84 blocks, r = 256, bf16 gradients, fp32 weights and core moments).  The subspace
refresh (rSVD, p = 8, q = 1) is timed separately in the same run.

Prints ONE JSON line (see the keys below).  `value` is the algorithmic bytes of one step
(G once, W read + written, U and V once for project and once for lift, the core arrays)
divided by the step time.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import synth_inputs as si  # noqa: E402

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 matrix-core peak, published


def step_bytes(m, n, r, g_bytes):
    """Algorithmic HBM bytes of one step for one block."""
    return m * n * g_bytes + 8 * m * n + 8 * r * (m + n) + 24 * r * r


def step_flops(m, n, r):
    return 4 * m * n * r + 4 * r * r * min(m, n)


def tvt_bytes(m, n, r):
    """Algorithmic bytes of the fused lift-and-apply kernel W <- bW + a (U D) V^T for one block:
    W (fp32) read and written once; the bf16 copies of U (m x r), V (n x r) and D (r x r) read once."""
    return 8 * m * n + 2 * r * (m + n) + 2 * r * r


def gv_bytes(m, n, r, g_bytes):
    """G once, the bf16 copy of V once, P = G V written once as bf16."""
    return m * n * g_bytes + 2 * n * r + 2 * m * r


def build_blocks(w: si.Workload, device):
    blocks = []
    for i, (m, n) in enumerate(w.shapes):
        key = si.stream_key(si.BASE_SEED, 2, i)
        sig = si.make_signal(m, n, w.signal_rank, w.spectrum, key, device=device)
        if w.workers > 1:
            G = torch.stack([si.gradient(sig, w.noise, si.stream_key(key, 100 + k), dtype=w.g_dtype)
                             for k in range(w.workers)])
        else:
            G = si.gradient(sig, w.noise, si.stream_key(key, 100), dtype=w.g_dtype)
        if n % 8 != 0:
            # odd widths (5461 in the 1B shapes): row pitch padded to 8 elements, which the bf16
            # kernels' 16-byte loads need; the matrix itself stays m x n (a strided view)
            ld = (n + 7) // 8 * 8
            Gp = torch.zeros(*G.shape[:-1], ld, dtype=G.dtype, device=G.device)
            Gp[..., :n] = G
            G = Gp[..., :n]
        r = w.r
        blocks.append(dict(
            G=G, W=si.weights(m, n, si.stream_key(key, 7), device=device),
            U=torch.empty(m, r, device=device), V=torch.empty(n, r, device=device),
            M=torch.zeros(r, r, device=device), Vm=torch.zeros(r, r, device=device),
            C=torch.empty(r, r, device=device), D=torch.empty(r, r, device=device)))
    return blocks


def cpu_baseline(w: si.Workload, blocks, omegas, budget_s=12.0):
    """The fp64 oracle, as it stands, on this host: whole steps of the whole workload (every
    block: project, Adam on the core, lift + apply) repeated until about budget_s seconds have
    passed, then the refresh of the first layer's blocks."""
    from oracle import tsr_oracle as orc
    r = w.r
    host = []
    for b in blocks:
        G = b["G"][0] if b["G"].dim() == 3 else b["G"]
        host.append(dict(G=orc.f64(G), U=orc.f64(b["U"]), V=orc.f64(b["V"]), W=orc.f64(b["W"]),
                         M=np.zeros((r, r)), Vm=np.zeros((r, r))))
    steps, t0 = 0, time.perf_counter()
    while True:
        for h in host:
            orc.tsr_adam_step(h["W"], [h["G"]], h["U"], h["V"], h["M"], h["Vm"], steps + 1, lr=1e-3)
        steps += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or steps >= 20:
            break
    g_bytes = 2 if w.g_dtype == torch.bfloat16 else 4
    nbytes = steps * sum(step_bytes(m, n, r, g_bytes) for m, n in w.shapes)
    n_refresh = min(7, len(host))
    t1 = time.perf_counter()
    for i in range(n_refresh):
        orc.refresh_rsvd(host[i]["G"], orc.f64(omegas[i]), r, w.p, w.q)
    dt_refresh = time.perf_counter() - t1
    return dict(value=nbytes / dt / 1e9, unit="GB/s", cores=orc.num_threads(), kind="oracle",
                sample="%d whole steps of all %d blocks in %.1f s (%.3f s per step); refresh of the first %d blocks "
                       "in %.1f s" % (steps, len(w.shapes), dt, dt / steps, n_refresh, dt_refresh),
                seconds_per_step=dt / steps, refresh_ms_per_matrix=dt_refresh / n_refresh * 1e3)


def read_traffic(path):
    """Optional rocprofv3 --pmc summary: lines `key: value`."""
    if not os.path.exists(path):
        return None
    out = {}
    for ln in open(path):
        if ":" in ln and not ln.startswith("#"):
            k, v = ln.split(":", 1)
            try:
                out[k.strip()] = float(v.strip())
            except ValueError:
                pass
    return out.get("tvt_traffic_bytes_per_launch")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="llama-130m")
    ap.add_argument("--layers", type=int, default=None, help="use fewer layers (debugging only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-refresh", action="store_true")
    ap.add_argument("--refresh-workers", type=int, default=0,
                    help="also time the N-worker refresh (averaged sketches) on one block of each distinct shape")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives are built); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import paper_2602_08007_amd as tsr
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = si.workload(args.workload, args.layers)
    g_bytes = 2 if w.g_dtype == torch.bfloat16 else 4
    blocks = build_blocks(w, dev)
    precision = tsr.TSR_PREC_BF16 if w.g_dtype == torch.bfloat16 else tsr.TSR_PREC_SPLIT
    plan = tsr.Plan(blocks, n_workers=w.workers, precision=precision, with_refresh=True, p=w.p)
    stream = torch.cuda.current_stream()

    # ---- refresh (initialises U, V from the gradients; timed on its second run)
    omegas = [si.omega(n, w.r + w.p, si.stream_key(si.BASE_SEED, 3, i), device=dev) for i, (m, n) in enumerate(w.shapes)]
    plan.tsr_refresh_batched(omegas, w.q)
    torch.cuda.synchronize()
    refresh = None
    if not args.no_refresh:
        # the refresh as a caller gets it (groups of blocks side by side on the library's streams) ...
        t0 = time.perf_counter()
        plan.tsr_refresh_batched(omegas, w.q)
        torch.cuda.synchronize()
        refresh_ms = (time.perf_counter() - t0) * 1e3
        # ... and once more with stage timing on, which runs it as one program on one stream
        plan.tsr_plan_profile_begin()
        t0 = time.perf_counter()
        plan.tsr_refresh_batched(omegas, w.q)
        torch.cuda.synchronize()
        refresh_single_ms = (time.perf_counter() - t0) * 1e3
        prof = plan.tsr_plan_profile_end()
        k = w.r + w.p
        gemm_flops = sum((2 * w.q + 2) * 2 * m * n * k for m, n in w.shapes)
        gemm_ms = prof["sketch_gemm"][0]
        refresh = dict(ms_total=refresh_ms, ms_per_matrix=refresh_ms / len(w.shapes),
                       ms_total_one_stream=refresh_single_ms,
                       gemm_ms=gemm_ms, gemm_tflops=gemm_flops / gemm_ms / 1e9,
                       gemm_mfma_frac=gemm_flops / gemm_ms / 1e9 / MFMA_BF16_PEAK_TFLOPS,
                       stages_ms={kk: round(v[0], 3) for kk, v in prof.items() if v[1]},
                       p=w.p, q=w.q)

    # ---- one plain copy of known size (256 MiB read + 256 MiB written): the measured HBM rate of
    # this machine and the reference that scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters
    n_copy = 64 * 1024 * 1024
    src = torch.zeros(n_copy, device=dev); dst = torch.empty(n_copy, device=dev)
    tsr.tsr_stream_scale(dst, src, 1.0)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        tsr.tsr_stream_scale(dst, src, 1.0)
    e1.record(); torch.cuda.synchronize()
    copy_gbps = 5 * 2 * n_copy * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst

    # ---- the timed step loop
    hyper = dict(lr=float(os.environ.get("TSR_BENCH_LR", "1e-3")), wd=0.0, beta1=0.9, beta2=0.999, eps=1e-8, scale=1.0)
    t = 1
    for _ in range(args.warmup):
        plan.tsr_step_batched(t, **hyper); t += 1
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        plan.tsr_step_batched(t, **hyper); t += 1
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # ---- same steps again with HIP events around every stage (per-kernel durations)
    plan.tsr_plan_profile_begin()
    for _ in range(args.steps):
        plan.tsr_step_batched(t, **hyper); t += 1
    prof = plan.tsr_plan_profile_end()
    stage_ms = {kk: v[0] / max(v[1], 1) for kk, v in prof.items() if v[1]}

    total_bytes = sum(step_bytes(m, n, w.r, g_bytes) for m, n in w.shapes) + \
        (w.workers - 1) * sum(m * n * g_bytes for m, n in w.shapes)
    total_flops = sum(step_flops(m, n, w.r) for m, n in w.shapes)
    value = total_bytes / (ms_per_step * 1e-3) / 1e9

    # dominant kernel = the longest stage of the step
    dom = max(("gv", "tvt"), key=lambda kk: stage_ms.get(kk, 0.0))
    if dom == "tvt":
        dom_bytes = sum(tvt_bytes(m, n, w.r) for m, n in w.shapes)
    else:
        dom_bytes = w.workers * sum(gv_bytes(m, n, w.r, g_bytes) for m, n in w.shapes)
    achieved = dom_bytes / (stage_ms[dom] * 1e-3) / 1e9
    roofline = dict(bound="hbm", kernel=dom, achieved=achieved, peak=HBM_PEAK_GBPS, unit="GB/s",
                    frac=achieved / HBM_PEAK_GBPS, ms_per_launch=stage_ms[dom],
                    traffic=read_traffic(os.path.join(ROOT, "profiles", "step_%s_traffic.txt" % w.name)))

    # ---- optional: refresh with N workers (per-worker sketch chains, averaged Q and B)
    refresh_workers = None
    if args.refresh_workers > 0:
        K = args.refresh_workers
        k = w.r + w.p
        per_shape = []
        for (m, n) in sorted(set(w.shapes)):
            key = si.stream_key(si.BASE_SEED, 5, m, n)
            sig = si.make_signal(m, n, w.signal_rank, w.spectrum, key, device=dev)
            Gs = torch.stack([si.gradient(sig, w.noise, si.stream_key(key, 100 + i), dtype=w.g_dtype) for i in range(K)])
            Om = si.omega(n, k, si.stream_key(key, 3), device=dev)
            U = torch.empty(m, w.r, device=dev); V = torch.empty(n, w.r, device=dev)
            ws = tsr.workspace(tsr.tsr_refresh_workers_workspace_bytes(m, n, w.r, w.p, K), dev)
            tsr.tsr_refresh_rsvd_workers(Gs, Om, w.r, w.p, w.q, U, V, None, ws)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            tsr.tsr_refresh_rsvd_workers(Gs, Om, w.r, w.p, w.q, U, V, None, ws)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3
            defect = float(torch.linalg.norm(U.double().T @ U.double() - torch.eye(w.r, device=dev, dtype=torch.float64)))
            per_shape.append({"shape": [m, n], "ms": round(ms, 3), "orthonormality_defect_U": defect,
                              "sketch_payload_bytes_per_worker": 4 * k * (m + n), "dense_bytes_fp32": 4 * m * n})
        refresh_workers = {"workers": K, "per_shape": per_shape}

    core_b, dense_b = plan.payload_bytes(4)
    out = {
        "metric": "Projected-Adam step GB/s + % HBM roofline; rSVD refresh ms/matrix + MFMA %",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if precision == tsr.TSR_PREC_BF16 else "f32",
        "dtype_detail": "bf16 MFMA operands, f32 accumulation, f32 weights and moments" if precision == tsr.TSR_PREC_BF16
                        else "f32 operands as 2-3 bf16 pieces, f32 accumulation",
        "data": "synthetic",
        "config": {"workload": w.name, "blocks": len(w.shapes), "r": w.r, "g_dtype": str(w.g_dtype).replace("torch.", ""),
                   "workers": w.workers},
        "hbm_frac": value / HBM_PEAK_GBPS, "copy_kernel_gbps": copy_gbps, "frac_of_copy_kernel": value / copy_gbps,
        "step_tflops": total_flops / (ms_per_step * 1e-3) / 1e12,
        "stage_ms": {kk: round(v, 4) for kk, v in stage_ms.items()},
        "roofline": roofline,
        "refresh": refresh,
        "refresh_workers": refresh_workers,
        "payload": {"core_bytes": core_b, "dense_bytes_fp32": dense_b, "ratio": dense_b / core_b},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, blocks, omegas)
    plan.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
