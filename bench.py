"""Benchmark of the TSR-Adam per-matrix optimizer hot path on one MI355X.

A "step" is one pass of the whole per-step path (project all blocks -> Adam on the cores ->
lift + apply) over one batch of synthetic LLaMA-shaped gradients already resident in HBM,
issued through the batched C-ABI call.  The workload at N=1 is the largest single-GPU
configuration, the LLaMA-1B-shaped optimizer step (168 blocks, r = 512, bf16 gradients, fp32
weights and core moments; refresh with p = 16, q = 2 timed separately in the same run).  The
LLaMA-130M-shaped step (84 blocks, r = 256) is measured in the same run and reported under the
key "secondary".

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


def cpu_baseline(w: si.Workload, blocks, omegas):
    """The fp64 oracle, as it stands, on this host, on a bounded sample of the workload: one whole
    step (project, Adam on the core, lift + apply) of ONE block of every distinct shape, scaled
    by the number of blocks of that shape, once with all host threads and once with one thread;
    then the refresh of one block (the smallest distinct shape that the plain-loop oracle
    finishes within seconds, else none)."""
    from oracle import tsr_oracle as orc
    r = w.r
    g_bytes = 2 if w.g_dtype == torch.bfloat16 else 4
    counts = {}
    first = {}
    for i, sh in enumerate(w.shapes):
        counts[sh] = counts.get(sh, 0) + 1
        first.setdefault(sh, i)
    all_threads = orc.num_threads()
    host = {}
    for sh, i in first.items():
        b = blocks[i]
        G = b["G"][0] if b["G"].dim() == 3 else b["G"]
        host[sh] = dict(G=orc.f64(G), U=orc.f64(b["U"]), V=orc.f64(b["V"]), W=orc.f64(b["W"]))
    per_threads = {}
    for threads in (all_threads, 1):
        orc.set_num_threads(threads)
        total = 0.0
        for sh, h in host.items():
            M, Vm = np.zeros((r, r)), np.zeros((r, r))
            t0 = time.perf_counter()
            orc.tsr_adam_step(h["W"], [h["G"]], h["U"], h["V"], M, Vm, 1, lr=1e-3)
            total += (time.perf_counter() - t0) * counts[sh]
        per_threads[threads] = total
    orc.set_num_threads(all_threads)
    nbytes = sum(step_bytes(m, n, r, g_bytes) for m, n in w.shapes)      # worker 0's gradient only
    out = dict(value=nbytes / per_threads[all_threads] / 1e9, unit="GB/s", cores=all_threads, kind="oracle",
               seconds_per_step=per_threads[all_threads],
               value_one_thread=nbytes / per_threads[1] / 1e9, seconds_per_step_one_thread=per_threads[1])
    sample = ("one step of one block of each of the %d distinct shapes, scaled by the block counts %s: %.2f s per whole step "
              "on %d threads, %.2f s on 1 thread" % (len(host), sorted(counts.values()), per_threads[all_threads],
                                                     all_threads, per_threads[1]))
    # refresh: only where the oracle's QR + Jacobi SVD finish in seconds (k up to about 300)
    if w.r + w.p <= 300:
        sh = min(host, key=lambda s_: s_[0] * s_[1])
        i = first[sh]
        t1 = time.perf_counter()
        orc.refresh_rsvd(host[sh]["G"], orc.f64(omegas[i]), r, w.p, w.q)
        dt = time.perf_counter() - t1
        out["refresh_ms_per_matrix"] = dt * 1e3
        sample += "; refresh of one %dx%d block in %.2f s on %d threads" % (sh[0], sh[1], dt, all_threads)
    out["sample"] = sample
    return out


def read_traffic(path):
    """rocprofv3 --pmc summary of an EARLIER profiling run kept with the sources (lines `key: value`);
    None when there is none for this workload."""
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
    return out


def step_bytes_needed(m, n, r, g_bytes, fast):
    """Bytes the kernels of the bf16 path actually have to move per block: as step_bytes, with the
    bases read as their bf16 copies (two bytes, not four) in both the projection and the lift."""
    if not fast:
        return step_bytes(m, n, r, g_bytes)
    return m * n * g_bytes + 8 * m * n + 4 * r * (m + n) + 24 * r * r


def run_workload(tsr, name, args, dev, with_cpu_baseline):
    """Builds the synthetic blocks of one workload, refreshes the bases, times the step loop and
    (optionally) the refresh; returns the measured figures."""
    w = si.workload(name, args.layers)
    g_bytes = 2 if w.g_dtype == torch.bfloat16 else 4
    blocks = build_blocks(w, dev)
    precision = tsr.TSR_PREC_BF16 if w.g_dtype == torch.bfloat16 else tsr.TSR_PREC_SPLIT
    plan = tsr.Plan(blocks, n_workers=w.workers, precision=precision, with_refresh=True, p=w.p)
    fast = plan.tsr_plan_kernel_path() == 1

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
        # MFMA products issued per useful product in the G-touching GEMMs: a bf16 gradient is exact in
        # one piece and meets two bf16 pieces of the small fp32 operand; an fp32 gradient and its
        # partner keep three pieces each, of which the six leading cross products are issued
        pieces = 2 if w.g_dtype == torch.bfloat16 else 6
        refresh = dict(ms_total=refresh_ms, ms_per_matrix=refresh_ms / len(w.shapes),
                       ms_total_one_stream=refresh_single_ms,
                       gemm_ms=gemm_ms, gemm_tflops=gemm_flops / gemm_ms / 1e9,
                       gemm_mfma_frac=gemm_flops / gemm_ms / 1e9 / MFMA_BF16_PEAK_TFLOPS,
                       gemm_mfma_products_per_useful_product=pieces,
                       gemm_issued_mfma_frac=pieces * gemm_flops / gemm_ms / 1e9 / MFMA_BF16_PEAK_TFLOPS,
                       gemm_ms_includes="transposed copy of G and splitting of the small operands (bf16 gradients)",
                       stages_ms={kk: round(v[0], 3) for kk, v in prof.items() if v[1]},
                       p=w.p, q=w.q)

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
    stage_ms = {kk: v[0] / args.steps for kk, v in prof.items() if v[1]}

    extra_g = (w.workers - 1) * sum(m * n * g_bytes for m, n in w.shapes)
    total_bytes = sum(step_bytes(m, n, w.r, g_bytes) for m, n in w.shapes) + extra_g
    needed_bytes = sum(step_bytes_needed(m, n, w.r, g_bytes, fast) for m, n in w.shapes) + extra_g
    total_flops = sum(step_flops(m, n, w.r) for m, n in w.shapes)
    value = total_bytes / (ms_per_step * 1e-3) / 1e9

    # dominant kernel = the longest stage of the step
    dom = max(("gv", "tvt"), key=lambda kk: stage_ms.get(kk, 0.0))
    if dom == "tvt":
        dom_bytes = sum(tvt_bytes(m, n, w.r) for m, n in w.shapes)
    else:
        dom_bytes = w.workers * sum(gv_bytes(m, n, w.r, g_bytes) for m, n in w.shapes)
    achieved = dom_bytes / (stage_ms[dom] * 1e-3) / 1e9
    traffic_file = os.path.join("profiles", "step_%s_traffic.txt" % w.name)
    traffic = read_traffic(os.path.join(ROOT, traffic_file))
    roofline = dict(bound="hbm", kernel=dom, achieved=achieved, peak=HBM_PEAK_GBPS, unit="GB/s",
                    frac=achieved / HBM_PEAK_GBPS, ms_per_launch=stage_ms[dom], algorithmic_bytes_per_launch=dom_bytes,
                    traffic=(traffic or {}).get("%s_traffic_bytes_per_launch" % dom),
                    traffic_source=("%s (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this command, "
                                    "not of this run)" % traffic_file) if traffic else None)

    core_b, dense_b = plan.payload_bytes(4)
    out = {
        "value": value, "ms_per_step": ms_per_step,
        "dtype": "bf16" if precision == tsr.TSR_PREC_BF16 else "f32",
        "dtype_detail": "bf16 MFMA operands, f32 accumulation, f32 weights and moments" if precision == tsr.TSR_PREC_BF16
                        else "f32 operands as 2-3 bf16 pieces, f32 accumulation",
        "config": {"workload": w.name, "blocks": len(w.shapes), "r": w.r, "g_dtype": str(w.g_dtype).replace("torch.", ""),
                   "workers": w.workers, "kernel_path": "bf16 family" if fast else "general grouped kernels"},
        "hbm_frac": value / HBM_PEAK_GBPS,
        "value_bytes_needed": needed_bytes / (ms_per_step * 1e-3) / 1e9,
        "hbm_frac_bytes_needed": needed_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "step_tflops": total_flops / (ms_per_step * 1e-3) / 1e12,
        "mfma_frac": total_flops / (ms_per_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "stage_ms": {kk: round(v, 4) for kk, v in stage_ms.items()},
        "roofline": roofline,
        "refresh": refresh,
        "payload": {"core_bytes": core_b, "dense_bytes_fp32": dense_b, "ratio": dense_b / core_b},
    }
    if with_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, blocks, omegas)
    plan.close()
    return out


def refresh_workers_bench(tsr, w, K, dev):
    """Refresh with K workers (per-worker sketch chains, averaged Q and B) on one block of each distinct shape."""
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
    return {"workers": K, "per_shape": per_shape}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama-1b",
                    help="llama-1b (default) | llama-130m | llama-350m-dp8 | single-60m | lm-head")
    ap.add_argument("--secondary", default="llama-130m", help="a second workload measured in the same run ('' = none)")
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

    main_res = run_workload(tsr, args.workload, args, dev, not args.no_cpu_baseline)
    torch.cuda.empty_cache()
    out = {
        "metric": "Projected-Adam step GB/s + % HBM roofline; rSVD refresh ms/matrix + MFMA %",
        "value": main_res["value"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "data": "synthetic", "copy_kernel_gbps": copy_gbps, "frac_of_copy_kernel": main_res["value"] / copy_gbps,
    }
    out.update({k: v for k, v in main_res.items() if k not in ("value", "ms_per_step")})
    if args.refresh_workers > 0:
        out["refresh_workers"] = refresh_workers_bench(tsr, si.workload(args.workload, args.layers), args.refresh_workers, dev)
    if args.secondary and args.secondary != args.workload:
        out["secondary"] = run_workload(tsr, args.secondary, args, dev, not args.no_cpu_baseline)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
