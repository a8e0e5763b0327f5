"""Helpers shared by the GPU parity tests."""
import os

import numpy as np
import torch

from oracle import tsr_oracle as orc


def rel_fro(a, b) -> float:
    a = orc.f64(a); b = orc.f64(b)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def max_abs_rel(a, b) -> float:
    """Largest element-wise error relative to the largest reference element: what a handful of
    wrong elements (a tile edge, a dropped lane) cannot hide behind a Frobenius norm."""
    a = orc.f64(a); b = orc.f64(b)
    return float(np.abs(a - b).max() / max(np.abs(b).max(), 1e-300))


def check_close(a, b, tol, what=""):
    """Relative Frobenius error AND largest element error (relative to the largest reference
    element) below tol; returns both for the record."""
    ef, em = rel_fro(a, b), max_abs_rel(a, b)
    assert ef < tol, "%s: relative Frobenius error %.3e >= %.1e" % (what, ef, tol)
    assert em < tol, "%s: largest element error %.3e (of the largest element) >= %.1e" % (what, em, tol)
    return ef, em


_LOG_PATH = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out", "parity_summary.txt")


def parity_log(line: str) -> None:
    """Append one line of measured parity figures to gpurun_out/parity_summary.txt (the folder a GPU
    run brings back) and print it."""
    print(line)
    try:
        os.makedirs(os.path.dirname(_LOG_PATH), exist_ok=True)
        with open(_LOG_PATH, "a") as f:
            f.write(line + "\n")
    except OSError:
        pass


def projector_err(X_gpu, X_ref) -> float:
    """|| X X^T - Y Y^T ||_F / || Y Y^T ||_F computed through the small r x r products."""
    X = orc.f64(X_gpu); Y = orc.f64(X_ref)
    # ||XX^T - YY^T||^2 = ||X^T X||^2 + ||Y^T Y||^2 - 2 ||X^T Y||^2
    a = np.linalg.norm(X.T @ X) ** 2; b = np.linalg.norm(Y.T @ Y) ** 2; c = np.linalg.norm(X.T @ Y) ** 2
    return float(np.sqrt(max(a + b - 2 * c, 0.0)) / np.sqrt(b))


def dev(x: torch.Tensor) -> torch.Tensor:
    return x.to("cuda").contiguous()


def padded(x: torch.Tensor, ld: int) -> torch.Tensor:
    """Copy of the 2-D tensor x on the GPU with leading dimension ld (a view into a wider buffer)."""
    m, n = x.shape
    buf = torch.zeros((m, ld), dtype=x.dtype, device="cuda")
    buf[:, :n] = x.to("cuda")
    return buf[:, :n]


def f32(x: float) -> float:
    """The value the C ABI receives for a float argument (hyper-parameters are inputs: the
    oracle gets exactly what the GPU gets)."""
    return float(np.float32(x))


B1, B2, EPS = f32(0.9), f32(0.999), f32(1e-8)


def plan_trajectory(plan, blocks, sample, steps, tol, label, lr=1e-3, wd=0.01, workers=1, next_grads=None,
                    bar_d=None, bar_move=None, bar_move_own=None, after_block=None, warm_steps=0, w_tol=None):
    """Run batched steps of `plan` and replay them in the oracle for the blocks in `sample`.

    The oracle follows its OWN trajectory from the common start: nothing the GPU computes is ever
    copied into it.  next_grads(t), if given, puts the gradients of step t into the device buffers
    first (a fresh draw per step); the oracle reads them back from there, so both sides see the
    same arrays.

    Start.  warm_steps = 0: cold start as Algorithm 1 states it (zero moments, t = 1).  At a cold
    first step D = c / (|c| + eps) is the sign of c, decided by the rounding of the smallest core
    entries in any arithmetic, so D and the movement are compared with the oracle's from the
    second step on, and at the first step on the GPU's own core only.  warm_steps = k: the ORACLE
    alone runs steps 1..k, its state (W, m, v rounded to fp32) is uploaded as the common start
    of both sides (every sampled block; `sample` must then cover the plan), and the compared
    steps are k + 1 ..: a state as it is in the middle of training, where D is a smooth function
    of the cores and every check applies from the first compared step.

    Checked per sampled block and step, Frobenius and largest-element errors both:
      * against the oracle's trajectory: core, both moments and weights at `tol`; D (bar_d) and
        the movement W_t - W_{t-1} (bar_move);
      * each kernel on its own inputs: Adam from the GPU's core and previous moments (fp32
        element-wise arithmetic: 1e-4 on D, 1e-5 on the moments), the lift from the GPU's D and
        previous weights (`tol` on W, bar_move_own on the movement).
    `steps` are the compared step numbers.  w_tol (default tol) is the bar on the weights against
    the oracle's trajectory: after a cold start they carry the sign decisions of D_1, which weigh
    more the smaller the block (the movement is a larger share of W).  Returns the list of
    measured figures (dicts)."""
    w_tol = tol if w_tol is None else w_tol
    bar_d = tol if bar_d is None else bar_d
    bar_move = tol if bar_move is None else bar_move
    bar_move_own = tol if bar_move_own is None else bar_move_own
    lr32, wd32 = f32(lr), f32(wd)
    steps = list(steps)
    state = {}
    for i in sample:
        b = blocks[i]
        state[i] = dict(W=orc.f64(b["W"]).copy(), M=orc.f64(b["M"]).copy(), Vm=orc.f64(b["Vm"]).copy(),
                        U=orc.f64(b["U"]), V=orc.f64(b["V"]))

    def grads_of(i):
        b = blocks[i]
        Gs = b["G"] if workers > 1 else b["G"][None]
        return [g for g in Gs]

    if warm_steps:
        assert steps[0] == warm_steps + 1 and len(list(sample)) == len(blocks)
        for t in range(1, warm_steps + 1):
            if next_grads is not None:
                next_grads(t)
            for i in sample:
                s = state[i]
                orc.tsr_adam_step(s["W"], grads_of(i), s["U"], s["V"], s["M"], s["Vm"], t, lr=lr32, wd=wd32,
                                  beta1=B1, beta2=B2, eps=EPS)
        for i in sample:                      # the oracle's state is the checkpoint both sides start from
            b, s = blocks[i], state[i]
            for k in ("W", "M", "Vm"):
                b[k].copy_(torch.from_numpy(s[k]).float())
                s[k][...] = orc.f64(b[k])
    compare_d_from = steps[0] if warm_steps else steps[0] + 1
    out = []
    for t in steps:
        if next_grads is not None:
            next_grads(t)
        before = {i: (orc.f64(blocks[i]["W"]).copy(), orc.f64(blocks[i]["M"]).copy(), orc.f64(blocks[i]["Vm"]).copy())
                  for i in sample}
        plan.tsr_step_batched(t, lr=lr, wd=wd)
        torch.cuda.synchronize()
        for i in sample:
            b, s = blocks[i], state[i]
            Wg0, Mg0, Vg0 = before[i]
            Wo0 = s["W"].copy()
            Cbar, D = orc.tsr_adam_step(s["W"], grads_of(i), s["U"], s["V"], s["M"], s["Vm"], t, lr=lr32, wd=wd32,
                                        beta1=B1, beta2=B2, eps=EPS)
            what = "%s block %d %s t=%d" % (label, i, tuple(b["W"].shape), t)
            e = dict(t=t, block=i)
            e["C"], e["C_max"] = check_close(b["C"], Cbar, tol, what + " core")
            e["M"], _ = check_close(b["M"], s["M"], tol, what + " first moment")
            e["Vm"], _ = check_close(b["Vm"], s["Vm"], 2 * tol, what + " second moment")
            e["W"], e["W_max"] = check_close(b["W"], s["W"], w_tol, what + " weights")
            # Adam on the GPU's own core and previous moments
            Mk, Vk = Mg0.copy(), Vg0.copy()
            Dk = orc.adam_core(orc.f64(b["C"]), Mk, Vk, t, B1, B2, EPS)
            e["D_own"], _ = check_close(b["D"], Dk, 1e-4, what + " D from the GPU's own core")
            assert rel_fro(b["M"], Mk) < 1e-5 and rel_fro(b["Vm"], Vk) < 1e-5, what
            # lift from the GPU's own D and previous weights
            Wk = orc.backproject_apply(Wg0.copy(), s["U"], s["V"], orc.f64(b["D"]), lr32, wd32)
            check_close(b["W"], Wk, tol, what + " weights from the GPU's own D")
            moved = orc.f64(b["W"]) - Wg0
            e["move_own"], e["move_own_max"] = check_close(moved, Wk - Wg0, bar_move_own, what + " movement from the GPU's own D")
            if t >= compare_d_from:
                e["D"], e["D_max"] = rel_fro(b["D"], D), max_abs_rel(b["D"], D)
                e["move"], e["move_max"] = rel_fro(moved, s["W"] - Wo0), max_abs_rel(moved, s["W"] - Wo0)
            parity_log("%s: %s" % (what, " ".join("%s=%.2e" % (k, v) for k, v in e.items() if k not in ("t", "block"))))
            if t >= compare_d_from:
                assert e["D"] < bar_d, "%s: D against the oracle's trajectory %.3e >= %.1e" % (what, e["D"], bar_d)
                assert e["move"] < bar_move, "%s: movement against the oracle's %.3e >= %.1e" % (what, e["move"], bar_move)
                assert e["move_max"] < 3 * bar_move, "%s: largest movement error %.3e >= %.1e" % (what, e["move_max"], 3 * bar_move)
            if after_block is not None:
                after_block(i, t)
            out.append(e)
    return out
