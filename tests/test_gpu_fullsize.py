"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times (the batched plan over all blocks), on sampled blocks the oracle can afford, and
through size-independent properties where the oracle cannot (the 1B-shape refresh)."""
import numpy as np
import pytest
import torch

import bench
import synth_inputs as si
from oracle import tsr_oracle as orc
from gpu_util import B1, B2, EPS, check_close, dev, f32, max_abs_rel, parity_log, plan_trajectory, projector_err, rel_fro

pytestmark = pytest.mark.gpu
TOL_F32 = 1e-4
TOL_BF16 = 1e-2


@pytest.fixture(scope="module")
def tsr():
    import paper_2602_08007_amd as t
    assert torch.cuda.is_available()
    return t


def orthonormality_defect(X):
    X = orc.f64(X)
    return float(np.abs(X.T @ X - np.eye(X.shape[1])).max())


def distinct_shape_samples(shapes, per_shape=1):
    seen, out = {}, []
    for i, s in enumerate(shapes):
        if seen.get(s, 0) < per_shape:
            seen[s] = seen.get(s, 0) + 1
            out.append(i)
    return out


def fresh_noise(blocks, key):
    """next_grads for plan_trajectory: same signal, a new noise draw on top at every step.
    (Stepping on the very gradient the bases were refreshed from makes the core exactly diagonal
    in exact arithmetic, so that D off the diagonal is decided by rounding noise on either side;
    parity of the trajectory is only well posed on a fresh gradient.)"""
    def put(t):
        for i, b in enumerate(blocks):
            G = b["G"]
            z = si.normal(tuple(G.shape), si.stream_key(key, t, i), std=1e-3, device=G.device)
            G.copy_((G.float() + z).to(G.dtype))
    return put


# Bars against the oracle's own trajectory for bf16 operand arithmetic from a COLD start (zero
# moments, t = 1, 2, 3, as the benchmark configurations state it).  D = mhat / (sqrt(vhat) + eps)
# divides by the size of the core entry: an absolute core error e (about 2e-3 of the core's norm
# spread over r^2 entries) is a relative error e / |c| in D, and most entries are projected noise
# three orders of magnitude below the leading ones.  Measured on every configuration: 1.5e-2 to
# 2.1e-2 at t = 2 (two draws in the moments), 1.1e-2 to 1.3e-2 at t = 3; the bar is 3e-2.  The
# movement from the GPU's own D (the lift's arithmetic alone) measures 3e-3 and keeps 1e-2.
BAR_D_BF16, BAR_MOVE_BF16, BAR_MOVE_OWN_BF16 = 3e-2, 3e-2, 1e-2


def check_step_against_oracle(tsr, w, blocks, plan, sample, tol, steps=(1, 2), label=""):
    """Plan steps on fresh gradients, replayed by the oracle on its own trajectory for the sampled blocks."""
    return plan_trajectory(plan, blocks, sample, steps, tol, label or w.name, lr=1e-3, wd=0.01, workers=w.workers,
                           next_grads=fresh_noise(blocks, si.stream_key(si.BASE_SEED, 77)),
                           bar_d=BAR_D_BF16, bar_move=BAR_MOVE_BF16, bar_move_own=BAR_MOVE_OWN_BF16)


def refresh_parity(w, blocks, omegas, i, label, tol):
    """Bases of block i against the oracle's refresh of the same gradient and Omega; logs the gap."""
    b = blocks[i]
    G = b["G"][0] if b["G"].dim() == 3 else b["G"]
    U_ref, V_ref, S_ref = orc.refresh_rsvd(G, omegas[i], w.r, w.p, w.q)
    eu, ev = projector_err(b["U"], U_ref), projector_err(b["V"], V_ref)
    gap = (S_ref[w.r - 1] - S_ref[w.r]) / S_ref[0]
    parity_log("%s block %d %s refresh (r=%d p=%d q=%d): relative gap %.2e projector errors U %.2e V %.2e"
               % (label, i, tuple(G.shape), w.r, w.p, w.q, gap, eu, ev))
    assert eu < tol and ev < tol, (label, i, eu, ev)
    return gap, eu, ev


# ------------------------------------------------------------------ configuration 2 (the benchmark workload)
def test_llama130m_full_model_step_and_refresh(tsr):
    w = si.workload("llama-130m")
    blocks = bench.build_blocks(w, torch.device("cuda:0"))
    assert len(blocks) == 84
    plan = tsr.Plan(blocks, n_workers=1, precision=tsr.TSR_PREC_BF16, with_refresh=True, p=w.p)
    omegas = [si.omega(n, w.r + w.p, si.stream_key(si.BASE_SEED, 3, i), device="cuda") for i, (m, n) in enumerate(w.shapes)]
    plan.tsr_refresh_batched(omegas, w.q)
    torch.cuda.synchronize()
    # properties on every block: orthonormal bases
    for b in blocks:
        assert orthonormality_defect(b["U"]) < 1e-4 and orthonormality_defect(b["V"]) < 1e-4
    sample = distinct_shape_samples(w.shapes)
    assert len(sample) == 3
    # refresh parity on one block of every distinct shape (bf16 gradient: 1e-2 on projectors)
    for i in sample:
        refresh_parity(w, blocks, omegas, i, "config2 llama-130m", TOL_BF16)
    check_step_against_oracle(tsr, w, blocks, plan, sample, TOL_BF16, steps=(1, 2, 3), label="config2 llama-130m")
    core, dense = plan.payload_bytes(4)
    assert core == 84 * 256 * 256 * 4 and dense == 4 * sum(m * n for m, n in w.shapes)
    plan.close()


# ------------------------------------------------------------------ configuration 3 (1B shapes, r = 512)
def test_llama1b_shapes_step_and_refresh_properties(tsr):
    w = si.workload("llama-1b", layers=2)            # 14 blocks at the full shapes
    blocks = bench.build_blocks(w, torch.device("cuda:0"))
    plan = tsr.Plan(blocks, n_workers=1, precision=tsr.TSR_PREC_BF16, with_refresh=True, p=w.p)
    omegas = [si.omega(n, w.r + w.p, si.stream_key(si.BASE_SEED, 3, i), device="cuda") for i, (m, n) in enumerate(w.shapes)]
    plan.tsr_refresh_batched(omegas, w.q)
    torch.cuda.synchronize()
    sample = distinct_shape_samples(w.shapes)
    for i in sample:
        b = blocks[i]
        assert orthonormality_defect(b["U"]) < 1e-4 and orthonormality_defect(b["V"]) < 1e-4
        # the refreshed bases diagonalize the gradient they came from, and capture (almost) the
        # energy of the best rank-r approximation (LAPACK's singular values as the yardstick)
        G = orc.f64(b["G"]); U = orc.f64(b["U"]); V = orc.f64(b["V"])
        C = U.T @ G @ V
        off = C - np.diag(np.diag(C))
        assert np.linalg.norm(off) / np.linalg.norm(C) < 1e-3
        d = np.diag(C)
        assert np.all(d > 0) and np.all(np.diff(d) <= 1e-6 * d[0])
        s = np.linalg.svd(G, compute_uv=False)
        best = np.sqrt((s[:w.r] ** 2).sum())
        print("1B block %d %s: captured/best energy %.6f" % (i, G.shape, np.linalg.norm(C) / best))
        # spectrum 1/sqrt(i) decays slowly: two power iterations leave a fraction of a percent
        assert np.linalg.norm(C) / best > 0.98
    # full oracle parity of the refresh on the square block (the only one the plain-loop oracle
    # finishes in about half a minute)
    refresh_parity(w, blocks, omegas, sample[0], "config3 llama-1b", TOL_BF16)
    # sampled blocks of the second layer too: the plan's tables, not just its first entries
    check_step_against_oracle(tsr, w, blocks, plan, sample + [len(blocks) - 1], TOL_BF16, steps=(1, 2), label="config3 llama-1b")
    plan.close()


@pytest.mark.parametrize("m,n", [(1100, 1600), (1600, 1100)])
def test_refresh_k528_nonsquare_against_oracle(tsr, m, n):
    """The 1B configuration's refresh parameters (r = 512, p = 16, q = 2, bf16 gradient, spectrum
    1/sqrt(i) + noise) on non-square blocks small enough for the plain-loop oracle."""
    w = si.workload("llama-1b", layers=1)
    key = si.stream_key(si.BASE_SEED, 6, m)
    sig = si.make_signal(m, n, w.signal_rank, w.spectrum, key, device="cuda")
    G = si.gradient(sig, w.noise, si.stream_key(key, 100), dtype=w.g_dtype)
    Om = si.omega(n, w.r + w.p, si.stream_key(key, 3), device="cuda")
    U = torch.empty(m, w.r, device="cuda"); V = torch.empty(n, w.r, device="cuda"); sigma = torch.empty(w.r + w.p, device="cuda")
    tsr.tsr_refresh_rsvd(G, Om, w.r, w.p, w.q, U, V, sigma)
    torch.cuda.synchronize()
    assert orthonormality_defect(U) < 1e-4 and orthonormality_defect(V) < 1e-4
    U_ref, V_ref, S_ref = orc.refresh_rsvd(G, Om, w.r, w.p, w.q)
    gap = (S_ref[w.r - 1] - S_ref[w.r]) / S_ref[0]
    eu, ev, es = projector_err(U, U_ref), projector_err(V, V_ref), rel_fro(sigma, S_ref)
    parity_log("config3-shaped %dx%d refresh (r=512 p=16 q=2, k=528): relative gap %.2e projector errors U %.2e V %.2e sigma %.2e"
               % (m, n, gap, eu, ev, es))
    assert eu < TOL_BF16 and ev < TOL_BF16 and es < TOL_F32


# ------------------------------------------------------------------ configuration 4 (embedding and LM head)
@pytest.mark.parametrize("kind", ["embedding", "lm-head"])
def test_embedding_path_full_size(tsr, kind):
    vocab, d, r, p, q = si.VOCAB, 2048, 128, 8, 1
    key = si.stream_key(si.BASE_SEED, 4, 0 if kind == "embedding" else 1)
    if kind == "embedding":
        ids = si.zipf_ids(256 * 1024, vocab, 1.1, si.stream_key(key, 1))
        G, rows = si.embedding_gradient(vocab, d, ids, si.stream_key(key, 2), std=1e-2, device="cuda")
        assert 15000 < rows.numel() < 26000
        G2, _ = si.embedding_gradient(vocab, d, si.zipf_ids(256 * 1024, vocab, 1.1, si.stream_key(key, 3)),
                                      si.stream_key(key, 4), std=1e-2, device="cuda")
    else:
        sig = si.make_signal(vocab, d, 256, "1/i", key, device="cuda")
        G = si.gradient(sig, 1e-3, si.stream_key(key, 2))
        G2 = si.gradient(sig, 1e-3, si.stream_key(key, 4))
    Om = si.omega(d, r + p, si.stream_key(key, 5), device="cuda")
    U = torch.empty(vocab, r, device="cuda"); V = torch.empty(d, r, device="cuda")
    sigma = torch.empty(r + p, device="cuda")
    tsr.tsr_refresh_rsvd(G, Om, r, p, q, U, V, sigma)
    torch.cuda.synchronize()
    assert orthonormality_defect(U) < 1e-4 and orthonormality_defect(V) < 1e-4
    U_ref, V_ref, S_ref = orc.refresh_rsvd(G, Om, r, p, q)
    gap = (S_ref[r - 1] - S_ref[r]) / S_ref[0]
    eu, ev = projector_err(U, U_ref), projector_err(V, V_ref)
    parity_log("config4 %s 32000x2048 refresh (r=128 p=8 q=1): relative gap %.2e projector errors U %.2e V %.2e sigma %.2e"
               % (kind, gap, eu, ev, rel_fro(sigma, S_ref)))
    assert rel_fro(sigma, S_ref) < TOL_F32
    # the embedding gradient is pure noise on ~20k rows: its top-128 cut is gap limited, so the
    # projector bar scales with the oracle's own relative gap
    bar = max(TOL_F32, 2e-7 / gap)
    assert eu < bar and ev < bar
    # one step on the next gradient, with the oracle's bases on both sides (arithmetic check)
    Ur = dev(torch.from_numpy(U_ref).float()); Vr = dev(torch.from_numpy(V_ref).float())
    W0 = si.weights(vocab, d, si.stream_key(key, 6), device="cuda")
    W = W0.clone()
    C = torch.empty(r, r, device="cuda"); D = torch.empty(r, r, device="cuda")
    M = torch.zeros(r, r, device="cuda"); Vm = torch.zeros(r, r, device="cuda")
    tsr.tsr_project_core(G2, Ur, Vr, C)
    tsr.tsr_adam_core(C, M, Vm, D, 1)
    tsr.tsr_backproject_apply(W, Ur, Vr, D, 1e-3)
    torch.cuda.synchronize()
    Wo = orc.f64(W0).copy(); Mo = np.zeros((r, r)); Vo = np.zeros((r, r))
    Co, Do = orc.tsr_adam_step(Wo, [G2], orc.f64(Ur), orc.f64(Vr), Mo, Vo, 1, lr=f32(1e-3), beta1=B1, beta2=B2, eps=EPS)
    ec, ecm = check_close(C, Co, TOL_F32, kind + " core")
    W_k = orc.backproject_apply(orc.f64(W0).copy(), orc.f64(Ur), orc.f64(Vr), orc.f64(D), f32(1e-3))
    ew, ewm = check_close(W, W_k, TOL_F32, kind + " weights from the GPU's own D")
    em, emm = check_close(orc.f64(W) - orc.f64(W0), W_k - orc.f64(W0), 2e-4, kind + " movement from the GPU's own D")
    parity_log("config4 %s step (oracle's bases): C=%.2e C_max=%.2e W=%.2e W_vs_oracle_trajectory=%.2e move_own=%.2e move_own_max=%.2e"
               % (kind, ec, ecm, ew, rel_fro(W, Wo), em, emm))


# ------------------------------------------------------------------ configuration 5 (K = 8 simulated workers)
def test_llama350m_eight_workers(tsr):
    w = si.workload("llama-350m-dp8", layers=2)      # 14 blocks x 8 worker gradients at the full shapes
    blocks = bench.build_blocks(w, torch.device("cuda:0"))
    assert blocks[0]["G"].shape[0] == 8
    plan = tsr.Plan(blocks, n_workers=8, precision=tsr.TSR_PREC_BF16, with_refresh=True, p=w.p)
    omegas = [si.omega(n, w.r + w.p, si.stream_key(si.BASE_SEED, 3, i), device="cuda") for i, (m, n) in enumerate(w.shapes)]
    plan.tsr_refresh_batched(omegas, w.q)           # bases from worker 0's gradient
    torch.cuda.synchronize()
    sample = distinct_shape_samples(w.shapes)
    for i in sample:
        assert orthonormality_defect(blocks[i]["U"]) < 1e-4 and orthonormality_defect(blocks[i]["V"]) < 1e-4
    check_step_against_oracle(tsr, w, blocks, plan, sample + [len(blocks) - 1], TOL_BF16, steps=(1, 2), label="config5 llama-350m-dp8")
    core, dense = plan.payload_bytes(4)
    # payload of the whole model (24 layers; 2 are resident here, every layer has the same blocks)
    full = si.model_shapes("350m")
    ratio = (4 * sum(m * n for m, n in full)) / (len(full) * 256 * 256 * 4)
    assert abs(ratio - 27.5) < 0.1 and dense / core == pytest.approx(ratio, rel=1e-9)
    parity_log("config5 llama-350m-dp8 payload per step and worker (24 layers): cores %.1f MB, dense fp32 gradient %.1f MB, ratio %.2f"
               % (core * 12 / 1e6, dense * 12 / 1e6, dense / core))
    plan.close()
