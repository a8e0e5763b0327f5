"""GPU parity: the HIP library, called through the C ABI, against the fp64 CPU oracle on the
same seeded inputs.  Tolerances (relative Frobenius error): 1e-4 on cores, updated weights and
subspace projectors for the split-precision ("fp32") path, 1e-2 for bf16 gradients with bf16
operand arithmetic; integer-free, so nothing is bit-exact here.  Per-kernel parity of project /
Adam / lift feeds the ORACLE's bases to the GPU, so that 1e-4 checks arithmetic and not the
conditioning of the subspace."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import tsr_oracle as orc
from gpu_util import B1, B2, EPS, check_close, dev, f32, max_abs_rel, padded, parity_log, plan_trajectory, projector_err, rel_fro

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4
TOL_BF16 = 1e-2


@pytest.fixture(scope="module")
def tsr():
    import paper_2602_08007_amd as t
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    assert t.tsr_device_count() >= 1
    return t


def bases(m, n, r, key):
    return si.orthonormal(m, r, si.stream_key(key, 1)).float(), si.orthonormal(n, r, si.stream_key(key, 2)).float()


# ------------------------------------------------------------------ Adam on the core
@pytest.mark.parametrize("count", [1, 64 * 64, 256 * 256 + 3])
def test_adam_core_steps(tsr, count):
    M = np.zeros(count); Vm = np.zeros(count)
    Md = torch.zeros(count, device="cuda"); Vd = torch.zeros(count, device="cuda"); Dd = torch.empty(count, device="cuda")
    for t in range(1, 6):
        C = si.normal((count,), si.stream_key(7, count, t), std=10.0 ** (-t))
        D = orc.adam_core(C, M, Vm, t, B1, B2, EPS)
        tsr.tsr_adam_core(dev(C), Md, Vd, Dd, t)
        torch.cuda.synchronize()
        assert rel_fro(Dd, D) < 1e-5, t
        assert rel_fro(Md, M) < 1e-6 and rel_fro(Vd, Vm) < 1e-6


def test_adam_first_step_closed_form_on_gpu(tsr):
    g = si.normal((64, 64), 11) * 1e-6
    Md = torch.zeros(64, 64, device="cuda"); Vd = torch.zeros(64, 64, device="cuda"); Dd = torch.empty(64, 64, device="cuda")
    tsr.tsr_adam_core(dev(g), Md, Vd, Dd, 1)
    expect = g.double() / (g.double().abs() + EPS)
    assert rel_fro(Dd, expect) < 1e-5


def test_sgd_core(tsr):
    M = np.zeros((32, 32)); Md = torch.zeros(32, 32, device="cuda"); Dd = torch.empty(32, 32, device="cuda")
    for t in range(1, 4):
        C = si.normal((32, 32), si.stream_key(13, t))
        D = orc.sgd_core(C, M, f32(0.9))
        tsr.tsr_sgd_core(dev(C), Md, Dd, 0.9)
        assert rel_fro(Dd, D) < 1e-6


def test_core_average(tsr):
    Cs = si.normal((8, 64, 64), 17)
    out = torch.empty(64, 64, device="cuda")
    tsr.tsr_core_average(dev(Cs), out)
    assert rel_fro(out, orc.core_average([c for c in Cs])) < 1e-6


# ------------------------------------------------------------------ project
PROJECT_CASES = [
    # m, n, r, dtype, padded ld or None
    (512, 1376, 64, torch.float32, None),      # configuration 1
    (200, 333, 17, torch.float32, None),       # ragged everything, unaligned rows
    (333, 200, 40, torch.float32, 208),
    (130, 257, 130, torch.float32, None),      # r = m
    (768, 2048, 256, torch.bfloat16, None),    # 130M shapes
    (2048, 768, 256, torch.bfloat16, None),
    (301, 515, 33, torch.bfloat16, None),      # odd leading dimension, bf16
    (301, 515, 33, torch.bfloat16, 520),
    (1, 9, 1, torch.float32, None),
]


@pytest.mark.parametrize("m,n,r,dtype,ld", PROJECT_CASES)
@pytest.mark.parametrize("prec", ["split", "bf16"])
def test_project_core(tsr, m, n, r, dtype, ld, prec):
    key = si.stream_key(101, m, n, r)
    sig = si.make_signal(m, n, min(r, 8), "1/i", key)
    G = si.gradient(sig, 1e-3, si.stream_key(key, 3), dtype=dtype)
    U, V = bases(m, n, r, key)
    C_ref = orc.project_core(G, U, V)
    Gd = padded(G, ld) if ld else dev(G)
    C = torch.full((r, r), float("nan"), device="cuda")
    precision = tsr.TSR_PREC_SPLIT if prec == "split" else tsr.TSR_PREC_BF16
    tsr.tsr_project_core(Gd, dev(U), dev(V), C, precision=precision)
    torch.cuda.synchronize()
    tol = TOL_F32 if prec == "split" else TOL_BF16
    check_close(C, C_ref, tol, "core")
    # alpha / accumulate: C <- C + 0.5 * core
    tsr.tsr_project_core(Gd, dev(U), dev(V), C, alpha=0.5, accumulate=True, precision=precision)
    check_close(C, 1.5 * C_ref, tol, "accumulated core")


def test_project_core_identity_closed_form(tsr):
    # U^T (U C0 V^T) V = C0 on the GPU path itself
    m, n, r = 384, 640, 48
    U, V = bases(m, n, r, 202)
    C0 = si.normal((r, r), 203)
    G = (U.double() @ C0.double() @ V.double().T).float()
    C = torch.empty(r, r, device="cuda")
    tsr.tsr_project_core(dev(G), dev(U), dev(V), C)
    assert rel_fro(C, C0) < TOL_F32


def test_worker_average_by_accumulation(tsr):
    m, n, r, K = 256, 384, 32, 4
    key = si.stream_key(301)
    sig = si.make_signal(m, n, r, "1/i", key)
    U, V = bases(m, n, r, key)
    Gs = [si.gradient(sig, 1e-3, si.stream_key(key, 10 + w)) for w in range(K)]
    ref = orc.core_average([orc.project_core(G, U, V) for G in Gs])
    C = torch.zeros(r, r, device="cuda")
    for w, G in enumerate(Gs):
        tsr.tsr_project_core(dev(G), dev(U), dev(V), C, alpha=1.0 / K, accumulate=(w > 0))
    assert rel_fro(C, ref) < TOL_F32


# ------------------------------------------------------------------ lift + apply
LIFT_CASES = [
    (512, 1376, 64, None), (200, 333, 17, None), (333, 200, 40, 208), (768, 2048, 256, None),
    (2048, 768, 256, None), (129, 131, 129, None), (1, 9, 1, None),
]


@pytest.mark.parametrize("m,n,r,ld", LIFT_CASES)
@pytest.mark.parametrize("prec", ["split", "bf16"])
def test_backproject_apply(tsr, m, n, r, ld, prec):
    key = si.stream_key(401, m, n, r)
    U, V = bases(m, n, r, key)
    D = si.normal((r, r), si.stream_key(key, 3)).clamp(-1, 1)
    W0 = si.weights(m, n, si.stream_key(key, 4))
    lr, wd, scale = 1e-2, 0.1, 0.75
    W_ref = orc.backproject_apply(orc.f64(W0).copy(), U, V, D, f32(lr), f32(wd), f32(scale))
    dW_ref = W_ref - orc.f64(W0)
    Wd = padded(W0, ld) if ld else dev(W0)
    precision = tsr.TSR_PREC_SPLIT if prec == "split" else tsr.TSR_PREC_BF16
    tsr.tsr_backproject_apply(Wd, dev(U), dev(V), dev(D), lr, wd, scale, precision=precision)
    torch.cuda.synchronize()
    tol = TOL_F32 if prec == "split" else TOL_BF16
    check_close(Wd, W_ref, tol, "weights")
    # the update itself (not hidden behind the much larger W)
    dW = orc.f64(Wd) - orc.f64(W0)
    check_close(dW, dW_ref, 2e-4 if prec == "split" else TOL_BF16, "movement")
    if ld:   # padding columns untouched
        assert torch.count_nonzero(Wd._base[:, n:]).item() == 0 if Wd._base is not None else True


# ------------------------------------------------------------------ refresh
def run_refresh(tsr, G, Om, r, p, q):
    m, n = G.shape
    U = torch.empty(m, r, device="cuda"); V = torch.empty(n, r, device="cuda")
    sigma = torch.empty(r + p, device="cuda")
    tsr.tsr_refresh_rsvd(dev(G), dev(Om), r, p, q, U, V, sigma)
    torch.cuda.synchronize()
    return U, V, sigma


def check_orthonormal(X, tol=1e-4):
    X = orc.f64(X)
    assert np.abs(X.T @ X - np.eye(X.shape[1])).max() < tol


# the last case has k = r + p = 560: beyond the blocked Cholesky and the multi-launch small SVD
# (both for k <= 544), so it runs their general variants (unblocked Cholesky, single-kernel QL)
@pytest.mark.parametrize("m,n,r,p,q", [(96, 160, 8, 4, 1), (160, 96, 8, 4, 0), (300, 260, 24, 8, 2),
                                       (640, 600, 552, 8, 1)])
def test_refresh_well_separated_spectrum(tsr, m, n, r, p, q):
    # singular values 2 .. 1 then a gap down to the noise: the top-r subspace is well conditioned
    G64, A, B = si.exact_lowrank(m, n, r, si.stream_key(501, m, n))
    G = (G64 + 1e-3 * si.normal((m, n), si.stream_key(502, m), dtype=torch.float64)).float()
    Om = si.omega(n, r + p, si.stream_key(503, n))
    U_ref, V_ref, S_ref = orc.refresh_rsvd(G, Om, r, p, q)
    U, V, sigma = run_refresh(tsr, G, Om, r, p, q)
    check_orthonormal(U); check_orthonormal(V)
    assert projector_err(U, U_ref) < TOL_F32
    assert projector_err(V, V_ref) < TOL_F32
    # the r retained singular values carry the bar; of the p oversampling directions, those whose
    # Cholesky pivot falls below the fp32 Gram matrix's resolution are dropped as dependent
    # (zero singular value) where Householder QR keeps them -- they never enter U or V
    assert rel_fro(sigma[:r], S_ref[:r]) < TOL_F32
    tail = orc.f64(sigma[r:])
    assert np.all((np.abs(tail - S_ref[r:]) < 1e-3 * S_ref[0]) | (tail < 1e-6 * S_ref[0]))


def test_refresh_exact_rank_r_input(tsr):
    # rank(G) = r < k: the sketch is rank deficient; the subspace must still be recovered
    m, n, r, p = 200, 150, 10, 6
    G64, A, B = si.exact_lowrank(m, n, r, 511)
    Om = si.omega(n, r + p, 512)
    U, V, sigma = run_refresh(tsr, G64.float(), Om, r, p, 1)
    check_orthonormal(U); check_orthonormal(V)
    assert projector_err(U, A) < TOL_F32
    assert projector_err(V, B) < TOL_F32
    assert rel_fro(sigma[:r], np.linspace(2.0, 1.0, r)) < TOL_F32
    assert float(sigma[r:].abs().max()) < 1e-4


@pytest.mark.parametrize("m,n", [(200, 150), (130, 320)])
def test_refresh_repeated_singular_values(tsr, m, n):
    # exact rank 8 with singular values 4,4,4,2,2,2,2,1: inside a group of equal values any
    # orthonormal basis is a valid set of singular vectors, so what is unique is compared: the
    # values, the top-r subspace, the subspace of the leading group, orthonormality.  The
    # eigen-solver sees groups of (numerically) equal eigenvalues plus p zeros.
    r, p = 8, 4
    A = si.orthonormal(m, r, si.stream_key(521, m))
    B = si.orthonormal(n, r, si.stream_key(522, n))
    sv = torch.tensor([4.0, 4.0, 4.0, 2.0, 2.0, 2.0, 2.0, 1.0], dtype=torch.float64)
    G64 = (A * sv[None, :]) @ B.T
    Om = si.omega(n, r + p, si.stream_key(523, n))
    U, V, sigma = run_refresh(tsr, G64.float(), Om, r, p, 1)
    check_orthonormal(U); check_orthonormal(V)
    assert projector_err(U, A) < TOL_F32 and projector_err(V, B) < TOL_F32
    assert projector_err(U[:, :3], A[:, :3]) < 1e-3 and projector_err(V[:, :3], B[:, :3]) < 1e-3
    assert rel_fro(sigma[:r], sv.numpy()) < TOL_F32
    assert float(sigma[r:].abs().max()) < 1e-4
    # the same through the oracle: values and subspaces agree
    Uo, Vo, so = orc.refresh_rsvd(G64.float().numpy(), orc.f64(Om), r, p, 1)
    assert projector_err(U, Uo) < TOL_F32 and projector_err(V, Vo) < TOL_F32
    assert rel_fro(sigma[:r], so[:r]) < TOL_F32


@pytest.mark.parametrize("g_dtype", [torch.float32, torch.bfloat16])
def test_refresh_steep_full_rank_spectrum(tsr, g_dtype):
    # full-rank gradient with a steep spectrum, sigma_i = 1 / i^2, noise 1e-7: sigma_r / sigma_1 =
    # 6e-4 lies INSIDE the retained rank, and the sketch's Gram matrix has a condition number of
    # about 1e9, far beyond what an unshifted Cholesky QR survives.  The bases must come out
    # orthonormal with no direction dropped; singular values and captured energy are well posed
    # (Weyl); the top-r projector is limited by the gap sigma_r - sigma_{r+1} = 3e-5 sigma_1 (its bar
    # scales with the oracle's gap, as for configuration 1), the leading directions are not.
    m, n, r, p, q = 300, 260, 40, 8, 1
    s_min = min(m, n)
    A = si.orthonormal(m, s_min, si.stream_key(541, 1)); B = si.orthonormal(n, s_min, si.stream_key(541, 2))
    sv = 1.0 / torch.arange(1, s_min + 1, dtype=torch.float64) ** 2
    G = ((A * sv[None, :]) @ B.T + 1e-7 * si.normal((m, n), si.stream_key(541, 3), dtype=torch.float64)).float().to(g_dtype)
    Om = si.omega(n, r + p, si.stream_key(541, 4))
    U_ref, V_ref, S_ref = orc.refresh_rsvd(G, Om, r, p, q)
    U, V, sigma = run_refresh(tsr, G, Om, r, p, q)
    check_orthonormal(U); check_orthonormal(V)
    assert float(orc.f64(U).std(axis=0).min()) > 0 and float(np.linalg.norm(orc.f64(U), axis=0).min()) > 0.999    # no zero column
    assert float(np.linalg.norm(orc.f64(V), axis=0).min()) > 0.999
    es = float(np.abs(orc.f64(sigma) - S_ref).max() / S_ref[0])
    gap = (S_ref[r - 1] - S_ref[r]) / S_ref[0]
    eu, ev = projector_err(U, U_ref), projector_err(V, V_ref)
    eu8, ev8 = projector_err(U[:, :8], U_ref[:, :8]), projector_err(V[:, :8], V_ref[:, :8])
    e_ref = np.linalg.norm(U_ref.T @ orc.f64(G) @ V_ref)
    e_gpu = np.linalg.norm(orc.f64(U).T @ orc.f64(G) @ orc.f64(V))
    parity_log("steep spectrum 1/i^2 %dx%d r=%d %s: relative gap %.2e sigma err / sigma_1 %.2e projector errors U %.2e V %.2e "
               "leading-8 U %.2e V %.2e captured energy diff %.2e"
               % (m, n, r, str(g_dtype)[6:], gap, es, eu, ev, eu8, ev8, abs(e_gpu - e_ref) / e_ref))
    assert es < 1e-5
    assert abs(e_gpu - e_ref) / e_ref < 1e-5
    assert eu8 < 1e-3 and ev8 < 1e-3
    assert eu < max(TOL_F32, 2e-7 / gap) and ev < max(TOL_F32, 2e-7 / gap)


def test_refresh_zero_gradient_is_finite(tsr):
    # degenerate input: nothing to find.  Every sketch column is dropped as dependent, the
    # singular values are zero and the bases come out as zeros: finite, no NaN from 0 / 0
    m, n, r, p = 96, 160, 8, 4
    Om = si.omega(n, r + p, 531)
    U, V, sigma = run_refresh(tsr, torch.zeros(m, n), Om, r, p, 1)
    assert torch.isfinite(U).all() and torch.isfinite(V).all() and torch.isfinite(sigma).all()
    assert float(sigma.abs().max()) == 0.0
    assert float(U.abs().max()) == 0.0 and float(V.abs().max()) == 0.0


def test_refresh_config1(tsr):
    # 512 x 1376, r = 64, p = 8, q = 1, spectrum 1/i + noise 1e-3.  The tail of the signal is
    # below the noise, so the top-r projector is gap limited: the well conditioned quantities
    # (singular values, orthonormality, captured energy) carry the 1e-4 bar, the projector is
    # compared with a bar scaled by the oracle's own relative gap.
    w = si.workload("single-60m")
    m, n = w.shapes[0]
    sig = si.make_signal(m, n, w.signal_rank, w.spectrum, si.stream_key(si.BASE_SEED, 1))
    G = si.gradient(sig, w.noise, si.stream_key(si.BASE_SEED, 1, 1))
    Om = si.omega(n, w.r + w.p, si.stream_key(si.BASE_SEED, 1, 99))
    U_ref, V_ref, S_ref = orc.refresh_rsvd(G, Om, w.r, w.p, w.q)
    U, V, sigma = run_refresh(tsr, G, Om, w.r, w.p, w.q)
    check_orthonormal(U); check_orthonormal(V)
    assert rel_fro(sigma, S_ref) < TOL_F32
    gap = (S_ref[w.r - 1] - S_ref[w.r]) / S_ref[0]
    eu, ev = projector_err(U, U_ref), projector_err(V, V_ref)
    parity_log("config1 single-60m 512x1376 refresh (r=64 p=8 q=1): relative gap %.2e projector errors U %.2e V %.2e sigma %.2e"
               % (gap, eu, ev, rel_fro(sigma, S_ref)))
    assert eu < max(TOL_F32, 2e-7 / gap) and ev < max(TOL_F32, 2e-7 / gap)
    # captured energy ||U^T G V||_F agrees
    e_ref = np.linalg.norm(U_ref.T @ orc.f64(G) @ V_ref)
    e_gpu = np.linalg.norm(orc.f64(U).T @ orc.f64(G) @ orc.f64(V))
    assert abs(e_gpu - e_ref) / e_ref < 1e-5


def test_refresh_bf16_gradient(tsr):
    m, n, r, p, q = 768, 768, 64, 8, 1
    G64, A, B = si.exact_lowrank(m, n, r, 521)
    G = (G64.float() + si.normal((m, n), 522, std=1e-3)).to(torch.bfloat16)
    Om = si.omega(n, r + p, 523)
    U_ref, V_ref, S_ref = orc.refresh_rsvd(G, Om, r, p, q)
    U, V, sigma = run_refresh(tsr, G, Om, r, p, q)
    check_orthonormal(U); check_orthonormal(V)
    assert projector_err(U, U_ref) < TOL_F32 and projector_err(V, V_ref) < TOL_F32
    assert rel_fro(sigma, S_ref) < TOL_F32


# ------------------------------------------------------------------ refresh with several workers
def _sign_fix(U, V):
    U, V = orc.f64(U).copy(), orc.f64(V).copy()
    s = np.sign(V[np.abs(V).argmax(axis=0), np.arange(V.shape[1])])
    return U * s, V * s


@pytest.mark.parametrize("workers,g_dtype,q", [(1, torch.float32, 1), (3, torch.float32, 1), (4, torch.bfloat16, 0),
                                               (2, torch.float32, 2)])
def test_refresh_workers_matches_oracle(tsr, workers, g_dtype, q):
    # shared well-separated signal (singular values 2 .. 1), independent noise per worker: the
    # averaged sketches, hence sigma, V and the (non-orthonormal) U = Qbar Ut_r, are well conditioned
    m, n, r, p = 300, 260, 24, 8
    G64, _, _ = si.exact_lowrank(m, n, r, si.stream_key(801, workers))
    Gs = torch.stack([(G64 + 2e-2 * si.normal((m, n), si.stream_key(802, w), dtype=torch.float64)).float().to(g_dtype)
                      for w in range(workers)])
    Om = si.omega(n, r + p, si.stream_key(803, workers))
    U_ref, V_ref, S_ref, Qbar, Bbar = orc.refresh_rsvd_workers([g for g in Gs], Om, r, p, q)
    U = torch.empty(m, r, device="cuda"); V = torch.empty(n, r, device="cuda"); sigma = torch.empty(r + p, device="cuda")
    tsr.tsr_refresh_rsvd_workers(dev(Gs), dev(Om), r, p, q, U, V, sigma)
    torch.cuda.synchronize()
    assert rel_fro(sigma[:r], S_ref[:r]) < TOL_F32
    check_orthonormal(V)
    Ug, Vg = _sign_fix(U, V)
    Ur, Vr = _sign_fix(U_ref, V_ref)
    assert np.linalg.norm(Vg - Vr) / np.linalg.norm(Vr) < 5e-4, np.linalg.norm(Vg - Vr) / np.linalg.norm(Vr)
    assert np.linalg.norm(Ug - Ur) / np.linalg.norm(Ur) < 5e-4, np.linalg.norm(Ug - Ur) / np.linalg.norm(Ur)
    # sign-free: the lifted rank-r matrix U diag(sigma_r) V^T; then the Gram matrix of U
    lift_ref = (U_ref * S_ref[:r]) @ V_ref.T
    lift_gpu = (orc.f64(U) * orc.f64(sigma[:r])) @ orc.f64(V).T
    assert rel_fro(lift_gpu, lift_ref) < TOL_F32
    assert np.abs(Ug.T @ Ug - Ur.T @ Ur).max() < 5e-4          # columns oriented alike first
    if workers > 1:
        assert np.linalg.norm(U_ref.T @ U_ref - np.eye(r)) > 1e-4       # the defect is real and reproduced above


# ------------------------------------------------------------------ comparison paths of the ablations
@pytest.mark.parametrize("m,n,r,dtype,prec", [(200, 333, 17, torch.float32, "split"), (333, 200, 40, torch.float32, "split"),
                                              (768, 2048, 256, torch.bfloat16, "bf16"), (512, 1376, 64, torch.bfloat16, "split")])
def test_one_sided_project_adam_lift(tsr, m, n, r, dtype, prec):
    # the one-sided variant (object U^T G, r x n) on the same kernels: two steps from a warm start,
    # the oracle on its own trajectory; the GPU holds the object transposed (n x r)
    key = si.stream_key(871, m, n, r)
    sig = si.make_signal(m, n, min(r, 16), "1/i", key)
    U = si.orthonormal(m, r, si.stream_key(key, 1)).float()
    W0 = si.weights(m, n, si.stream_key(key, 4))
    precision = tsr.TSR_PREC_SPLIT if prec == "split" else tsr.TSR_PREC_BF16
    tol = TOL_F32 if prec == "split" else TOL_BF16
    lr, wd = f32(1e-3), f32(0.01)
    W = orc.f64(W0).copy(); M1 = np.zeros((r, n)); V1 = np.zeros((r, n))
    U64 = orc.f64(U)
    grads = [si.gradient(sig, 1e-3, si.stream_key(key, 10 + t), dtype=dtype) for t in range(1, 6)]
    for t in (1, 2, 3):                                       # warm start: the oracle alone
        orc.one_sided_adam_step(W, [grads[t - 1]], U64, M1, V1, t, lr=lr, wd=wd, beta1=B1, beta2=B2, eps=EPS)
    Wd = dev(torch.from_numpy(W).float()); W = orc.f64(Wd).copy()
    Md = dev(torch.from_numpy(M1.T.copy()).float()); Vd = dev(torch.from_numpy(V1.T.copy()).float())   # n x r on the GPU
    M1[...] = orc.f64(Md).T; V1[...] = orc.f64(Vd).T
    Ud = dev(U)
    Ct = torch.full((n, r), float("nan"), device="cuda"); Dt = torch.empty(n, r, device="cuda")
    for t in (4, 5):
        G = grads[t - 1]
        Wg0, Wo0 = orc.f64(Wd).copy(), W.copy()
        C1, D1 = orc.one_sided_adam_step(W, [G], U64, M1, V1, t, lr=lr, wd=wd, beta1=B1, beta2=B2, eps=EPS)
        tsr.tsr_project_one_sided(dev(G), Ud, Ct, precision=precision)
        tsr.tsr_adam_core(Ct, Md, Vd, Dt, t)
        tsr.tsr_backproject_one_sided(Wd, Ud, Dt, 1e-3, 0.01, precision=precision)
        torch.cuda.synchronize()
        ec, _ = check_close(Ct, C1.T, tol, "one-sided object t=%d" % t)
        check_close(Md, M1.T, tol, "first moment"); check_close(Vd, V1.T, 2 * tol, "second moment")
        ew, _ = check_close(Wd, W, tol, "weights t=%d" % t)
        Wk = orc.backproject_one_sided(Wg0.copy(), U64, orc.f64(Dt).T, lr, wd)
        check_close(Wd, Wk, tol, "weights from the GPU's own D")
        emo, _ = check_close(orc.f64(Wd) - Wg0, Wk - Wg0, BAR_MOVE_OWN[prec], "movement from the GPU's own D")
        ed, em = rel_fro(Dt, D1.T), rel_fro(orc.f64(Wd) - Wg0, W - Wo0)
        parity_log("one-sided %dx%d r=%d %s t=%d: C=%.2e W=%.2e move_own=%.2e D=%.2e move=%.2e" % (m, n, r, prec, t, ec, ew, emo, ed, em))
        assert ed < BAR_D[prec] and em < BAR_MOVE[prec], (t, ed, em)
    # accumulate / alpha as in the two-sided call
    ref = orc.project_one_sided(grads[4], U64).T
    tsr.tsr_project_one_sided(dev(grads[4]), Ud, Ct, alpha=0.5, accumulate=True, precision=precision)
    check_close(Ct, 1.5 * ref, tol, "accumulated one-sided object")


@pytest.mark.parametrize("m,n,r,dtype", [(96, 160, 8, torch.float32), (160, 96, 8, torch.float32), (130, 131, 24, torch.bfloat16),
                                         (512, 1376, 64, torch.float32)])
def test_refresh_exact_svd_matches_oracle(tsr, m, n, r, dtype):
    # well separated leading singular values (2 .. 1), then the noise floor
    G64, A, B = si.exact_lowrank(m, n, r, si.stream_key(881, m, n))
    G = (G64 + 1e-3 * si.normal((m, n), si.stream_key(882, m), dtype=torch.float64)).float().to(dtype)
    U = torch.empty(m, r, device="cuda"); V = torch.empty(n, r, device="cuda"); sigma = torch.empty(min(m, n), device="cuda")
    tsr.tsr_refresh_exact_svd(dev(G), r, U, V, sigma)
    torch.cuda.synchronize()
    check_orthonormal(U); check_orthonormal(V)
    U_ref, V_ref, S_ref = orc.refresh_exact_svd(G, r)
    eu, ev, es = projector_err(U, U_ref), projector_err(V, V_ref), rel_fro(sigma[:r], S_ref[:r])
    parity_log("exact-SVD refresh %dx%d r=%d %s: projector errors U %.2e V %.2e sigma_r %.2e" % (m, n, r, str(dtype)[6:], eu, ev, es))
    assert eu < TOL_F32 and ev < TOL_F32 and es < TOL_F32
    # LAPACK agrees on what is unique (the leading values; the subspace through the projector)
    u, s, vt = np.linalg.svd(orc.f64(G), full_matrices=False)
    assert rel_fro(sigma[:r], s[:r]) < TOL_F32 and projector_err(U, u[:, :r]) < TOL_F32
    # the whole spectrum: absolute accuracy relative to the largest value
    assert np.abs(orc.f64(sigma) - S_ref).max() < 1e-4 * S_ref[0]
    # the randomized refresh finds the same subspace (the comparison the ablation makes)
    p, q = 8, 1
    if r + p <= min(m, n):
        Om = si.omega(n, r + p, si.stream_key(883, n))
        Ur = torch.empty(m, r, device="cuda"); Vr = torch.empty(n, r, device="cuda")
        tsr.tsr_refresh_rsvd(dev(G), dev(Om), r, p, q, Ur, Vr)
        assert projector_err(Ur, U) < 1e-3 and projector_err(Vr, V) < 1e-3


# ------------------------------------------------------------------ moment re-alignment
@pytest.mark.parametrize("m,n,r", [(300, 260, 24), (768, 2048, 256), (130, 75, 33)])
def test_realign_moment_matches_oracle(tsr, m, n, r):
    # new bases = old bases turned by a small random rotation of the whole space plus noise, as a
    # refresh produces; also checks that in-place use leaves nothing else touched
    Uo, Vo = bases(m, n, r, si.stream_key(851, m))
    Un, Vn = bases(m, n, r, si.stream_key(852, m))
    # not orthonormal on purpose: the formula does not need it
    Un = (si.orthonormal(m, r, si.stream_key(853, m)) * 0.2 + Uo).float().contiguous()
    Vn = (si.orthonormal(n, r, si.stream_key(854, m)) * 0.2 + Vo).float().contiguous()
    M0 = si.normal((r, r), si.stream_key(855, m))
    M_ref = orc.realign_moment(M0, Uo, Vo, Un, Vn)
    M = dev(M0)
    tsr.tsr_realign_moment(dev(Uo), dev(Vo), dev(Un), dev(Vn), M)
    torch.cuda.synchronize()
    assert rel_fro(M, M_ref) < TOL_F32


# ------------------------------------------------------------------ configuration 1 end to end
def test_config1_refresh_then_ten_steps(tsr):
    """Refresh on G_1, then steps 1..10 on G_1..G_10 (the initial refresh and step 1 share a
    gradient, as a refresh step inside the loop does).

    At that shared step the core is diag(sigma) in exact arithmetic (U^T G V = Ut_r^T B Vt_r),
    so every off-diagonal entry of C is pure rounding noise and D = c / (|c| + 1e-8) there is
    decided by noise of either implementation: parity of D_1 (hence of the absolute W_t) is
    ill-posed.  What is well posed is checked to the fp32 bar: C, m, v at every step, D and
    the weight movement from step 2 on, and each kernel at step 1 against the oracle applied
    to that kernel's own inputs."""
    w = si.workload("single-60m")
    m, n = w.shapes[0]
    r = w.r
    lr = f32(1e-3)
    base = si.stream_key(si.BASE_SEED, 1)
    sig = si.make_signal(m, n, w.signal_rank, w.spectrum, base)
    W0 = si.weights(m, n, si.stream_key(base, 7))
    Om = si.omega(n, r + w.p, si.stream_key(base, 99))
    grads = [si.gradient(sig, w.noise, si.stream_key(base, t)) for t in range(1, 11)]
    U_ref, V_ref, _ = orc.refresh_rsvd(grads[0], Om, r, w.p, w.q)
    # track A: the GPU kernels fed with the oracle's bases (rounded to fp32 for both sides)
    Ur, Vr = dev(torch.from_numpy(U_ref).float()), dev(torch.from_numpy(V_ref).float())
    Ur64, Vr64 = orc.f64(Ur), orc.f64(Vr)
    Wa = dev(W0); Ma = torch.zeros(r, r, device="cuda"); Va = torch.zeros(r, r, device="cuda")
    Ca = torch.empty(r, r, device="cuda"); Da = torch.empty(r, r, device="cuda")
    # track B: the GPU's own refresh
    U = torch.empty(m, r, device="cuda"); V = torch.empty(n, r, device="cuda")
    tsr.tsr_refresh_rsvd(dev(grads[0]), dev(Om), r, w.p, w.q, U, V)
    Wb = dev(W0); Mb = torch.zeros(r, r, device="cuda"); Vb = torch.zeros(r, r, device="cuda")
    Cb = torch.empty(r, r, device="cuda"); Db = torch.empty(r, r, device="cuda")
    # oracle
    W = orc.f64(W0).copy(); M = np.zeros((r, r)); Vm = np.zeros((r, r))
    wnorm = np.linalg.norm(W)
    W1 = Wa1 = Wb1 = None
    for t, G in enumerate(grads, start=1):
        Cbar, D = orc.tsr_adam_step(W, [G], Ur64, Vr64, M, Vm, t, lr=lr, beta1=B1, beta2=B2, eps=EPS)
        Gd = dev(G)
        W_before = orc.f64(Wa).copy()
        tsr.tsr_project_core(Gd, Ur, Vr, Ca); tsr.tsr_adam_core(Ca, Ma, Va, Da, t)
        tsr.tsr_backproject_apply(Wa, Ur, Vr, Da, lr)
        assert rel_fro(Ca, Cbar) < TOL_F32, t
        assert rel_fro(Ma, M) < TOL_F32 and rel_fro(Va, Vm) < 2 * TOL_F32, t
        if t == 1:
            assert np.abs(np.diag(orc.f64(Da)) - np.diag(D)).max() < 1e-5
            assert float(Da.abs().max()) <= 1.0 + 1e-6
            # each kernel against the oracle on that kernel's own inputs
            D_k = orc.adam_core(orc.f64(Ca), np.zeros((r, r)), np.zeros((r, r)), 1, B1, B2, EPS)
            assert rel_fro(Da, D_k) < 1e-5
            W_k = orc.backproject_apply(W_before.copy(), Ur64, Vr64, orc.f64(Da), lr)
            assert rel_fro(Wa, W_k) < TOL_F32
            assert rel_fro(orc.f64(Wa) - W_before, W_k - W_before) < 2e-4
            W1, Wa1 = W.copy(), orc.f64(Wa).copy()
        else:
            # D divides by |c|: an absolute error e in an off-diagonal core entry of size ~1e-3
            # (projected noise) is a relative error e / 1e-3 in D; e ~ 1e-6 for the split path
            assert rel_fro(Da, D) < 5e-3, t
            moved_ref = W - W1
            moved = orc.f64(Wa) - Wa1
            assert np.linalg.norm(moved - moved_ref) / wnorm < TOL_F32, t
            parity_log("config1 single-60m t=%d (oracle's bases, refresh gradient = G_1): C=%.2e D=%.2e movement since t=1: %.2e"
                       % (t, rel_fro(Ca, Cbar), rel_fro(Da, D), rel_fro(moved, moved_ref)))
            assert rel_fro(moved, moved_ref) < 5e-3, t
        tsr.tsr_project_core(Gd, U, V, Cb); tsr.tsr_adam_core(Cb, Mb, Vb, Db, t)
        tsr.tsr_backproject_apply(Wb, U, V, Db, lr)
        if t == 1:
            Wb1 = orc.f64(Wb).copy()
    # track B: weight movement after the shared step, own bases vs oracle bases (sign free)
    moved_ref = W - W1
    moved_b = orc.f64(Wb) - Wb1
    parity_log("config1 single-60m own bases (GPU refresh): movement error / |W| = %.2e, / |movement| = %.2e"
               % (np.linalg.norm(moved_b - moved_ref) / wnorm, rel_fro(moved_b, moved_ref)))
    assert np.linalg.norm(moved_b - moved_ref) / wnorm < TOL_F32


def test_config1_separate_refresh_gradient_ten_steps(tsr):
    """The well-posed variant of configuration 1: the bases come from a refresh on a separate draw
    G_0, then steps 1..10 run on G_1..G_10 with the oracle's bases on both sides and the oracle on
    its own trajectory (nothing re-synchronised).  No step projects the gradient its bases were
    computed from, so the core is generic and the absolute weights are comparable: 1e-4 on the
    core, the moments and W_t at every step, and the bars of the fp32 path on D and on the
    movement (from step 2 on; D_1 = sign(c) is decided by rounding for the smallest entries)."""
    w = si.workload("single-60m")
    m, n = w.shapes[0]
    r = w.r
    lr = f32(1e-3)
    base = si.stream_key(si.BASE_SEED, 1)
    sig = si.make_signal(m, n, w.signal_rank, w.spectrum, base)
    W0 = si.weights(m, n, si.stream_key(base, 7))
    Om = si.omega(n, r + w.p, si.stream_key(base, 99))
    G0 = si.gradient(sig, w.noise, si.stream_key(base, 500))
    U_ref, V_ref, _ = orc.refresh_rsvd(G0, Om, r, w.p, w.q)
    Ur, Vr = dev(torch.from_numpy(U_ref).float()), dev(torch.from_numpy(V_ref).float())
    Ur64, Vr64 = orc.f64(Ur), orc.f64(Vr)
    Wd = dev(W0); Md = torch.zeros(r, r, device="cuda"); Vd = torch.zeros(r, r, device="cuda")
    Cd = torch.empty(r, r, device="cuda"); Dd = torch.empty(r, r, device="cuda")
    W = orc.f64(W0).copy(); M = np.zeros((r, r)); Vm = np.zeros((r, r))
    for t in range(1, 11):
        G = si.gradient(sig, w.noise, si.stream_key(base, 500 + t))
        W_prev, Wd_prev = W.copy(), orc.f64(Wd).copy()
        Cbar, D = orc.tsr_adam_step(W, [G], Ur64, Vr64, M, Vm, t, lr=lr, beta1=B1, beta2=B2, eps=EPS)
        tsr.tsr_project_core(dev(G), Ur, Vr, Cd); tsr.tsr_adam_core(Cd, Md, Vd, Dd, t)
        tsr.tsr_backproject_apply(Wd, Ur, Vr, Dd, lr)
        torch.cuda.synchronize()
        ec, _ = check_close(Cd, Cbar, TOL_F32, "core t=%d" % t)
        check_close(Md, M, TOL_F32, "first moment t=%d" % t); check_close(Vd, Vm, 2 * TOL_F32, "second moment t=%d" % t)
        ew, ewm = check_close(Wd, W, TOL_F32, "weights t=%d" % t)
        ed, em = rel_fro(Dd, D), rel_fro(orc.f64(Wd) - Wd_prev, W - W_prev)
        parity_log("config1 single-60m t=%d (oracle's bases, refresh gradient G_0 separate): C=%.2e W=%.2e W_max=%.2e D=%.2e move=%.2e"
                   % (t, ec, ew, ewm, ed, em))
        if t >= 2:
            assert ed < 5e-3 and em < 5e-3, (t, ed, em)
    # the whole displacement after ten steps
    total = rel_fro(orc.f64(Wd) - orc.f64(W0), W - orc.f64(W0))
    parity_log("config1 single-60m W_10 - W_0 against the oracle's: %.2e" % total)
    assert total < 5e-3


# ------------------------------------------------------------------ batched plan
SENTINEL = 12345.0


def guarded(x: torch.Tensor, extra_rows=3, extra_cols=8):
    """GPU copy of x as a view inside a larger buffer whose surroundings hold a sentinel."""
    m, n = x.shape
    full = torch.full((m + extra_rows, n + extra_cols), SENTINEL, dtype=x.dtype, device="cuda")
    full[:m, :n] = x.to("cuda")
    return full[:m, :n], full


def guards_intact(full: torch.Tensor, m: int, n: int) -> bool:
    return bool((full[m:, :] == SENTINEL).all() and (full[:m, n:] == SENTINEL).all())


def make_blocks(shapes, r, workers, g_dtype, key, noise=1e-3, guard_w=False, pad_g=False):
    blocks, host = [], []
    for i, (m, n) in enumerate(shapes):
        k = si.stream_key(key, i)
        sig = si.make_signal(m, n, r, "1/i", k)
        Gs = torch.stack([si.gradient(sig, noise, si.stream_key(k, 10 + w), dtype=g_dtype) for w in range(workers)])
        U, V = bases(m, n, r, k)
        W0 = si.weights(m, n, si.stream_key(k, 4))
        host.append(dict(G=Gs, U=U, V=V, W=W0, sig=sig, key=k, noise=noise, g_dtype=g_dtype, workers=workers))
        Wd, Wfull = guarded(W0) if guard_w else (dev(W0), None)
        host[-1]["W_full"] = Wfull
        Gd = dev(Gs) if workers > 1 else dev(Gs[0])
        if pad_g:
            # row pitch rounded up to 8 elements; the padding holds NaN, which no kernel may let through
            ld = (n + 7) // 8 * 8
            Gp = torch.full((*Gd.shape[:-1], ld), float("nan"), dtype=Gd.dtype, device="cuda")
            Gp[..., :n] = Gd
            Gd = Gp[..., :n]
        blocks.append(dict(G=Gd, W=Wd, U=dev(U), V=dev(V),
                           M=torch.zeros(r, r, device="cuda"), Vm=torch.zeros(r, r, device="cuda"),
                           C=torch.empty(r, r, device="cuda"), D=torch.empty(r, r, device="cuda")))
    return blocks, host


def fresh_gradients(blocks, host):
    """next_grads for plan_trajectory: a new noise draw per step and worker on the same signal,
    written into the device buffers the plan was created on (padding, if any, is left alone)."""
    def put(t):
        if t == 1:
            return                      # step 1 runs on the gradients the blocks were made with
        for b, h in zip(blocks, host):
            Gs = torch.stack([si.gradient(h["sig"], h["noise"], si.stream_key(h["key"], 1000 * t + w), dtype=h["g_dtype"])
                              for w in range(h["workers"])])
            b["G"].copy_(Gs.to("cuda") if h["workers"] > 1 else Gs[0].to("cuda"))
    return put


# Bars of the checks against the oracle's own trajectory (no re-synchronisation) from a warm
# start (see plan_trajectory).  The core, the moments and the weights carry the stated tolerance
# of the arithmetic (1e-4 split, 1e-2 bf16 operands).  The normalized update D = mhat / (sqrt(vhat)
# + eps) divides by the size of the core entry, so an absolute core error e (uniform over the
# entries: about 2e-6 resp. 2e-3 of the core's norm, spread over r^2 entries) is a relative error
# e / |c| in D, largest where the entry is smallest; D and the movement W_t - W_{t-1} therefore
# carry ten to thirty times the core's error, more the smaller the block (fewer entries to
# average over).  Measured over all cases of this file: split 1.0e-4, bf16 9e-3 .. 6.0e-2 (r = 512
# .. r = 64 blocks; the model-sized blocks of test_gpu_fullsize.py measure 1e-2 .. 2e-2); the
# movement computed from the GPU's OWN D (the lift's arithmetic alone) measures 1.9e-5 resp.
# 3.3e-3 and keeps the stated tolerance.
BAR_D = {"split": 3e-4, "bf16": 1e-1}
BAR_MOVE = {"split": 3e-4, "bf16": 1e-1}
BAR_MOVE_OWN = {"split": TOL_F32, "bf16": TOL_BF16}
COLD_BAR = {"split": 1e-3, "bf16": 2e-1}
WARM = 3          # steps the oracle runs alone before the compared ones


@pytest.mark.parametrize("workers,g_dtype,prec", [(1, torch.float32, "split"), (1, torch.bfloat16, "bf16"),
                                                  (3, torch.bfloat16, "split"), (3, torch.bfloat16, "bf16"),
                                                  (1, torch.float32, "bf16")])
def test_step_batched_matches_oracle(tsr, workers, g_dtype, prec):
    # warm start, then four compared steps, a fresh gradient at each, the oracle on its own trajectory
    shapes = [(256, 256), (256, 688), (688, 256), (200, 336), (256, 256)]
    r = 32
    blocks, host = make_blocks(shapes, r, workers, g_dtype, si.stream_key(601, workers))
    precision = tsr.TSR_PREC_SPLIT if prec == "split" else tsr.TSR_PREC_BF16
    plan = tsr.Plan(blocks, n_workers=workers, precision=precision)
    assert plan.tsr_plan_kernel_path() == (1 if prec == "bf16" else 0)
    tol = TOL_F32 if prec == "split" else TOL_BF16
    plan_trajectory(plan, blocks, range(len(shapes)), range(WARM + 1, WARM + 5), tol,
                    "batched-%s-w%d-%s" % (prec, workers, str(g_dtype)[6:]),
                    wd=0.01, workers=workers, next_grads=fresh_gradients(blocks, host), warm_steps=WARM,
                    bar_d=BAR_D[prec], bar_move=BAR_MOVE[prec], bar_move_own=BAR_MOVE_OWN[prec])
    core, dense = plan.payload_bytes(4)
    assert core == len(shapes) * r * r * 4 and dense == 4 * sum(m * n for m, n in shapes)
    plan.close()


@pytest.mark.parametrize("prec", ["split", "bf16"])
def test_step_batched_cold_start(tsr, prec):
    # Algorithm 1's start (zero moments, t = 1, 2, 3): at t = 1 D is the sign of the core entry, so
    # the step is checked kernel by kernel on the GPU's own core; at t = 2, 3 against the oracle
    # with the bar a cold start needs: the moments of an entry rest on two or three draws, so D
    # still divides by the smallest of them (measured on these small blocks: split 2.3e-4, bf16
    # 1.0e-1; model-sized blocks measure 2e-2, see test_gpu_fullsize.py)
    shapes = [(256, 688), (688, 256), (200, 336)]
    r = 32
    g_dtype = torch.float32 if prec == "split" else torch.bfloat16
    blocks, host = make_blocks(shapes, r, 1, g_dtype, si.stream_key(605))
    plan = tsr.Plan(blocks, precision=tsr.TSR_PREC_SPLIT if prec == "split" else tsr.TSR_PREC_BF16)
    tol = TOL_F32 if prec == "split" else TOL_BF16
    plan_trajectory(plan, blocks, range(len(shapes)), (1, 2, 3), tol, "cold-start-%s" % prec, wd=0.0,
                    next_grads=fresh_gradients(blocks, host), bar_d=COLD_BAR[prec], bar_move=COLD_BAR[prec],
                    bar_move_own=BAR_MOVE_OWN[prec], w_tol=10 * tol)
    plan.close()


@pytest.mark.parametrize("r", [64, 128, 256, 512])       # 512: beyond the fused lift kernel, on the NT GEMM pair
@pytest.mark.parametrize("workers", [1, 2])
@pytest.mark.parametrize("rows16", [True, False, "padded"])
def test_bf16_plan_fused_lift_ranks(tsr, r, workers, rows16):
    # ragged shapes (partial row panels, partial column tiles) with weight decay.  With gradient
    # rows that are multiples of 16 bytes the plan runs the k-contiguous bf16 kernels and, at
    # these ranks, the fused lift kernel; with odd row lengths it must fall back to the general
    # kernels and still meet the same bar -- unless the caller pads the row pitch to 8 elements
    # ("padded": odd n, NaN in the padding), which is all the bf16 kernels need.
    if rows16 is True:
        shapes = [(r + 37, 2 * r + 64), (3 * r + 5, r), (r, r), (2 * r, 5 * r + 136), (r + 1, 2 * r + 8)]
    else:
        shapes = [(r + 37, 2 * r + 61), (3 * r + 5, r), (r, r), (2 * r, 5 * r + 130), (r + 1, 2 * r + 4)]
    blocks, host = make_blocks(shapes, r, workers, torch.bfloat16, si.stream_key(631, r), guard_w=True,
                               pad_g=(rows16 == "padded"))
    plan = tsr.Plan(blocks, n_workers=workers, precision=tsr.TSR_PREC_BF16)
    assert plan.tsr_plan_kernel_path() == (1 if rows16 else 0)

    def guards(i, t):
        assert guards_intact(host[i]["W_full"], *blocks[i]["W"].shape)    # nothing written outside the m x n block
    plan_trajectory(plan, blocks, range(len(shapes)), range(WARM + 1, WARM + 4), TOL_BF16,
                    "lift-ranks-r%d-w%d-%s" % (r, workers, rows16),
                    wd=0.05, workers=workers, next_grads=fresh_gradients(blocks, host), warm_steps=WARM,
                    bar_d=BAR_D["bf16"], bar_move=BAR_MOVE["bf16"], bar_move_own=BAR_MOVE_OWN["bf16"], after_block=guards)
    plan.close()


@pytest.mark.parametrize("guard", [True, False])
def test_bf16_plan_rank512_weight_update_edges(tsr, guard):
    # Rank 512: the weight update runs on the wave-specialised kernel, which moves W in 16-byte row
    # pieces.  Column counts that are not multiples of four make the last piece of a row start at
    # column n - 4 and overlap its neighbour (5461 is the width of the 1B workload; 517 leaves a last
    # tile of five columns, 1085 one of 61); rows of W are then not 16-byte aligned either, and with
    # guard = False they follow each other without a gap, so a piece that ran over the end of a row
    # would corrupt the next one.  Partial row tiles as well (549 and 1541 rows).
    r = 512
    shapes = [(549, 1085), (1541, 517), (512, 512), (640, 5461)]
    blocks, host = make_blocks(shapes, r, 1, torch.bfloat16, si.stream_key(633), guard_w=guard, pad_g=True)
    plan = tsr.Plan(blocks, n_workers=1, precision=tsr.TSR_PREC_BF16)
    assert plan.tsr_plan_kernel_path() == 1

    def guards(i, t):
        if guard:
            assert guards_intact(host[i]["W_full"], *blocks[i]["W"].shape)
    plan_trajectory(plan, blocks, range(len(shapes)), range(WARM + 1, WARM + 4), TOL_BF16, "rank512-edges-guard%d" % guard,
                    wd=0.05, next_grads=fresh_gradients(blocks, host), warm_steps=WARM,
                    bar_d=BAR_D["bf16"], bar_move=BAR_MOVE["bf16"], bar_move_own=BAR_MOVE_OWN["bf16"], after_block=guards)
    plan.close()


@pytest.mark.parametrize("r", [64, 96, 256])
def test_bf16_plan_adam_in_core_epilogue(tsr, r, monkeypatch):
    # With one worker and cores that U^T P writes whole (no k split), Adam runs in the epilogue
    # of that GEMM.  A model-sized batch gets there by itself; these few ragged blocks are kept
    # from splitting k by the tile-count knob.  r = 96 takes the unfused lift (row-major D^T).
    monkeypatch.setenv("TSR_TUNE_UTP_TILES", "1")
    shapes = [(r + 37, 2 * r + 64), (3 * r + 5, r), (r, r), (2 * r, 5 * r + 136)]
    blocks, host = make_blocks(shapes, r, 1, torch.bfloat16, si.stream_key(641, r), guard_w=True)
    plan = tsr.Plan(blocks, n_workers=1, precision=tsr.TSR_PREC_BF16)
    assert plan.tsr_plan_kernel_path() == 1

    def guards(i, t):
        assert guards_intact(host[i]["W_full"], *blocks[i]["W"].shape)
    plan_trajectory(plan, blocks, range(len(shapes)), range(WARM + 1, WARM + 5), TOL_BF16, "adam-epilogue-r%d" % r,
                    wd=0.05, next_grads=fresh_gradients(blocks, host), warm_steps=WARM,
                    bar_d=BAR_D["bf16"], bar_move=BAR_MOVE["bf16"], bar_move_own=BAR_MOVE_OWN["bf16"], after_block=guards)
    plan.close()


def test_bf16_plan_follows_changed_bases(tsr):
    # the bf16 plan keeps bf16 copies of the bases: after the caller rewrites U, V and says
    # so, the next step must use the new ones
    shapes = [(320, 448), (130, 264)]
    r = 64
    blocks, host = make_blocks(shapes, r, 1, torch.bfloat16, 611)
    plan = tsr.Plan(blocks, precision=tsr.TSR_PREC_BF16)
    assert plan.tsr_plan_kernel_path() == 1
    plan.tsr_step_batched(1, lr=1e-3)
    for i, (b, h, (m, n)) in enumerate(zip(blocks, host, shapes)):
        U2, V2 = bases(m, n, r, si.stream_key(612, i))
        h["U"], h["V"] = U2, V2
        b["U"].copy_(U2); b["V"].copy_(V2)
    plan.tsr_plan_bases_changed()
    plan.tsr_step_batched(2, lr=1e-3)
    torch.cuda.synchronize()
    for b, h in zip(blocks, host):
        C_ref = orc.project_core(h["G"][0], h["U"], h["V"])
        assert rel_fro(b["C"], C_ref) < TOL_BF16
    plan.close()


@pytest.mark.parametrize("prec", ["split", "bf16"])
def test_zero_learning_rate_leaves_weights_untouched(tsr, prec):
    shapes = [(256, 384), (130, 257)]
    blocks, host = make_blocks(shapes, 32, 1, torch.bfloat16, 621)
    W0 = [b["W"].clone() for b in blocks]
    plan = tsr.Plan(blocks, precision=tsr.TSR_PREC_SPLIT if prec == "split" else tsr.TSR_PREC_BF16)
    plan.tsr_step_batched(1, lr=0.0, wd=0.1)
    torch.cuda.synchronize()
    for b, w0 in zip(blocks, W0):
        assert torch.equal(b["W"], w0)
    plan.close()


def test_refresh_batched_matches_single(tsr):
    shapes = [(192, 256), (256, 192), (320, 320)]
    r, p, q = 16, 8, 1
    blocks, host = make_blocks(shapes, r, 1, torch.float32, 701, noise=1e-3)
    for b, h, (m, n) in zip(blocks, host, shapes):   # well separated spectra
        G64, _, _ = si.exact_lowrank(m, n, r, si.stream_key(702, m, n))
        h["G"] = (G64.float() + si.normal((m, n), si.stream_key(703, m), std=1e-3))[None]
        b["G"].copy_(h["G"][0])
    plan = tsr.Plan(blocks, with_refresh=True, p=p)
    omegas = [si.omega(n, r + p, si.stream_key(704, i)) for i, (m, n) in enumerate(shapes)]
    plan.tsr_refresh_batched([dev(o) for o in omegas], q)
    torch.cuda.synchronize()
    for b, h, om in zip(blocks, host, omegas):
        U_ref, V_ref, _ = orc.refresh_rsvd(h["G"][0], om, r, p, q)
        assert projector_err(b["U"], U_ref) < TOL_F32 and projector_err(b["V"], V_ref) < TOL_F32
        check_orthonormal(b["U"]); check_orthonormal(b["V"])
    plan.close()


@pytest.mark.parametrize("nt", ["1", "0"])
def test_refresh_batched_bf16_gradients(tsr, nt, monkeypatch):
    # the plan's refresh on bf16 gradients: the products with G run on the k-contiguous bf16 family
    # (transposed copy of G, small operand in two bf16 pieces) or, with the knob off or a gradient
    # that family cannot read (unaligned row pitch), on the general kernel; ragged shapes, a row
    # pitch padded with NaN, power iterations 0..2; every block against the oracle
    monkeypatch.setenv("TSR_TUNE_REFRESH_NT", nt)
    shapes = [(192, 256), (333, 200), (130, 264), (264, 131), (520, 1000), (200, 333)]
    r, p = 24, 8
    blocks, host = make_blocks(shapes, r, 1, torch.bfloat16, 721, noise=1e-3, pad_g=True)
    for i, (b, h, (m, n)) in enumerate(zip(blocks, host, shapes)):
        G64, _, _ = si.exact_lowrank(m, n, r, si.stream_key(722, i))
        h["G"] = (G64.float() + si.normal((m, n), si.stream_key(723, i), std=1e-3)).to(torch.bfloat16)[None]
        b["G"].copy_(h["G"][0])
    plan = tsr.Plan(blocks, with_refresh=True, p=p)
    omegas = [si.omega(n, r + p, si.stream_key(724, i)) for i, (m, n) in enumerate(shapes)]
    dev_om = [dev(o) for o in omegas]
    for q in (1, 0, 2):
        plan.tsr_refresh_batched(dev_om, q)
        torch.cuda.synchronize()
        for b, h, om, (m, n) in zip(blocks, host, omegas, shapes):
            U_ref, V_ref, _ = orc.refresh_rsvd(h["G"][0], om, r, p, q)
            eu, ev = projector_err(b["U"], U_ref), projector_err(b["V"], V_ref)
            parity_log("plan refresh bf16 G (nt=%s) %dx%d q=%d: projector errors U %.2e V %.2e" % (nt, m, n, q, eu, ev))
            assert eu < TOL_F32 and ev < TOL_F32, (m, n, q, eu, ev)
            check_orthonormal(b["U"]); check_orthonormal(b["V"])
    plan.close()


def test_refresh_batched_mixed_gradient_types(tsr):
    # one plan with bf16 gradients the NT family can read, a bf16 gradient it cannot (odd row pitch:
    # general kernel) and fp32 gradients (general kernel, three pieces): every block against the oracle
    shapes = [(192, 256), (256, 192), (333, 200), (200, 333), (320, 320), (130, 264)]
    dtypes = [torch.bfloat16, torch.float32, torch.bfloat16, torch.float32, torch.bfloat16, torch.bfloat16]
    r, p, q = 16, 8, 1
    blocks, host = [], []
    for i, ((m, n), dt) in enumerate(zip(shapes, dtypes)):
        b, h = make_blocks([(m, n)], r, 1, dt, si.stream_key(731, i), noise=1e-3)
        G64, _, _ = si.exact_lowrank(m, n, r, si.stream_key(732, i))
        G = (G64.float() + si.normal((m, n), si.stream_key(733, i), std=1e-3)).to(dt)
        if i == 4:
            # row pitch n + 1 elements: rows are not 16-byte aligned, the block stays on the general kernel
            Gp = torch.zeros(m, n + 1, dtype=dt, device="cuda")
            Gp[:, :n] = dev(G)
            b[0]["G"] = Gp[:, :n]
        else:
            b[0]["G"].copy_(G)
        h[0]["G"] = G[None]
        blocks += b; host += h
    plan = tsr.Plan(blocks, with_refresh=True, p=p)
    omegas = [si.omega(n, r + p, si.stream_key(734, i)) for i, (m, n) in enumerate(shapes)]
    plan.tsr_refresh_batched([dev(o) for o in omegas], q)
    torch.cuda.synchronize()
    for b, h, om, (m, n), dt in zip(blocks, host, omegas, shapes, dtypes):
        U_ref, V_ref, _ = orc.refresh_rsvd(h["G"][0], om, r, p, q)
        eu, ev = projector_err(b["U"], U_ref), projector_err(b["V"], V_ref)
        parity_log("plan refresh mixed types %dx%d %s: projector errors U %.2e V %.2e" % (m, n, str(dt)[6:], eu, ev))
        assert eu < TOL_F32 and ev < TOL_F32, (m, n, dt, eu, ev)
        check_orthonormal(b["U"]); check_orthonormal(b["V"])
    plan.close()


@pytest.mark.parametrize("groups", [1, 2, 3])
def test_refresh_batched_in_groups(tsr, groups, monkeypatch):
    # twelve blocks of mixed shapes and dtypes: the batched refresh cuts them into groups that run
    # side by side on streams of the plan; followed at once by work on the caller's stream
    # (the steps), which must see the refreshed bases.  Every grouping gives the same answer.
    monkeypatch.setenv("TSR_TUNE_REFRESH_GROUPS", str(groups))
    shapes = [(192, 256), (256, 192), (320, 320), (130, 264)] * 3
    r, p, q = 16, 8, 1
    blocks, host = make_blocks(shapes, r, 1, torch.float32, 711, noise=1e-3)
    for i, (b, h, (m, n)) in enumerate(zip(blocks, host, shapes)):
        G64, _, _ = si.exact_lowrank(m, n, r, si.stream_key(712, i))
        h["G"] = (G64.float() + si.normal((m, n), si.stream_key(713, i), std=1e-3))[None]
        b["G"].copy_(h["G"][0])
    plan = tsr.Plan(blocks, with_refresh=True, p=p)
    omegas = [si.omega(n, r + p, si.stream_key(714, i)) for i, (m, n) in enumerate(shapes)]
    dev_om = [dev(o) for o in omegas]
    for rep in range(2):                                   # twice: the side streams are reused
        plan.tsr_refresh_batched(dev_om, q)
        plan.tsr_step_batched(1 + rep, lr=0.0)             # queued behind the refresh; lr = 0 leaves W alone
    torch.cuda.synchronize()
    for b, h, om in zip(blocks, host, omegas):
        U_ref, V_ref, _ = orc.refresh_rsvd(h["G"][0], om, r, p, q)
        assert projector_err(b["U"], U_ref) < TOL_F32 and projector_err(b["V"], V_ref) < TOL_F32
        check_orthonormal(b["U"]); check_orthonormal(b["V"])
        # the step that followed projected with the refreshed bases
        assert rel_fro(b["C"], orc.project_core(h["G"][0], orc.f64(b["U"]), orc.f64(b["V"]))) < TOL_F32
    plan.close()


def test_determinism_bitwise(tsr):
    # split-k partials are reduced in a fixed order: two runs give identical bits
    m, n, r = 512, 1376, 64
    key = si.stream_key(801)
    sig = si.make_signal(m, n, r, "1/i", key)
    G = dev(si.gradient(sig, 1e-3, si.stream_key(key, 1)))
    U, V = bases(m, n, r, key)
    U, V = dev(U), dev(V)
    C1 = torch.empty(r, r, device="cuda"); C2 = torch.empty(r, r, device="cuda")
    tsr.tsr_project_core(G, U, V, C1); tsr.tsr_project_core(G, U, V, C2)
    assert torch.equal(C1, C2)


def _bf16_plan_run(tsr, steps, restart_at=None):
    """Runs `steps` plan steps of a small bf16 model; with restart_at the plan is destroyed after
    that many steps and a new one is created on the same caller-owned buffers (a checkpoint is a
    copy of those buffers: there is no other state).  Returns W, M, Vm of every block."""
    shapes = [(320, 448), (448, 320), (256, 256), (130, 264)]
    r = 64
    blocks, host = make_blocks(shapes, r, 1, torch.bfloat16, si.stream_key(901))
    put = fresh_gradients(blocks, host)
    plan = tsr.Plan(blocks, precision=tsr.TSR_PREC_BF16)
    assert plan.tsr_plan_kernel_path() == 1
    for t in range(1, steps + 1):
        put(t)
        plan.tsr_step_batched(t, lr=1e-3, wd=0.01)
        if restart_at is not None and t == restart_at:
            torch.cuda.synchronize()
            plan.close()
            saved = [{k: b[k].clone() for k in ("W", "U", "V", "M", "Vm")} for b in blocks]      # the checkpoint
            for b, sv in zip(blocks, saved):
                for k, v in sv.items():
                    b[k].zero_(); b[k].copy_(v)                                                    # restored
            plan = tsr.Plan(blocks, precision=tsr.TSR_PREC_BF16)
    torch.cuda.synchronize()
    out = [(b["W"].clone(), b["M"].clone(), b["Vm"].clone()) for b in blocks]
    plan.close()
    return out


@pytest.mark.parametrize("r", [64, 512])       # 512: the wide-tile kernels and the wave-specialised weight update
def test_step_under_graph_capture_replays_bitwise(tsr, r):
    # the batched step is kernel launches on the caller's stream and nothing else (no allocation, no
    # copy, no host synchronisation), so it can be captured into a HIP graph; three replays, with
    # eager work and synchronisations between them, must leave exactly what three eager steps leave
    # (the step count and the hyper-parameters are baked into the captured launches)
    if r == 64:
        shapes = [(320, 448), (448, 320), (256, 256), (130, 264)]
    else:
        shapes = [(640, 1085), (1541, 520), (512, 512)]
    blocks, host = make_blocks(shapes, r, 1, torch.bfloat16, si.stream_key(911, r), pad_g=True)
    plan = tsr.Plan(blocks, precision=tsr.TSR_PREC_BF16)
    assert plan.tsr_plan_kernel_path() == 1
    for t in (1, 2):                                            # warm: shadows of the bases built, kernels configured
        plan.tsr_step_batched(t, lr=1e-3, wd=0.01)
    torch.cuda.synchronize()
    keys = ("W", "M", "Vm", "C", "D")
    start = [{k: b[k].clone() for k in keys} for b in blocks]

    def restore():
        for b, sv in zip(blocks, start):
            for k in keys:
                b[k].copy_(sv[k])
    for _ in range(3):
        plan.tsr_step_batched(7, lr=1e-3, wd=0.01)
    torch.cuda.synchronize()
    eager = [{k: b[k].clone() for k in keys} for b in blocks]
    restore()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        plan.tsr_step_batched(7, lr=1e-3, wd=0.01)              # binding: launches on torch's current (capturing) stream
    restore()                                                   # (capture runs nothing; be sure of the start state anyway)
    torch.cuda.synchronize()
    scratch = torch.zeros(1024, device="cuda")
    for rep in range(3):
        graph.replay()
        scratch.add_(1.0)                                       # eager work between the replays
        torch.cuda.synchronize()
    for b, ev in zip(blocks, eager):
        for k in keys:
            assert torch.equal(b[k], ev[k]), k
    plan.close()


def test_split_run_five_plus_five_equals_ten_bitwise(tsr):
    # all optimizer state is the caller's flat buffers (W, U, V, m, v and the step count): ten steps
    # in one go and five + checkpoint / restore / new plan + five give identical bits
    a = _bf16_plan_run(tsr, 10)
    b = _bf16_plan_run(tsr, 10, restart_at=5)
    for (Wa, Ma, Va), (Wb, Mb, Vb) in zip(a, b):
        assert torch.equal(Wa, Wb) and torch.equal(Ma, Mb) and torch.equal(Va, Vb)


def test_whole_step_determinism_bitwise_bf16_plan(tsr):
    # every reduction of the bf16 plan (k-split partials, worker sums) has a fixed order: two runs
    # of the same steps give identical bits
    a = _bf16_plan_run(tsr, 3)
    b = _bf16_plan_run(tsr, 3)
    for (Wa, Ma, Va), (Wb, Mb, Vb) in zip(a, b):
        assert torch.equal(Wa, Wb) and torch.equal(Ma, Mb) and torch.equal(Va, Vb)
