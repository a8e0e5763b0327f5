"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests re-types an oracle formula or re-calls an oracle routine as its own
reference: the expected values are closed forms, invariants, brute force, numpy's LAPACK
routines on tiny inputs, or numbers printed in the paper.
"""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import tsr_oracle as orc

RNG = np.random.default_rng(1234)


def orthonormal(rows, cols, key):
    return si.orthonormal(rows, cols, key).numpy()


def rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


# ------------------------------------------------------------------ products
@pytest.mark.parametrize("M,N,K", [(3, 5, 7), (8, 2, 11), (1, 1, 1), (13, 17, 4)])
def test_matmul_variants_match_numpy(M, N, K):
    A = RNG.standard_normal((M, K)); B = RNG.standard_normal((K, N))
    assert np.allclose(orc.matmul(A, B), A @ B, rtol=0, atol=1e-13)
    At = np.ascontiguousarray(A.T); Bt = np.ascontiguousarray(B.T)
    assert np.allclose(orc.matmul(At, B, ta=True), A @ B, rtol=0, atol=1e-13)
    assert np.allclose(orc.matmul(A, Bt, tb=True), A @ B, rtol=0, atol=1e-13)


def test_matmul_by_hand():
    A = np.array([[1., 2.], [3., 4.], [5., 6.]])
    B = np.array([[1., 0., -1.], [2., 1., 0.]])
    expect = np.array([[5., 2., -1.], [11., 4., -3.], [17., 6., -5.]])
    assert np.array_equal(orc.matmul(A, B), expect)


# ------------------------------------------------------------------ project / lift
@pytest.mark.parametrize("m,n,r", [(24, 40, 5), (40, 24, 7), (9, 9, 9)])
def test_project_of_lift_is_identity(m, n, r):
    # U^T (U C0 V^T) V = C0 for orthonormal U, V
    U = orthonormal(m, r, 11); V = orthonormal(n, r, 12)
    C0 = RNG.standard_normal((r, r))
    G = U @ C0 @ V.T
    assert rel(orc.project_core(G, U, V), C0) < 1e-13


def test_project_matches_definition_elementwise():
    # C[a,b] = sum_ij U[i,a] G[i,j] V[j,b], brute force with Python loops
    m, n, r = 6, 5, 3
    G = RNG.standard_normal((m, n)); U = RNG.standard_normal((m, r)); V = RNG.standard_normal((n, r))
    C = np.zeros((r, r))
    for a in range(r):
        for b in range(r):
            for i in range(m):
                for j in range(n):
                    C[a, b] += U[i, a] * G[i, j] * V[j, b]
    assert np.allclose(orc.project_core(G, U, V), C, rtol=0, atol=1e-13)


def test_project_idempotent_and_linear():
    m, n, r, K = 30, 22, 6, 5
    U = orthonormal(m, r, 21); V = orthonormal(n, r, 22)
    Gs = [RNG.standard_normal((m, n)) for _ in range(K)]
    C = orc.project_core(Gs[0], U, V)
    again = orc.project_core(U @ C @ V.T, U, V)
    assert rel(again, C) < 1e-13
    mean_of_cores = orc.core_average([orc.project_core(G, U, V) for G in Gs])
    core_of_mean = orc.project_core(sum(Gs) / K, U, V)
    assert rel(mean_of_cores, core_of_mean) < 1e-13


def test_core_average_is_arithmetic_mean():
    cores = [np.full((3, 3), float(i)) for i in (1, 2, 6)]
    assert np.allclose(orc.core_average(cores), np.full((3, 3), 3.0))
    one = RNG.standard_normal((4, 4))
    assert np.array_equal(orc.core_average([one]), one)


# ------------------------------------------------------------------ Adam on the core
def test_adam_first_step_closed_form():
    # m0 = v0 = 0  =>  D = g / (|g| + eps) elementwise; values around eps make the
    # placement of eps (outside the root, after bias correction) matter
    g = np.array([[1.0, -2.5, 3e-8], [-1e-8, 0.0, 7e-9], [1e-3, -4e-12, 5.0]])
    M = np.zeros_like(g); Vm = np.zeros_like(g)
    D = orc.adam_core(g, M, Vm, t=1, beta1=0.9, beta2=0.999, eps=1e-8)
    assert np.allclose(D, g / (np.abs(g) + 1e-8), rtol=1e-12, atol=0)
    assert np.allclose(M, 0.1 * g, rtol=1e-12) and np.allclose(Vm, 0.001 * g * g, rtol=1e-9)


def test_adam_constant_core_every_step():
    # constant core g: m_t = (1-b1^t) g, v_t = (1-b2^t) g^2, so D_t = g/(|g|+eps) for all t
    g = RNG.standard_normal((5, 5)) * np.logspace(-9, 1, 25).reshape(5, 5)
    M = np.zeros_like(g); Vm = np.zeros_like(g)
    for t in range(1, 40):
        D = orc.adam_core(g, M, Vm, t=t, beta1=0.9, beta2=0.999, eps=1e-8)
        assert np.allclose(D, g / (np.abs(g) + 1e-8), rtol=1e-10, atol=0), t
        assert np.allclose(M, (1 - 0.9 ** t) * g, rtol=1e-10)
        assert np.allclose(Vm, (1 - 0.999 ** t) * g * g, rtol=1e-9)


def test_adam_two_steps_by_hand():
    # scalar case worked by hand: g1 = 1, g2 = -1, b1 = 0.5, b2 = 0.5, eps = 0
    M = np.zeros((1, 1)); Vm = np.zeros((1, 1))
    D1 = orc.adam_core(np.array([[1.0]]), M, Vm, t=1, beta1=0.5, beta2=0.5, eps=0.0)
    assert D1[0, 0] == pytest.approx(1.0)
    D2 = orc.adam_core(np.array([[-1.0]]), M, Vm, t=2, beta1=0.5, beta2=0.5, eps=0.0)
    # m2 = .5*.5 - .5 = -.25 ; v2 = .5*.5 + .5 = .75 ; mhat = -.25/.75 ; vhat = .75/.75 = 1
    assert M[0, 0] == pytest.approx(-0.25) and Vm[0, 0] == pytest.approx(0.75)
    assert D2[0, 0] == pytest.approx(-1.0 / 3.0)


def dense_adamw(W, grads, lr, wd, b1, b2, eps):
    """Dense AdamW exactly as the background section writes it (moment recursions, bias
    correction, decoupled decay)."""
    m = np.zeros_like(W); v = np.zeros_like(W)
    for t, g in enumerate(grads, start=1):
        m = b1 * m + (1 - b1) * g
        v = b2 * v + (1 - b2) * g * g
        W = W - lr * ((m / (1 - b1 ** t)) / (np.sqrt(v / (1 - b2 ** t)) + eps) + wd * W)
    return W


def test_identity_bases_reduce_to_dense_adamw():
    n = 7
    I = np.eye(n)
    W = RNG.standard_normal((n, n)); grads = [RNG.standard_normal((n, n)) for _ in range(6)]
    expect = dense_adamw(W.copy(), grads, 1e-2, 0.1, 0.9, 0.999, 1e-8)
    M = np.zeros((n, n)); Vm = np.zeros((n, n)); Wo = W.copy()
    for t, g in enumerate(grads, start=1):
        orc.tsr_adam_step(Wo, [g], I, I, M, Vm, t, lr=1e-2, wd=0.1)
    assert rel(Wo, expect) < 1e-13


# ------------------------------------------------------------------ lift + apply
def test_first_step_weight_closed_form():
    m, n, r = 20, 31, 4
    U = orthonormal(m, r, 31); V = orthonormal(n, r, 32)
    G = RNG.standard_normal((m, n)); W0 = RNG.standard_normal((m, n)) * 0.02
    g = U.T @ G @ V
    expect = W0 - 1e-3 * U @ (g / (np.abs(g) + 1e-8)) @ V.T
    W = W0.copy(); M = np.zeros((r, r)); Vm = np.zeros((r, r))
    orc.tsr_adam_step(W, [G], U, V, M, Vm, 1, lr=1e-3)
    assert rel(W, expect) < 1e-13


def test_constant_gradient_T_steps_closed_form():
    m, n, r, T = 12, 9, 3, 25
    U = orthonormal(m, r, 41); V = orthonormal(n, r, 42)
    G = RNG.standard_normal((m, n)); W0 = RNG.standard_normal((m, n))
    g = U.T @ G @ V
    expect = W0 - T * 1e-3 * U @ (g / (np.abs(g) + 1e-8)) @ V.T
    W = W0.copy(); M = np.zeros((r, r)); Vm = np.zeros((r, r))
    for t in range(1, T + 1):
        orc.tsr_adam_step(W, [G], U, V, M, Vm, t, lr=1e-3)
    assert rel(W, expect) < 1e-12


def test_weight_decay_only():
    # zero gradient => D = 0 => W_T = (1 - lr*wd)^T W0
    m, n, r, T = 8, 10, 2, 7
    U = orthonormal(m, r, 51); V = orthonormal(n, r, 52)
    W0 = RNG.standard_normal((m, n)); W = W0.copy()
    M = np.zeros((r, r)); Vm = np.zeros((r, r))
    for t in range(1, T + 1):
        orc.tsr_adam_step(W, [np.zeros((m, n))], U, V, M, Vm, t, lr=0.1, wd=0.3)
    assert rel(W, (1 - 0.03) ** T * W0) < 1e-13


def test_apply_uses_pre_update_weights_and_scale():
    m, n, r = 6, 4, 2
    U = RNG.standard_normal((m, r)); V = RNG.standard_normal((n, r)); D = RNG.standard_normal((r, r))
    W0 = RNG.standard_normal((m, n))
    expect = W0 - 0.5 * (0.75 * (U @ D @ V.T) + 0.2 * W0)
    W = orc.backproject_apply(W0.copy(), U, V, D, lr=0.5, wd=0.2, scale=0.75)
    assert rel(W, expect) < 1e-14


def test_sign_flips_of_bases_leave_weights_unchanged():
    m, n, r, T = 16, 12, 4, 5
    U = orthonormal(m, r, 61); V = orthonormal(n, r, 62)
    su = np.array([1, -1, -1, 1.0]); sv = np.array([-1, 1, -1, 1.0])
    grads = [RNG.standard_normal((m, n)) for _ in range(T)]
    W0 = RNG.standard_normal((m, n))
    outs = []
    for (Uu, Vv) in ((U, V), (U * su, V * sv)):
        W = W0.copy(); M = np.zeros((r, r)); Vm = np.zeros((r, r))
        for t, g in enumerate(grads, start=1):
            orc.tsr_adam_step(W, [g], Uu, Vv, M, Vm, t, lr=1e-2)
        outs.append(W)
    assert rel(outs[1], outs[0]) < 1e-13


def test_sgd_core_recursion():
    # Algorithm 2: m_t = (1-beta) sum_s beta^(t-s) C_s ; D = m
    cores = [RNG.standard_normal((3, 3)) for _ in range(5)]
    M = np.zeros((3, 3))
    for t, c in enumerate(cores, start=1):
        D = orc.sgd_core(c, M, beta=0.8)
        expect = sum(0.2 * 0.8 ** (t - s) * cores[s - 1] for s in range(1, t + 1))
        assert np.allclose(D, expect, rtol=1e-12, atol=1e-15)
        assert np.array_equal(D, M)


# ------------------------------------------------------------------ thin QR
@pytest.mark.parametrize("rows,k", [(30, 30), (50, 7), (9, 1), (64, 20)])
def test_householder_qr_invariants(rows, k):
    Y = RNG.standard_normal((rows, k))
    Q, R = orc.householder_qr(Y)
    assert np.abs(Q.T @ Q - np.eye(k)).max() < 1e-12
    assert rel(Q @ (Q.T @ Y), Y) < 1e-12
    assert rel(Q @ R, Y) < 1e-12
    assert np.abs(np.tril(R, -1)).max() == 0.0
    # against LAPACK: R is unique up to row signs
    Rl = np.linalg.qr(Y)[1]
    assert np.allclose(np.abs(R), np.abs(Rl), rtol=1e-9, atol=1e-12)


def test_householder_qr_rank_deficient_still_orthonormal():
    rows, k, rank = 40, 10, 4
    Y = RNG.standard_normal((rows, rank)) @ RNG.standard_normal((rank, k))
    Y[:, 3] = 0.0
    Q, _ = orc.householder_qr(Y)
    assert np.abs(Q.T @ Q - np.eye(k)).max() < 1e-12
    assert rel(Q @ (Q.T @ Y), Y) < 1e-12
    Qz, _ = orc.householder_qr(np.zeros((12, 5)))
    assert np.abs(Qz.T @ Qz - np.eye(5)).max() < 1e-12


# ------------------------------------------------------------------ small SVD
@pytest.mark.parametrize("k,n", [(5, 5), (6, 19), (1, 8), (12, 40)])
def test_jacobi_svd_against_lapack_and_invariants(k, n):
    B = RNG.standard_normal((k, n))
    Ut, S, Vt, sweeps = orc.jacobi_svd(B)
    assert sweeps < 30
    assert rel(Ut @ np.diag(S) @ Vt.T, B) < 1e-13
    assert np.abs(Ut.T @ Ut - np.eye(k)).max() < 1e-13
    assert np.abs(Vt.T @ Vt - np.eye(k)).max() < 1e-13
    assert np.all(np.diff(S) <= 0)
    assert np.allclose(S, np.linalg.svd(B, compute_uv=False), rtol=1e-12, atol=1e-14)


def test_jacobi_svd_known_singular_values():
    k, n = 4, 9
    X = orthonormal(k, k, 71); Z = orthonormal(n, k, 72)
    s = np.array([3.0, 2.0, 0.5, 0.0])
    Ut, S, Vt, _ = orc.jacobi_svd(X @ np.diag(s) @ Z.T)
    assert np.allclose(S, s, atol=1e-14)
    for j in range(3):  # singular vectors up to sign
        assert abs(abs(Ut[:, j] @ X[:, j]) - 1) < 1e-12
        assert abs(abs(Vt[:, j] @ Z[:, j]) - 1) < 1e-12


def test_full_svd_both_orientations():
    for shape in ((7, 11), (11, 7)):
        G = RNG.standard_normal(shape)
        U, S, V = orc.full_svd(G)
        assert rel(U @ np.diag(S) @ V.T, G) < 1e-13
        assert np.allclose(S, np.linalg.svd(G, compute_uv=False), rtol=1e-12)


# ------------------------------------------------------------------ rSVD refresh
def projector(X):
    return X @ X.T


@pytest.mark.parametrize("m,n,r,p,q", [(60, 45, 6, 4, 1), (45, 60, 6, 4, 0), (80, 80, 10, 5, 2)])
def test_rsvd_recovers_exact_rank_r_subspace(m, n, r, p, q):
    G, A, B = si.exact_lowrank(m, n, r, 81)
    G, A, B = G.numpy(), A.numpy(), B.numpy()
    Om = si.omega(n, r + p, 82).numpy()
    U, V, S = orc.refresh_rsvd(G, Om, r, p, q)
    assert np.linalg.norm(projector(U) - projector(A)) < 1e-10
    assert np.linalg.norm(projector(V) - projector(B)) < 1e-10
    assert np.abs(U.T @ U - np.eye(r)).max() < 1e-12
    assert np.abs(V.T @ V - np.eye(r)).max() < 1e-12
    assert np.allclose(S[:r], np.linspace(2.0, 1.0, r), rtol=1e-11)
    assert np.abs(S[r:]).max() < 1e-12


@pytest.mark.parametrize("m,n,r,q", [(12, 20, 4, 0), (12, 20, 4, 1), (20, 12, 5, 2)])
def test_rsvd_with_full_sketch_is_truncated_svd(m, n, r, q):
    # k = min(m, n): range(Q) is everything, so the refresh is the exact truncated SVD
    G = RNG.standard_normal((m, n))
    k = min(m, n)
    Om = si.omega(n, k, 91).numpy()
    U, V, S = orc.refresh_rsvd(G, Om, r, k - r, q)
    Ub, Sb, Vb = orc.full_svd(G)                     # brute force: Jacobi on G itself
    Ul, Sl, Vlt = np.linalg.svd(G, full_matrices=False)  # LAPACK
    assert np.allclose(S, Sl, rtol=1e-11)
    assert np.allclose(Sb, Sl, rtol=1e-11)
    for ref_u, ref_v in ((Ub[:, :r], Vb[:, :r]), (Ul[:, :r], Vlt.T[:, :r])):
        assert np.linalg.norm(projector(U) - projector(ref_u)) < 1e-9
        assert np.linalg.norm(projector(V) - projector(ref_v)) < 1e-9
    # U S V^T is the best rank-r approximation: its error is the tail of the spectrum
    err = np.linalg.norm(G - U @ np.diag(S[:r]) @ V.T)
    assert err == pytest.approx(np.sqrt((Sl[r:] ** 2).sum()), rel=1e-9)


def test_rsvd_power_iterations_do_not_change_full_rank_capture_but_help_decay():
    # slowly decaying spectrum: more power iterations can only tighten the captured energy
    m, n, r, p = 70, 90, 8, 4
    X = orthonormal(m, 40, 101); Z = orthonormal(n, 40, 102)
    s = 1.0 / np.sqrt(np.arange(1, 41))
    G = X @ np.diag(s) @ Z.T
    Om = si.omega(n, r + p, 103).numpy()
    best = np.sqrt((s[r:] ** 2).sum())
    errs = []
    for q in (0, 1, 3):
        U, V, S = orc.refresh_rsvd(G, Om, r, p, q)
        errs.append(np.linalg.norm(G - U @ (U.T @ G @ V) @ V.T))
        assert errs[-1] >= best * (1 - 1e-9)
    assert errs[2] <= errs[1] <= errs[0]
    assert errs[2] < 1.05 * best


def test_rsvd_independent_of_orth_basis():
    # post-multiplying Q by a rotation (another valid output of orth) leaves U U^T and
    # V V^T unchanged: composed here from the oracle's pieces with q = 0
    m, n, r, p = 40, 33, 5, 3
    k = r + p
    G = RNG.standard_normal((m, n)); Om = si.omega(n, k, 111).numpy()
    U0, V0, _ = orc.refresh_rsvd(G, Om, r, p, 0)
    Q, _ = orc.householder_qr(G @ Om)
    Rot = orthonormal(k, k, 112)
    Q2 = Q @ Rot
    Ut, S, Vt, _ = orc.jacobi_svd(Q2.T @ G)
    U1 = Q2 @ Ut[:, :r]; V1 = Vt[:, :r]
    assert np.linalg.norm(projector(U1) - projector(U0)) < 1e-9
    assert np.linalg.norm(projector(V1) - projector(V0)) < 1e-9


def test_rsvd_unchanged_by_triangular_rescaling_inside_the_power_iteration():
    # The oracle takes orth at every normalisation of the power iteration (Section 3.5).  What
    # the refresh returns does not depend on how well the INTERMEDIATE bases are normalised:
    # replacing orth(X) by X T^-1 for any upper-triangular T (which is what a single Cholesky
    # pass of a thin QR delivers) keeps every span, and keeps the positively oriented Q factor of
    # the final sketch.  Composed here from the oracle's QR and SVD with q = 2 against the
    # oracle's own refresh.
    m, n, r, p, q = 36, 29, 5, 3, 2
    k = r + p
    G = RNG.standard_normal((m, n)); Om = si.omega(n, k, 131).numpy()
    U0, V0, S0, Q0 = orc.refresh_rsvd(G, Om, r, p, q, return_q=True)

    def loose(X, seed):          # X T^-1 with a fixed, far from orthonormalising, triangular T
        T = np.triu(np.random.default_rng(seed).uniform(0.5, 2.0, (k, k)))
        return X @ np.linalg.inv(T)

    Y = loose(G @ Om, 1)
    for it in range(q):
        Z = loose(G.T @ Y, 10 + it)
        Y = G @ Z
        if it + 1 < q:
            Y = loose(Y, 20 + it)
    Q, R = orc.householder_qr(Y)
    sgn = np.sign(np.diag(R)); sgn[sgn == 0] = 1.0
    Q = Q * sgn                                   # orientation diag(R) > 0
    # same span, and the same basis up to the sign convention of the oracle's own QR
    assert np.linalg.norm(projector(Q) - projector(Q0)) < 1e-9
    assert np.abs(np.abs(Q0.T @ Q) - np.eye(k)).max() < 1e-8
    Ut, S, Vt, _ = orc.jacobi_svd(Q.T @ G)
    assert np.allclose(S, S0, rtol=1e-9)
    assert np.linalg.norm(projector(Q @ Ut[:, :r]) - projector(U0)) < 1e-8
    assert np.linalg.norm(projector(Vt[:, :r]) - projector(V0)) < 1e-8


def test_rsvd_rejects_oversized_sketch():
    G = RNG.standard_normal((10, 8))
    with pytest.raises(ValueError):
        orc.refresh_rsvd(G, np.zeros((8, 9)), 6, 3, 1)


def test_rsvd_returns_final_q():
    m, n, r, p = 30, 26, 4, 3
    G = RNG.standard_normal((m, n)); Om = si.omega(n, r + p, 121).numpy()
    U, V, S, Q = orc.refresh_rsvd(G, Om, r, p, 1, return_q=True)
    assert np.abs(Q.T @ Q - np.eye(r + p)).max() < 1e-12
    # U lies in range(Q); S are the singular values of Q^T G
    assert rel(Q @ (Q.T @ U), U) < 1e-12
    assert np.allclose(S, np.linalg.svd(Q.T @ G, compute_uv=False), rtol=1e-11)


# ------------------------------------------------------------------ multi-worker refresh (Algorithm 1, N > 1)
def _sign_fix(U, V):
    s = np.sign(V[np.abs(V).argmax(axis=0), np.arange(V.shape[1])])
    return U * s, V * s


def test_workers_refresh_single_worker_is_the_plain_refresh():
    m, n, r, p, q = 40, 30, 4, 3, 1
    G64, _, _ = si.exact_lowrank(m, n, r, 901)
    G = orc.f64(G64) + 1e-3 * orc.f64(si.normal((m, n), 902, dtype=torch.float64))
    Om = si.omega(n, r + p, 903)
    U1, V1, S1 = orc.refresh_rsvd(G, Om, r, p, q)
    U2, V2, S2, Qbar, Bbar = orc.refresh_rsvd_workers([G], Om, r, p, q)
    assert np.allclose(S1, S2, atol=1e-12)
    U1, V1 = _sign_fix(U1, V1); U2, V2 = _sign_fix(U2, V2)
    assert np.allclose(U1, U2, atol=1e-10) and np.allclose(V1, V2, atol=1e-10)
    assert np.allclose(Qbar.T @ Qbar, np.eye(r + p), atol=1e-12)


def test_workers_refresh_identical_workers_change_nothing():
    # averaging N copies of the same sketches is the identity: the result equals one worker's
    m, n, r, p, q = 36, 44, 5, 2, 1
    G64, _, _ = si.exact_lowrank(m, n, r, 911)
    G = orc.f64(G64) + 1e-3 * orc.f64(si.normal((m, n), 912, dtype=torch.float64))
    Om = si.omega(n, r + p, 913)
    U1, V1, S1, _, _ = orc.refresh_rsvd_workers([G], Om, r, p, q)
    U3, V3, S3, _, _ = orc.refresh_rsvd_workers([G, G.copy(), G.copy()], Om, r, p, q)
    assert np.allclose(S1, S3, atol=1e-12)
    U1, V1 = _sign_fix(U1, V1); U3, V3 = _sign_fix(U3, V3)
    assert np.allclose(U1, U3, atol=1e-10) and np.allclose(V1, V3, atol=1e-10)


def test_workers_refresh_structure_of_the_averaged_sketches():
    # what the definition fixes for N > 1, checked without power iterations (q = 0), where each
    # worker's basis is the thin QR factor of G_i Omega: numpy's QR, oriented to diag(R) > 0,
    # gives the same unique factor.  Bbar and Qbar are the plain means of the workers' sketches,
    # sigma are Bbar's singular values, V is orthonormal, U Sigma_r V^T is Qbar times the best
    # rank-r approximation of Bbar, and Qbar^T Qbar <= I (a mean of orthonormal bases contracts).
    m, n, r, p, q, N = 48, 40, 4, 4, 0, 3
    G64, _, _ = si.exact_lowrank(m, n, r, 921)
    Gs = [orc.f64(G64) + 5e-2 * orc.f64(si.normal((m, n), 922 + w, dtype=torch.float64)) for w in range(N)]
    Om = si.omega(n, r + p, 929)
    U, V, S, Qbar, Bbar = orc.refresh_rsvd_workers(Gs, Om, r, p, q)
    Qi = []
    for G in Gs:
        Qn, Rn = np.linalg.qr(G @ orc.f64(Om))
        Qi.append(Qn * np.sign(np.diag(Rn)))
    assert np.allclose(Qbar, sum(Qi) / N, atol=1e-10)
    assert np.allclose(Bbar, sum(Q.T @ G for Q, G in zip(Qi, Gs)) / N, atol=1e-10)
    assert np.allclose(S, np.linalg.svd(Bbar, compute_uv=False), atol=1e-10)
    assert np.allclose(V.T @ V, np.eye(r), atol=1e-10)
    Ub, Sb, Vbt = np.linalg.svd(Bbar, full_matrices=False)
    lifted = Qbar @ (Ub[:, :r] * Sb[:r]) @ Vbt[:r]
    assert np.allclose((U * S[:r]) @ V.T, lifted, atol=1e-9)
    gram = Qbar.T @ Qbar
    assert np.linalg.eigvalsh(gram).max() <= 1.0 + 1e-12
    assert np.linalg.norm(U.T @ U - np.eye(r)) > 1e-6          # the workers differ: U is not orthonormal


def test_workers_refresh_nearby_workers_keep_the_mean_basis_nearly_orthonormal():
    # gradients that differ by a small perturbation have nearby sketches; with every worker's
    # basis oriented the same way their mean stays within O(perturbation) of orthonormal.  A
    # sign convention that flipped columns from worker to worker would cancel whole directions
    # (defect of order one).
    m, n, r, p, q, N = 60, 50, 6, 0, 1, 4
    G64, _, _ = si.exact_lowrank(m, n, r, 931)
    Gs = [orc.f64(G64) + 1e-6 * orc.f64(si.normal((m, n), 932 + w, dtype=torch.float64)) for w in range(N)]
    Om = si.omega(n, r + p, 939)
    U, V, S, Qbar, Bbar = orc.refresh_rsvd_workers(Gs, Om, r, p, q)
    assert np.abs(Qbar.T @ Qbar - np.eye(r)).max() < 1e-4
    assert np.abs(U.T @ U - np.eye(r)).max() < 1e-4
    assert np.allclose(S, np.linspace(2.0, 1.0, r), atol=1e-4)


# ------------------------------------------------------------------ moment re-alignment (Appendix B)
def test_realign_moment_is_the_doubly_projected_lifted_moment():
    # the defining equation of the assumption, with the projectors formed explicitly by numpy
    m, n, r = 30, 24, 5
    Uo, Vo = orthonormal(m, r, 941), orthonormal(n, r, 942)
    Un, Vn = orthonormal(m, r, 943), orthonormal(n, r, 944)
    M = RNG.standard_normal((r, r))
    M2 = orc.realign_moment(M, Uo, Vo, Un, Vn)
    lifted_old = Uo @ M @ Vo.T
    assert np.allclose(Un @ M2 @ Vn.T, (Un @ Un.T) @ lifted_old @ (Vn @ Vn.T), atol=1e-12)


def test_realign_moment_unchanged_bases_and_rotated_bases():
    m, n, r = 28, 33, 6
    U, V = orthonormal(m, r, 951), orthonormal(n, r, 952)
    M = RNG.standard_normal((r, r))
    assert np.allclose(orc.realign_moment(M, U, V, U, V), M, atol=1e-12)
    # same subspaces, rotated coordinates: the lifted moment does not move at all
    Ru, _ = np.linalg.qr(RNG.standard_normal((r, r))); Rv, _ = np.linalg.qr(RNG.standard_normal((r, r)))
    U2, V2 = U @ Ru, V @ Rv
    M2 = orc.realign_moment(M, U, V, U2, V2)
    assert np.allclose(M2, Ru.T @ M @ Rv, atol=1e-12)
    assert np.allclose(U2 @ M2 @ V2.T, U @ M @ V.T, atol=1e-12)


def test_realign_moment_orthogonal_subspace_loses_everything():
    m, n, r = 20, 20, 4
    Q = orthonormal(m, 2 * r, 961)
    U_old, U_new = Q[:, :r].copy(), Q[:, r:].copy()          # orthogonal column spaces
    V = orthonormal(n, r, 962)
    M = RNG.standard_normal((r, r))
    assert np.abs(orc.realign_moment(M, U_old, V, U_new, V)).max() < 1e-13


# ------------------------------------------------------------------ comparison paths (ablations)
def test_one_sided_projection_and_lift_brute_force_and_identity_basis():
    m, n, r = 9, 13, 4
    G = RNG.standard_normal((m, n)); U = orthonormal(m, r, 4101)
    C1 = orc.project_one_sided(G, U)
    expect = np.zeros((r, n))
    for a in range(r):
        for j in range(n):
            expect[a, j] = sum(U[i, a] * G[i, j] for i in range(m))
    assert np.allclose(C1, expect, rtol=0, atol=1e-13)
    # followed by a right projection it is the two-sided core: (U^T G) V = U^T G V
    V = orthonormal(n, r, 4103)
    assert np.allclose(C1 @ V, orc.project_core(G, U, V), rtol=0, atol=1e-13)
    W0 = RNG.standard_normal((m, n)); D1 = RNG.standard_normal((r, n))
    W = orc.backproject_one_sided(W0.copy(), U, D1, 0.1, 0.01, 0.5)
    assert np.allclose(W, W0 - 0.1 * (0.5 * U @ D1 + 0.01 * W0), rtol=0, atol=1e-13)
    # a one-sided update that happens to lie in a right subspace, D1 = D V^T, is the two-sided lift
    D = RNG.standard_normal((r, r))
    assert np.allclose(orc.backproject_one_sided(W0.copy(), U, D @ V.T, 0.1, 0.01, 0.5),
                       orc.backproject_apply(W0.copy(), U, V, D, 0.1, 0.01, 0.5), rtol=0, atol=1e-13)


def test_one_sided_first_step_closed_form():
    # zero moments, t = 1: D1 = c / (|c| + eps) element-wise on the r x n object
    m, n, r = 12, 7, 3
    G = RNG.standard_normal((m, n)); U = orthonormal(m, r, 4102)
    W0 = RNG.standard_normal((m, n)); M1 = np.zeros((r, n)); V1 = np.zeros((r, n))
    W = W0.copy()
    C1, D1 = orc.one_sided_adam_step(W, [G], U, M1, V1, 1, lr=0.01)
    c = U.T @ G
    assert np.allclose(D1, c / (np.abs(c) + 1e-8), rtol=1e-12, atol=0)
    assert np.allclose(W, W0 - 0.01 * U @ (c / (np.abs(c) + 1e-8)), rtol=0, atol=1e-13)
    # with U square orthogonal (r = m) and Adam's sign-like first step, U D1 is not sign(G): the
    # projection matters; with U = I it is the dense first AdamW step
    W = W0.copy()
    orc.one_sided_adam_step(W, [G], np.eye(m), np.zeros((m, n)), np.zeros((m, n)), 1, lr=0.01)
    assert np.allclose(W, W0 - 0.01 * G / (np.abs(G) + 1e-8), rtol=0, atol=1e-13)


@pytest.mark.parametrize("m,n,r", [(12, 20, 4), (20, 12, 5), (9, 9, 9)])
def test_exact_svd_refresh_against_lapack_and_full_sketch(m, n, r):
    G = RNG.standard_normal((m, n))
    U, V, S = orc.refresh_exact_svd(G, r)
    u, s, vt = np.linalg.svd(G, full_matrices=False)
    assert np.allclose(S, s, rtol=1e-11, atol=1e-13)
    assert rel(U @ U.T, u[:, :r] @ u[:, :r].T) < 1e-10 and rel(V @ V.T, vt[:r].T @ vt[:r]) < 1e-10
    # best rank-r approximation (Eckart-Young): the residual is the tail of the spectrum
    resid = np.linalg.norm(G - (U * S[:r]) @ V.T)
    assert resid == pytest.approx(np.sqrt((s[r:] ** 2).sum()), rel=1e-10, abs=1e-12)
    # the randomized refresh with a full-width sketch is this same subspace
    k = min(m, n)
    if r < k:
        Om = RNG.standard_normal((n, k))
        Ur, Vr, _ = orc.refresh_rsvd(G, Om, r, k - r, 1)
        assert rel(Ur @ Ur.T, U @ U.T) < 1e-9 and rel(Vr @ Vr.T, V @ V.T) < 1e-9
