"""ctypes wrapper of the plain-C fp64 oracle (tsr_oracle.c).  TEST INFRASTRUCTURE ONLY.

Every function takes and returns C-contiguous float64 numpy arrays.  Inputs given in
fp32 or bf16 are widened exactly by the caller (`f64`) before they get here.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

_lib = ctypes.CDLL(_build.build(force=False))
_dp = ctypes.POINTER(ctypes.c_double)
_i = ctypes.c_int


def _p(a):
    return None if a is None else a.ctypes.data_as(_dp)


def f64(x) -> np.ndarray:
    """Exact widening of a numpy array or torch tensor (fp32 / bf16 / fp64) to fp64."""
    if hasattr(x, "detach"):
        import torch
        x = x.detach().to("cpu").to(torch.float64).numpy()
    return np.ascontiguousarray(x, dtype=np.float64)


def num_threads() -> int:
    return int(_lib.orc_num_threads())


def set_num_threads(n: int) -> None:
    """OpenMP threads of the products from now on (timing only; results do not depend on it)."""
    _lib.orc_set_num_threads(_i(int(n)))


def matmul(A, B, ta=False, tb=False):
    """op(A) op(B) by triple loops; supports NN, TN (A^T B) and NT (A B^T)."""
    A, B = f64(A), f64(B)
    if not ta and not tb:
        M, K = A.shape; N = B.shape[1]; assert B.shape[0] == K
        C = np.empty((M, N)); _lib.orc_matmul_nn(_p(A), _p(B), _p(C), _i(M), _i(N), _i(K))
    elif ta and not tb:
        K, M = A.shape; N = B.shape[1]; assert B.shape[0] == K
        C = np.empty((M, N)); _lib.orc_matmul_tn(_p(A), _p(B), _p(C), _i(M), _i(N), _i(K))
    elif not ta and tb:
        M, K = A.shape; N = B.shape[0]; assert B.shape[1] == K
        C = np.empty((M, N)); _lib.orc_matmul_nt(_p(A), _p(B), _p(C), _i(M), _i(N), _i(K))
    else:
        raise ValueError("TT not needed")
    return C


def project_core(G, U, V):
    """C = U^T G V (Section 3.3)."""
    G, U, V = f64(G), f64(U), f64(V)
    m, n = G.shape; r = U.shape[1]
    assert U.shape == (m, r) and V.shape == (n, r)
    C = np.empty((r, r))
    rc = _lib.orc_project_core(_p(G), _p(U), _p(V), _p(C), _i(m), _i(n), _i(r))
    assert rc == 0
    return C


def core_average(cores):
    """Arithmetic mean of the workers' cores, summed in worker order (AR of Algorithm 1)."""
    Cs = np.ascontiguousarray(np.stack([f64(c) for c in cores]))
    K, r, _ = Cs.shape
    out = np.empty((r, r))
    _lib.orc_core_average(_p(Cs), _p(out), _i(K), _i(r))
    return out


def adam_core(C, M, Vm, t, beta1=0.9, beta2=0.999, eps=1e-8):
    """Adam moments + bias-corrected normalized update on the core; M, Vm in place; returns D."""
    C = f64(C)
    assert M.dtype == np.float64 and Vm.dtype == np.float64 and M.flags.c_contiguous and Vm.flags.c_contiguous
    assert t >= 1
    D = np.empty_like(C)
    _lib.orc_adam_core(_p(C), _p(M), _p(Vm), _p(D), ctypes.c_long(C.size), _i(t),
                       ctypes.c_double(beta1), ctypes.c_double(beta2), ctypes.c_double(eps))
    return D


def sgd_core(C, M, beta=0.9):
    """Momentum core update of Algorithm 2; M in place; returns D = M."""
    C = f64(C)
    assert M.dtype == np.float64 and M.flags.c_contiguous
    D = np.empty_like(C)
    _lib.orc_sgd_core(_p(C), _p(M), _p(D), ctypes.c_long(C.size), ctypes.c_double(beta))
    return D


def backproject_apply(W, U, V, D, lr, wd=0.0, scale=1.0):
    """W <- W - lr (scale U D V^T + wd W), in place on the float64 array W."""
    assert W.dtype == np.float64 and W.flags.c_contiguous
    U, V, D = f64(U), f64(V), f64(D)
    m, n = W.shape; r = U.shape[1]
    assert U.shape == (m, r) and V.shape == (n, r) and D.shape == (r, r)
    rc = _lib.orc_backproject_apply(_p(W), _p(U), _p(V), _p(D), _i(m), _i(n), _i(r),
                                    ctypes.c_double(lr), ctypes.c_double(wd), ctypes.c_double(scale))
    assert rc == 0
    return W


def householder_qr(Y):
    """Thin QR by Householder reflections; returns (Q, R), Q always orthonormal."""
    Y = f64(Y)
    rows, k = Y.shape
    assert rows >= k
    Q = np.empty((rows, k)); R = np.empty((k, k))
    rc = _lib.orc_householder_qr(_p(Y), _p(Q), _p(R), _i(rows), _i(k))
    assert rc == 0
    return Q, R


def jacobi_svd(B):
    """One-sided Jacobi SVD of a k x n matrix (k <= n): returns (Ut k x k, S k, Vt n x k, sweeps)."""
    B = f64(B)
    k, n = B.shape
    assert k <= n
    Ut = np.empty((k, k)); S = np.empty(k); Vt = np.empty((n, k))
    sweeps = _lib.orc_jacobi_svd(_p(B), _p(Ut), _p(S), _p(Vt), _i(k), _i(n))
    assert sweeps >= 0
    return Ut, S, Vt, sweeps


def full_svd(G):
    """Brute-force SVD of a small matrix by Jacobi on the matrix itself (no sketch):
    returns (U m x s, S s, V n x s), s = min(m, n)."""
    G = f64(G)
    m, n = G.shape
    if m <= n:
        Ut, S, Vt, _ = jacobi_svd(G)
        return Ut, S, Vt
    Ut, S, Vt, _ = jacobi_svd(np.ascontiguousarray(G.T))
    return Vt, S, Ut


def refresh_rsvd(G, Omega, r, p, q, return_q=False):
    """Randomized-SVD refresh of (U, V) (Section 3.5), single worker.
    Returns (U m x r, V n x r, sigma k[, Q m x k])."""
    G, Omega = f64(G), f64(Omega)
    m, n = G.shape; k = r + p
    assert Omega.shape == (n, k)
    U = np.empty((m, r)); V = np.empty((n, r)); S = np.empty(k)
    Q = np.empty((m, k)) if return_q else None
    rc = _lib.orc_refresh_rsvd(_p(G), _p(Omega), _p(U), _p(V), _p(S), _p(Q),
                               _i(m), _i(n), _i(r), _i(p), _i(q))
    if rc == -2:
        raise ValueError("need 0 < r, r + p <= min(m, n)")
    assert rc == 0
    return (U, V, S, Q) if return_q else (U, V, S)


def refresh_rsvd_workers(G_workers, Omega, r, p, q):
    """Refresh branch of Algorithm 1 with N workers (Section 3.5): every worker i runs the sketch
    chain on its own gradient with the shared Omega (Y_i = G_i Omega, Q_i = orth(Y_i), q rounds of
    Yrow = G_i^T Q_i, Qrow = orth(Yrow), Y_i = G_i Qrow, Q_i = orth(Y_i)) and forms B_i = Q_i^T G_i;
    the sketches are averaged, Bbar = AR(B_i), Qbar = AR(Q_i); Bbar = Ut S Vt^T;
    U = Qbar Ut[:, :r], V = Vt[:, :r].  U is orthonormal only when the Q_i coincide.
    orth is the thin QR factor with diag(R) > 0 (see `orth` below).
    Returns (U m x r, V n x r, sigma k, Qbar m x k, Bbar k x n)."""
    Omega = f64(Omega)
    n, k = Omega.shape
    assert k == r + p

    def orth(Y):
        # Averaging the workers' Q_i only means something if every worker orients the columns of
        # its basis the same way: orth is the unique thin QR factor, the one whose R has a
        # positive diagonal (the Householder routine leaves the signs of diag(R) arbitrary).
        Q, R = householder_qr(Y)
        s = np.where(np.diag(R) < 0.0, -1.0, 1.0)
        return Q * s

    Qs, Bs = [], []
    for G in G_workers:
        G = f64(G)
        m = G.shape[0]
        assert G.shape[1] == n and k <= min(m, n)
        Q = orth(matmul(G, Omega))
        for _ in range(q):
            Qrow = orth(matmul(G, Q, ta=True))
            Q = orth(matmul(G, Qrow))
        Qs.append(Q)
        Bs.append(matmul(Q, G, ta=True))
    N = len(Qs)
    Qbar = np.zeros_like(Qs[0]); Bbar = np.zeros_like(Bs[0])
    for Q, B in zip(Qs, Bs):
        Qbar += Q; Bbar += B
    Qbar /= N; Bbar /= N
    Ut, S, Vt, _ = jacobi_svd(Bbar)
    U = matmul(Qbar, np.ascontiguousarray(Ut[:, :r]))
    V = np.ascontiguousarray(Vt[:, :r])
    return U, V, S, Qbar, Bbar


def realign_moment(M, U_old, V_old, U_new, V_new):
    """First moment re-expressed in refreshed bases (refresh-alignment assumption of the
    convergence analysis, Appendix B): the core M' whose lifted matrix U_new M' V_new^T is the
    old lifted matrix U_old M V_old^T projected onto the new subspaces,
        M' = (U_new^T U_old) M (V_old^T V_new)."""
    A = matmul(U_new, U_old, ta=True)           # r x r
    B = matmul(V_old, V_new, ta=True)           # r x r
    return matmul(matmul(A, f64(M)), B)


def tsr_adam_step(W, G_workers, U, V, M, Vm, t, lr, wd=0.0, beta1=0.9, beta2=0.999, eps=1e-8, scale=1.0):
    """One non-refresh iteration of Algorithm 1 for one matrix block: project every
    worker's gradient, average the cores, Adam on the core, lift and apply.
    W, M, Vm are updated in place; returns (Cbar, D)."""
    cores = [project_core(G, U, V) for G in G_workers]
    Cbar = core_average(cores)
    D = adam_core(Cbar, M, Vm, t, beta1, beta2, eps)
    backproject_apply(W, U, V, D, lr, wd, scale)
    return Cbar, D


# ------------------------------------------------------------------ comparison paths of the ablations
def project_one_sided(G, U):
    """One-sided projection C1 = U^T G (r x n): the synchronized object of the one-sided row of
    the table of communication objects (Table 1), compared with the two-sided core in the
    ablation on two-sidedness (Section 4.3)."""
    return matmul(U, G, ta=True)


def backproject_one_sided(W, U, D1, lr, wd=0.0, scale=1.0):
    """W <- W - lr (scale U D1 + wd W) with the r x n one-sided update D1, in place on the fp64
    array W (the lift of the one-sided variant; pre-update W in the decay, as in Algorithm 1)."""
    dW = matmul(U, D1)
    W -= lr * (scale * dW + wd * W)
    return W


def one_sided_adam_step(W, G_workers, U, M1, V1, t, lr, wd=0.0, beta1=0.9, beta2=0.999, eps=1e-8, scale=1.0):
    """One iteration of the one-sided variant for one block: project every worker's gradient with
    U alone, average the r x n objects, Adam on them (the same element-wise lines of Algorithm 1),
    lift with U and apply.  W, M1, V1 (r x n) in place; returns (C1bar, D1)."""
    objs = [project_one_sided(G, U) for G in G_workers]
    C1 = np.zeros_like(objs[0])
    for c in objs:                      # arithmetic mean, summed in worker order (AR of Algorithm 1)
        C1 += c
    C1 /= len(objs)
    D1 = adam_core(C1, M1, V1, t, beta1, beta2, eps)
    backproject_one_sided(W, U, D1, lr, wd, scale)
    return C1, D1


def refresh_exact_svd(G, r):
    """Exact-SVD refresh (what Section 3.5 replaces by the randomized sketch, compared in the
    ablation on randomized SVD): the r leading singular triplets of the (synchronized) gradient
    itself, by Jacobi on the matrix.  Returns (U m x r, V n x r, sigma min(m, n))."""
    Uf, S, Vf = full_svd(G)
    return np.ascontiguousarray(Uf[:, :r]), np.ascontiguousarray(Vf[:, :r]), S
