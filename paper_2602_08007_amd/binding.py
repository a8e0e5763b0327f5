"""ctypes binding of include/tsr.h.  Argument marshalling only.

Functions keep the C names.  Tensors are torch CUDA tensors (PyTorch supplies device
memory and the stream, nothing else); sizes and leading dimensions are taken from them.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import torch

__all__ = [
    "TSR_F32", "TSR_BF16", "TSR_PREC_SPLIT", "TSR_PREC_BF16", "TsrError", "lib", "lib_path",
    "tsr_status_string", "tsr_device_count",
    "tsr_stream_scale", "tsr_project_workspace_bytes", "tsr_project_core", "tsr_project_core_static",
    "TSR_PROJECT_STATIC_SCRATCH_BYTES", "tsr_core_average", "tsr_adam_core", "tsr_sgd_core",
    "tsr_backproject_workspace_bytes", "tsr_backproject_apply",
    "tsr_refresh_workspace_bytes", "tsr_refresh_rsvd", "tsr_refresh_workers_workspace_bytes", "tsr_refresh_rsvd_workers",
    "tsr_realign_workspace_bytes", "tsr_realign_moment",
    "tsr_one_sided_workspace_bytes", "tsr_project_one_sided", "tsr_backproject_one_sided",
    "tsr_refresh_exact_workspace_bytes", "tsr_refresh_exact_svd",
    "tsr_matrix_desc", "tsr_hyper", "Plan", "workspace",
]

TSR_F32, TSR_BF16 = 0, 1
TSR_PREC_SPLIT, TSR_PREC_BF16 = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
lib_path = os.path.join(_HERE, "libtsr.so")
if not os.path.exists(lib_path):
    # nothing built yet: compile the library in-tree (hipcc, gfx950); there is no other code path
    import importlib.util as _ilu
    _spec = _ilu.spec_from_file_location("_tsr_lib_build", os.path.join(_HERE, "build.py"))
    _mod = _ilu.module_from_spec(_spec)
    try:
        _spec.loader.exec_module(_mod)
        _mod.build()
    except Exception as e:  # noqa: BLE001
        raise ImportError(
            "libtsr.so is not built and building it failed (%s): run `python -c 'import __graft_entry__ as g; g.build()'`; "
            "there is no fallback path" % e)
lib = ctypes.CDLL(lib_path)

_vp, _i, _ll, _f, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_longlong, ctypes.c_float, ctypes.c_size_t


class tsr_matrix_desc(ctypes.Structure):
    _fields_ = [("G", _vp), ("g_dtype", _i), ("m", _i), ("n", _i), ("r", _i), ("ldg", _ll), ("g_stride", _ll),
                ("W", _vp), ("ldw", _ll), ("U", _vp), ("V", _vp), ("M", _vp), ("Vm", _vp), ("C", _vp), ("D", _vp)]


class tsr_hyper(ctypes.Structure):
    _fields_ = [("lr", _f), ("wd", _f), ("beta1", _f), ("beta2", _f), ("eps", _f), ("scale", _f)]


def _sig(name, restype, *argtypes):
    fn = getattr(lib, name)
    fn.restype = restype
    fn.argtypes = list(argtypes)
    return fn


_status_string = _sig("tsr_status_string", ctypes.c_char_p, _i)
_last_hip = _sig("tsr_last_hip_error", _i)
_device_count = _sig("tsr_device_count", _i)
_project_ws = _sig("tsr_project_workspace_bytes", _sz, _i, _i, _i)
_project = _sig("tsr_project_core", _i, _vp, _i, _i, _i, _ll, _vp, _vp, _i, _f, _i, _vp, _i, _vp, _sz, _vp)
_project_static = _sig("tsr_project_core_static", _i, _vp, _i, _i, _i, _ll, _vp, _vp, _i, _f, _i, _vp, _i, _vp)
_average = _sig("tsr_core_average", _i, _vp, _i, _i, _vp, _vp)
_stream_scale = _sig("tsr_stream_scale", _i, _vp, _vp, _ll, _f, _vp)
_adam = _sig("tsr_adam_core", _i, _vp, _vp, _vp, _vp, _ll, _i, _f, _f, _f, _vp)
_sgd = _sig("tsr_sgd_core", _i, _vp, _vp, _vp, _ll, _f, _vp)
_lift_ws = _sig("tsr_backproject_workspace_bytes", _sz, _i, _i, _i)
_lift = _sig("tsr_backproject_apply", _i, _vp, _i, _i, _ll, _vp, _vp, _vp, _i, _f, _f, _f, _i, _vp, _sz, _vp)
_refresh_ws = _sig("tsr_refresh_workspace_bytes", _sz, _i, _i, _i, _i)
_refresh = _sig("tsr_refresh_rsvd", _i, _vp, _i, _i, _i, _ll, _vp, _i, _i, _i, _vp, _vp, _vp, _vp, _sz, _vp)
_realign_ws = _sig("tsr_realign_workspace_bytes", _sz, _i, _i, _i)
_realign = _sig("tsr_realign_moment", _i, _vp, _vp, _vp, _vp, _i, _i, _i, _vp, _vp, _sz, _vp)
_one_sided_ws = _sig("tsr_one_sided_workspace_bytes", _sz, _i, _i, _i)
_project_one = _sig("tsr_project_one_sided", _i, _vp, _i, _i, _i, _ll, _vp, _i, _f, _i, _vp, _i, _vp, _sz, _vp)
_lift_one = _sig("tsr_backproject_one_sided", _i, _vp, _i, _i, _ll, _vp, _vp, _i, _f, _f, _f, _i, _vp, _sz, _vp)
_exact_ws = _sig("tsr_refresh_exact_workspace_bytes", _sz, _i, _i, _i)
_exact = _sig("tsr_refresh_exact_svd", _i, _vp, _i, _i, _i, _ll, _i, _vp, _vp, _vp, _vp, _sz, _vp)
_refresh_workers_ws = _sig("tsr_refresh_workers_workspace_bytes", _sz, _i, _i, _i, _i, _i)
_refresh_workers = _sig("tsr_refresh_rsvd_workers", _i, _vp, _i, _i, _i, _ll, _ll, _i, _vp, _i, _i, _i, _vp, _vp, _vp, _vp,
                        _sz, _vp)
_plan_ws = _sig("tsr_plan_workspace_bytes", _sz, ctypes.POINTER(tsr_matrix_desc), _i, _i, _i, _i, _i)
_bases_changed = _sig("tsr_plan_bases_changed", _i, _vp)
_kernel_path = _sig("tsr_plan_kernel_path", _i, _vp)
_plan_create = _sig("tsr_plan_create", _i, ctypes.POINTER(tsr_matrix_desc), _i, _i, _i, _i, _i, _vp, _sz, _vp,
                    ctypes.POINTER(_vp))
_plan_destroy = _sig("tsr_plan_destroy", None, _vp)
_step_batched = _sig("tsr_step_batched", _i, _vp, _i, ctypes.POINTER(tsr_hyper), _vp)
_refresh_batched = _sig("tsr_refresh_batched", _i, _vp, ctypes.POINTER(_vp), _i, _vp)
_prof_begin = _sig("tsr_plan_profile_begin", _i, _vp)
_prof_end = _sig("tsr_plan_profile_end", _i, _vp, _vp, ctypes.POINTER(_f), ctypes.POINTER(_i))
_payload = _sig("tsr_plan_payload_bytes", None, _vp, _i, ctypes.POINTER(_ll), ctypes.POINTER(_ll))


class TsrError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        msg = _status_string(status).decode()
        if status == -5:
            msg += " (hipError %d)" % _last_hip()
        super().__init__("tsr: %s" % msg)


def _check(status: int) -> None:
    if status != 0:
        raise TsrError(status)


def tsr_status_string(status: int) -> str:
    return _status_string(status).decode()


def tsr_device_count() -> int:
    return int(_device_count())


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _gdtype(G: torch.Tensor) -> int:
    if G.dtype == torch.float32:
        return TSR_F32
    if G.dtype == torch.bfloat16:
        return TSR_BF16
    raise TypeError("G must be float32 or bfloat16")


def _f32c(*ts):
    for t in ts:
        if t is not None and (t.dtype != torch.float32 or not t.is_contiguous()):
            raise TypeError("expected contiguous float32 tensors")


def _ld(t: torch.Tensor) -> int:
    if t.dim() != 2 or t.stride(1) != 1:
        raise TypeError("expected a row-major 2-D tensor (unit column stride)")
    return t.stride(0)


def workspace(nbytes: int, device="cuda") -> torch.Tensor:
    """A 256-byte aligned device buffer of at least nbytes (torch allocations are 512-byte aligned)."""
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def _temp_workspace(nbytes: int, device, stream) -> torch.Tensor:
    """Workspace for a one-shot call that did not bring its own.  It is dropped when the call
    returns, while the kernels may still be queued: that is safe on torch's current stream (the
    caching allocator reuses the block in stream order) and is made safe on any other stream by
    telling the allocator which stream uses the block."""
    ws = workspace(nbytes, device)
    if stream is not None and isinstance(stream, torch.cuda.Stream) and stream != torch.cuda.current_stream(ws.device):
        ws.record_stream(stream)
    elif stream is not None and not isinstance(stream, torch.cuda.Stream):
        raise ValueError("pass a torch.cuda.Stream, or an explicit ws together with a raw stream handle")
    return ws


def tsr_project_workspace_bytes(m: int, n: int, r: int) -> int:
    return int(_project_ws(m, n, r))


def tsr_project_core(G, U, V, C, alpha=1.0, accumulate=False, precision=TSR_PREC_SPLIT, ws=None, stream=None):
    m, n = G.shape
    r = U.shape[1]
    _f32c(U, V, C)
    if ws is None:
        ws = _temp_workspace(tsr_project_workspace_bytes(m, n, r), G.device, stream)
    _check(_project(_ptr(G), _gdtype(G), m, n, _ld(G), _ptr(U), _ptr(V), r, alpha, int(bool(accumulate)), _ptr(C),
                    precision, _ptr(ws), ws.numel(), _stream(stream)))
    return C


TSR_PROJECT_STATIC_SCRATCH_BYTES = 16 << 20


def tsr_project_core_static(G, U, V, C, alpha=1.0, accumulate=False, precision=TSR_PREC_SPLIT, stream=None):
    """tsr_project_core on the library's built-in scratch: nothing is allocated, here or there."""
    m, n = G.shape
    r = U.shape[1]
    _f32c(U, V, C)
    _check(_project_static(_ptr(G), _gdtype(G), m, n, _ld(G), _ptr(U), _ptr(V), r, alpha, int(bool(accumulate)), _ptr(C),
                           precision, _stream(stream)))
    return C


def tsr_core_average(Cs, Cbar, stream=None):
    _f32c(Cs, Cbar)
    K, r = Cs.shape[0], Cs.shape[1]
    _check(_average(_ptr(Cs), K, r, _ptr(Cbar), _stream(stream)))
    return Cbar


def tsr_stream_scale(dst, src, scale=1.0, stream=None):
    _f32c(dst, src)
    _check(_stream_scale(_ptr(dst), _ptr(src), src.numel(), scale, _stream(stream)))
    return dst


def tsr_adam_core(C, M, Vm, D, t, beta1=0.9, beta2=0.999, eps=1e-8, stream=None):
    _f32c(C, M, Vm, D)
    _check(_adam(_ptr(C), _ptr(M), _ptr(Vm), _ptr(D), C.numel(), t, beta1, beta2, eps, _stream(stream)))
    return D


def tsr_sgd_core(C, M, D, beta=0.9, stream=None):
    _f32c(C, M, D)
    _check(_sgd(_ptr(C), _ptr(M), _ptr(D), C.numel(), beta, _stream(stream)))
    return D


def tsr_backproject_workspace_bytes(m: int, n: int, r: int) -> int:
    return int(_lift_ws(m, n, r))


def tsr_backproject_apply(W, U, V, D, lr, wd=0.0, scale=1.0, precision=TSR_PREC_SPLIT, ws=None, stream=None):
    m, n = W.shape
    r = U.shape[1]
    _f32c(U, V, D)
    if W.dtype != torch.float32:
        raise TypeError("W must be float32")
    if ws is None:
        ws = _temp_workspace(tsr_backproject_workspace_bytes(m, n, r), W.device, stream)
    _check(_lift(_ptr(W), m, n, _ld(W), _ptr(U), _ptr(V), _ptr(D), r, lr, wd, scale, precision, _ptr(ws), ws.numel(),
                 _stream(stream)))
    return W


def tsr_refresh_workspace_bytes(m: int, n: int, r: int, p: int) -> int:
    return int(_refresh_ws(m, n, r, p))


def tsr_refresh_rsvd(G, Omega, r, p, q, U, V, sigma=None, ws=None, stream=None):
    m, n = G.shape
    _f32c(Omega, U, V, sigma)
    if tuple(Omega.shape) != (n, r + p):
        raise ValueError("Omega must be n x (r+p)")
    if ws is None:
        ws = _temp_workspace(tsr_refresh_workspace_bytes(m, n, r, p), G.device, stream)
    _check(_refresh(_ptr(G), _gdtype(G), m, n, _ld(G), _ptr(Omega), r, p, q, _ptr(U), _ptr(V), _ptr(sigma), _ptr(ws),
                    ws.numel(), _stream(stream)))
    return U, V


def tsr_refresh_workers_workspace_bytes(m: int, n: int, r: int, p: int, n_workers: int) -> int:
    return int(_refresh_workers_ws(m, n, r, p, n_workers))


def tsr_refresh_rsvd_workers(G, Omega, r, p, q, U, V, sigma=None, ws=None, stream=None):
    """G: the workers' gradients stacked as [workers, m, n] (contiguous)."""
    if G.dim() != 3 or not G.is_contiguous():
        raise ValueError("G must be a contiguous [workers, m, n] tensor")
    K, m, n = G.shape
    _f32c(Omega, U, V, sigma)
    if tuple(Omega.shape) != (n, r + p):
        raise ValueError("Omega must be n x (r+p)")
    if ws is None:
        ws = _temp_workspace(tsr_refresh_workers_workspace_bytes(m, n, r, p, K), G.device, stream)
    _check(_refresh_workers(_ptr(G), _gdtype(G), m, n, n, m * n, K, _ptr(Omega), r, p, q, _ptr(U), _ptr(V), _ptr(sigma),
                            _ptr(ws), ws.numel(), _stream(stream)))
    return U, V


def tsr_realign_workspace_bytes(m: int, n: int, r: int) -> int:
    return int(_realign_ws(m, n, r))


def tsr_realign_moment(U_old, V_old, U_new, V_new, M, ws=None, stream=None):
    m, r = U_old.shape
    n = V_old.shape[0]
    _f32c(U_old, V_old, U_new, V_new, M)
    if tuple(U_new.shape) != (m, r) or tuple(V_old.shape) != (n, r) or tuple(V_new.shape) != (n, r) or tuple(M.shape) != (r, r):
        raise ValueError("shape mismatch")
    if ws is None:
        ws = _temp_workspace(tsr_realign_workspace_bytes(m, n, r), M.device, stream)
    _check(_realign(_ptr(U_old), _ptr(V_old), _ptr(U_new), _ptr(V_new), m, n, r, _ptr(M), _ptr(ws), ws.numel(),
                    _stream(stream)))
    return M


def tsr_one_sided_workspace_bytes(m: int, n: int, r: int) -> int:
    return int(_one_sided_ws(m, n, r))


def tsr_project_one_sided(G, U, Ct, alpha=1.0, accumulate=False, precision=TSR_PREC_SPLIT, ws=None, stream=None):
    """Ct (n x r) <- alpha G^T U (+ Ct): the one-sided object U^T G, held transposed."""
    m, n = G.shape
    r = U.shape[1]
    _f32c(U, Ct)
    if tuple(Ct.shape) != (n, r):
        raise ValueError("Ct must be n x r")
    if ws is None:
        ws = _temp_workspace(tsr_one_sided_workspace_bytes(m, n, r), G.device, stream)
    _check(_project_one(_ptr(G), _gdtype(G), m, n, _ld(G), _ptr(U), r, alpha, int(bool(accumulate)), _ptr(Ct), precision,
                        _ptr(ws), ws.numel(), _stream(stream)))
    return Ct


def tsr_backproject_one_sided(W, U, Dt, lr, wd=0.0, scale=1.0, precision=TSR_PREC_SPLIT, ws=None, stream=None):
    """W <- W - lr (scale U Dt^T + wd W) with the transposed one-sided update Dt (n x r)."""
    m, n = W.shape
    r = U.shape[1]
    _f32c(U, Dt)
    if W.dtype != torch.float32 or tuple(Dt.shape) != (n, r):
        raise TypeError("W must be float32 and Dt n x r")
    if ws is None:
        ws = _temp_workspace(tsr_one_sided_workspace_bytes(m, n, r), W.device, stream)
    _check(_lift_one(_ptr(W), m, n, _ld(W), _ptr(U), _ptr(Dt), r, lr, wd, scale, precision, _ptr(ws), ws.numel(),
                     _stream(stream)))
    return W


def tsr_refresh_exact_workspace_bytes(m: int, n: int, r: int) -> int:
    return int(_exact_ws(m, n, r))


def tsr_refresh_exact_svd(G, r, U, V, sigma=None, ws=None, stream=None):
    m, n = G.shape
    _f32c(U, V, sigma)
    if ws is None:
        nbytes = tsr_refresh_exact_workspace_bytes(m, n, r)
        if nbytes == 0:
            raise TsrError(-2)
        ws = _temp_workspace(nbytes, G.device, stream)
    _check(_exact(_ptr(G), _gdtype(G), m, n, _ld(G), r, _ptr(U), _ptr(V), _ptr(sigma), _ptr(ws), ws.numel(), _stream(stream)))
    return U, V


class Plan:
    """Batched all-layers plan (tsr_plan_* / tsr_step_batched / tsr_refresh_batched).

    blocks: sequence of dicts with tensors G (n_workers stacked as [workers, m, ld] or a single
    [m, ld] matrix), W, U, V, M, Vm, C, D.  The plan's workspace is a torch buffer owned here."""

    def __init__(self, blocks: Sequence[dict], n_workers=1, precision=TSR_PREC_SPLIT, with_refresh=False, p=0,
                 stream=None):
        self._handle = _vp()
        self.count = len(blocks)
        self.n_workers = n_workers
        self._keep = list(blocks)
        arr = (tsr_matrix_desc * self.count)()
        for d, b in zip(arr, blocks):
            G, W, U = b["G"], b["W"], b["U"]
            g2 = G[0] if G.dim() == 3 else G
            if (G.dim() == 3) != (n_workers > 1) and not (G.dim() == 3 and G.shape[0] == 1):
                raise ValueError("G must be [workers, m, n] when n_workers > 1")
            m, n = W.shape
            _f32c(U, b["V"], b["M"], b["Vm"], b["C"], b["D"])
            d.G = _ptr(G); d.g_dtype = _gdtype(G); d.m = m; d.n = n; d.r = U.shape[1]
            d.ldg = _ld(g2); d.g_stride = G.stride(0) if G.dim() == 3 else 0
            d.W = _ptr(W); d.ldw = _ld(W)
            d.U = _ptr(U); d.V = _ptr(b["V"]); d.M = _ptr(b["M"]); d.Vm = _ptr(b["Vm"]); d.C = _ptr(b["C"]); d.D = _ptr(b["D"])
        self._descs = arr
        nbytes = int(_plan_ws(arr, self.count, n_workers, precision, int(with_refresh), p))
        if nbytes == 0:
            raise TsrError(-2)
        self.ws = workspace(nbytes, blocks[0]["W"].device)
        _check(_plan_create(arr, self.count, n_workers, precision, int(with_refresh), p, _ptr(self.ws), self.ws.numel(),
                            _stream(stream), ctypes.byref(self._handle)))

    def tsr_step_batched(self, t, lr, wd=0.0, beta1=0.9, beta2=0.999, eps=1e-8, scale=1.0, stream=None):
        h = tsr_hyper(lr, wd, beta1, beta2, eps, scale)
        _check(_step_batched(self._handle, t, ctypes.byref(h), _stream(stream)))

    def tsr_plan_kernel_path(self):
        return _kernel_path(self._handle)

    def tsr_plan_bases_changed(self):
        _check(_bases_changed(self._handle))

    def tsr_refresh_batched(self, omegas: List[torch.Tensor], q, stream=None):
        _f32c(*omegas)
        arr = (_vp * self.count)(*[_ptr(o) for o in omegas])
        _check(_refresh_batched(self._handle, arr, q, _stream(stream)))

    PROF_KINDS = ("gv", "utp", "adam", "ud", "tvt", "sketch_gemm", "orth_gemm", "chol", "jacobi", "basis_gemm")

    def tsr_plan_profile_begin(self):
        _check(_prof_begin(self._handle))

    def tsr_plan_profile_end(self, stream=None):
        """{kind: (milliseconds, stages)} summed since tsr_plan_profile_begin; synchronizes."""
        n = len(self.PROF_KINDS)
        ms = (_f * n)()
        cnt = (_i * n)()
        _check(_prof_end(self._handle, _stream(stream), ms, cnt))
        return {k: (float(ms[i]), int(cnt[i])) for i, k in enumerate(self.PROF_KINDS)}

    def payload_bytes(self, bytes_per_dense_element=4):
        c, d = _ll(), _ll()
        _payload(self._handle, bytes_per_dense_element, ctypes.byref(c), ctypes.byref(d))
        return int(c.value), int(d.value)

    def close(self):
        if self._handle:
            _plan_destroy(self._handle)
            self._handle = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
