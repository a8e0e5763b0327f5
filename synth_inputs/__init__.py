"""Seeded synthetic inputs for the TSR-Adam hot path (shared by tests, bench and smoke).

This module holds NO arithmetic of the method itself: it only manufactures the
operands (gradients, weights, sketch matrices, token ids) that both the HIP
library and the CPU oracle consume.  Every array is produced once and the very
same array is handed to both sides, so no generator parity between the two
implementations is ever needed.

Random numbers come from a counter-based generator written here (a 64-bit
mixing function applied to ``key + index``), evaluated with wrapping int64
tensor arithmetic, so the same code runs on the CPU and on the GPU and the
value of element ``i`` of a stream does not depend on how many elements are
drawn.

The shapes are the LLaMA shapes the paper trains (appendix table of model
hyper-parameters; the 1B hidden size printed there is garbled and is read as
2048).  The gradients stand in for the paper's C4 pre-training gradients, which
need a dataset and a training stack that are not available: a low-rank signal
with a decaying spectrum plus white noise.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Sequence, Tuple

import numpy as np
import torch

BASE_SEED = 20260208

_MASK64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB


def _to_i64(x: int) -> int:
    """Reinterpret an unsigned 64-bit integer as a signed one."""
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


def mix64_int(x: int) -> int:
    """Reference (pure Python, arbitrary precision) 64-bit finaliser."""
    x &= _MASK64
    x = ((x ^ (x >> 30)) * _M1) & _MASK64
    x = ((x ^ (x >> 27)) * _M2) & _MASK64
    return x ^ (x >> 31)


def stream_key(seed: int, *ids: int) -> int:
    """Fold a seed and a tuple of small integers (config, matrix, worker, step,
    role ...) into one 64-bit stream key."""
    k = mix64_int(seed)
    for v in ids:
        k = mix64_int((k + _GOLDEN * (int(v) + 1)) & _MASK64)
    return k


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of an int64 tensor."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix64(x: torch.Tensor) -> torch.Tensor:
    x = (x ^ _lsr(x, 30)) * _to_i64(_M1)
    x = (x ^ _lsr(x, 27)) * _to_i64(_M2)
    return x ^ _lsr(x, 31)


def raw_bits(count: int, key: int, device="cpu", offset: int = 0) -> torch.Tensor:
    """64 pseudo-random bits for counters offset .. offset+count-1 (int64 tensor)."""
    idx = torch.arange(offset, offset + count, dtype=torch.int64, device=device)
    return _mix64(idx * _to_i64(_GOLDEN) + _to_i64(key))


def uniform01(count: int, key: int, device="cpu", offset: int = 0) -> torch.Tensor:
    """float64 uniforms strictly inside (0, 1)."""
    h = raw_bits(count, key, device, offset)
    return (_lsr(h, 11).to(torch.float64) + 0.5) * (1.0 / (1 << 53))


def normal(shape: Sequence[int], key: int, std: float = 1.0, device="cpu",
           dtype=torch.float32) -> torch.Tensor:
    """iid N(0, std^2) by Box-Muller on two 32-bit halves of one 64-bit draw."""
    count = int(np.prod(shape)) if len(shape) else 1
    out = torch.empty(count, dtype=dtype, device=device)
    chunk = 1 << 24
    for o in range(0, count, chunk):
        c = min(chunk, count - o)
        h = raw_bits(c, key, device, o)
        u1 = (_lsr(h, 32).to(torch.float64) + 0.5) * (1.0 / (1 << 32))
        u2 = ((h & 0xFFFFFFFF).to(torch.float64) + 0.5) * (1.0 / (1 << 32))
        z = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)
        out[o:o + c] = (z * std).to(dtype)
    return out.reshape(tuple(shape))


def orthonormal(rows: int, cols: int, key: int) -> torch.Tensor:
    """rows x cols matrix with orthonormal columns (float64, CPU): the Q factor
    of a seeded Gaussian matrix.  Input manufacture only."""
    g = normal((rows, cols), key, dtype=torch.float64).numpy()
    q, _ = np.linalg.qr(g)
    return torch.from_numpy(np.ascontiguousarray(q))


def spectrum(rank: int, kind: str) -> torch.Tensor:
    i = torch.arange(1, rank + 1, dtype=torch.float64)
    if kind == "1/i":
        return 1.0 / i
    if kind == "1/sqrt(i)":
        return 1.0 / torch.sqrt(i)
    if kind == "flat":
        return torch.ones(rank, dtype=torch.float64)
    raise ValueError(kind)


@dataclass
class Signal:
    """Fixed low-rank part A diag(s) B^T of a gradient stream."""
    A: torch.Tensor  # m x rank, fp32 on `device`
    sB: torch.Tensor  # n x rank, fp32 on `device`, columns of B scaled by s

    def dense(self) -> torch.Tensor:
        return self.A @ self.sB.T


def make_signal(m: int, n: int, rank: int, kind: str, key: int, device="cpu") -> Signal:
    A = orthonormal(m, rank, stream_key(key, 1))
    B = orthonormal(n, rank, stream_key(key, 2))
    s = spectrum(rank, kind)
    return Signal(A.to(torch.float32).to(device), (B * s[None, :]).to(torch.float32).to(device))


def gradient(sig: Signal, noise_std: float, key: int, dtype=torch.float32) -> torch.Tensor:
    """G = A diag(s) B^T + noise_std * Z with Z iid N(0,1) drawn from stream `key`.
    For bf16 the fp32 sum is rounded once, to nearest even; that rounded array is
    the input of both implementations."""
    m, n = sig.A.shape[0], sig.sB.shape[0]
    g = sig.dense()
    if noise_std != 0.0:
        g += normal((m, n), key, std=noise_std, device=g.device, dtype=torch.float32)
    return g.to(dtype).contiguous()


def exact_lowrank(m: int, n: int, rank: int, key: int) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """float64 matrix of exact rank `rank` with well separated singular values
    (from 2 down to 1) together with its orthonormal factors, for closed-form checks."""
    A = orthonormal(m, rank, stream_key(key, 1))
    B = orthonormal(n, rank, stream_key(key, 2))
    s = torch.linspace(2.0, 1.0, rank, dtype=torch.float64)
    return (A * s[None, :]) @ B.T, A, B


def weights(m: int, n: int, key: int, std: float = 0.02, device="cpu") -> torch.Tensor:
    return normal((m, n), key, std=std, device=device, dtype=torch.float32)


def omega(n: int, k: int, key: int, device="cpu") -> torch.Tensor:
    """Gaussian test matrix of the range sketch, n x k, N(0,1), fp32."""
    return normal((n, k), key, std=1.0, device=device, dtype=torch.float32)


def zipf_ids(count: int, vocab: int, s: float, key: int) -> torch.Tensor:
    """`count` token ids in [0, vocab) with P(id = j) proportional to (j+1)^-s,
    by inverse CDF on the seeded uniforms (CPU int64)."""
    w = np.arange(1, vocab + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    u = uniform01(count, key).numpy()
    ids = np.searchsorted(cdf, u, side="left")
    return torch.from_numpy(np.minimum(ids, vocab - 1).astype(np.int64))


def embedding_gradient(vocab: int, d: int, ids: torch.Tensor, key: int, std: float = 1e-2,
                       device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """Row-sparse embedding gradient: rows listed in `ids` (multiplicity ignored)
    are iid N(0, std^2), every other row is exactly zero.  Returns (G, sorted
    distinct row ids)."""
    rows = torch.unique(ids)
    g = torch.zeros((vocab, d), dtype=torch.float32, device=device)
    vals = normal((rows.numel(), d), key, std=std, device=device, dtype=torch.float32)
    g[rows.to(device)] = vals
    return g, rows


# --------------------------------------------------------------------------
# Model shapes (vocabulary 32000 for all)
# --------------------------------------------------------------------------
LLAMA = {
    "60m": dict(hidden=512, inter=1376, layers=8),
    "130m": dict(hidden=768, inter=2048, layers=12),
    "350m": dict(hidden=1024, inter=2736, layers=24),
    "1b": dict(hidden=2048, inter=5461, layers=24),
}
VOCAB = 32000


def layer_shapes(model: str) -> List[Tuple[int, int]]:
    """(m, n) of the seven matrix blocks of one transformer layer: four
    attention projections, gate, up, down."""
    c = LLAMA[model]
    h, f = c["hidden"], c["inter"]
    return [(h, h)] * 4 + [(h, f)] * 2 + [(f, h)]


def model_shapes(model: str, layers: int | None = None) -> List[Tuple[int, int]]:
    n_layers = LLAMA[model]["layers"] if layers is None else layers
    return layer_shapes(model) * n_layers


@dataclass
class Workload:
    name: str
    shapes: List[Tuple[int, int]]
    r: int
    p: int
    q: int
    g_dtype: torch.dtype
    signal_rank: int
    spectrum: str
    noise: float
    workers: int = 1


def workload(name: str, layers: int | None = None) -> Workload:
    """The synthetic workloads, one per benchmark configuration."""
    if name == "single-60m":
        return Workload(name, [(512, 1376)], 64, 8, 1, torch.float32, 64, "1/i", 1e-3)
    if name == "llama-130m":
        return Workload(name, model_shapes("130m", layers), 256, 8, 1, torch.bfloat16, 256, "1/i", 1e-3)
    if name == "llama-1b":
        return Workload(name, model_shapes("1b", layers), 512, 16, 2, torch.bfloat16, 512, "1/sqrt(i)", 1e-3)
    if name == "llama-350m-dp8":
        return Workload(name, model_shapes("350m", layers), 256, 8, 1, torch.bfloat16, 256, "1/i", 1e-3, workers=8)
    if name == "lm-head":
        return Workload(name, [(VOCAB, 2048)], 128, 8, 1, torch.float32, 256, "1/i", 1e-3)
    raise ValueError(name)
