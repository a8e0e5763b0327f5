"""Communication-byte and optimizer-state formulas of the paper, written out plainly.
TEST INFRASTRUCTURE ONLY (see the package docstring).

Sources: the table of synchronized objects (Table 1), the table of weight / optimizer
state sizes (Table 2), the definition of per-step communicated bytes B_t with
Bytes/Step, PeakBytes and CumulativeBytes (Section 3.2), and the description of what is
synchronized on refresh steps (end of Section 3.5).
"""
from __future__ import annotations

from typing import Iterable, List, Sequence, Tuple


def synchronized_elements(method: str, m: int, n: int, r: int) -> int:
    """Scalar entries synchronized per step for one m x n block (Table 1)."""
    if method == "adamw":
        return m * n
    if method == "lora":
        return r * m + r * n
    if method == "one-sided":
        return r * n
    if method == "tsr":
        return r * r
    raise ValueError(method)


def refresh_elements(m: int, n: int, r: int, p: int) -> int:
    """Entries synchronized on a TSR refresh step: the core plus the sketches Q (m x k)
    and B (k x n), k = r + p (Section 3.5)."""
    k = r + p
    return r * r + m * k + k * n


def state_elements(method: str, kind: str, m: int, n: int, r: int) -> int:
    """Optimizer-state entries (Table 2).  kind = 'linear' (W is m x n) or 'embedding'
    (vocabulary m, width n, r = embedding rank)."""
    if kind == "linear":
        return {"adam": 2 * m * n, "lora": 2 * m * r + 2 * n * r,
                "one-sided": m * r + 2 * n * r, "tsr": m * r + n * r + 2 * r * r}[method]
    if kind == "embedding":
        dense = m * n + 2 * m * n
        return {"adam": dense, "lora": dense, "one-sided": dense,
                "tsr": m * r + r * n + 2 * r * r}[method]
    raise ValueError(kind)


def step_bytes(elements_per_block: Iterable[int], b_dtype: int) -> int:
    """B_t = sum over blocks of b_dtype * |S_t| (Section 3.2)."""
    return b_dtype * sum(elements_per_block)


def bytes_per_step(per_step: Sequence[int]) -> float:
    return sum(per_step) / len(per_step)


def peak_bytes(per_step: Sequence[int]) -> int:
    return max(per_step)


def cumulative_bytes(per_step: Sequence[int], t: int) -> int:
    return sum(per_step[:t])


def dense_model_elements(hidden: int, inter: int, layers: int, vocab: int) -> int:
    """Matrix-shaped entries of a LLaMA-style model as the dense baseline row of the main
    results table counts them: every linear block plus ONE vocabulary-sized matrix."""
    per_layer = 4 * hidden * hidden + 3 * hidden * inter
    return layers * per_layer + vocab * hidden


def tsr_schedule_bytes(shapes: List[Tuple[int, int]], r: int, p: int, K: int, T: int, b_dtype: int = 4) -> List[int]:
    """B_t for t = 1..T for blocks `shapes` under Algorithm 1's schedule (refresh iff
    t mod K == 0)."""
    out = []
    for t in range(1, T + 1):
        if t % K == 0:
            out.append(step_bytes((refresh_elements(m, n, r, p) for m, n in shapes), b_dtype))
        else:
            out.append(step_bytes((synchronized_elements("tsr", m, n, r) for m, n in shapes), b_dtype))
    return out


def exact_svd_refresh_elements(m: int, n: int, r: int) -> int:
    """Entries synchronized on a refresh step when the refresh is an exact SVD: the dense averaged
    gradient itself (Section 3.5: an exact SVD needs the full gradient), plus the core."""
    return r * r + m * n


def schedule_bytes(shapes: List[Tuple[int, int]], r: int, p: int, K: int, T: int, method: str = "tsr",
                   refresh: str = "rsvd", b_dtype: int = 4) -> List[int]:
    """B_t for t = 1..T (refresh iff t mod K == 0) for the ablation variants: method 'tsr'
    (r x r cores) or 'one-sided' (r x n objects, Table 1); refresh 'rsvd' (sketches Q and B,
    Section 3.5) or 'exact' (dense gradient)."""
    out = []
    for t in range(1, T + 1):
        total = 0
        for m, n in shapes:
            step = synchronized_elements(method, m, n, r)
            if t % K == 0:
                k = r + p
                total += step + (m * k + k * n if refresh == "rsvd" else m * n)
            else:
                total += step
        out.append(b_dtype * total)
    return out
