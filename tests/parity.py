"""Acceptance rule shared by the parity tests (test infrastructure).

A GPU fp16 result passes when, for every output element,
|gpu - y| <= 4e-3 * S  (S = sum_k |a*w| from the oracle; S == 0 -> gpu must be
+-0), and when the per-row argmax (lowest index on ties) equals the oracle's.

The argmax of a row is compared exactly unless the row is *near-tied*: some
other column lies within what one fp16 rounding of the two candidates plus the
fp32 accumulation error can erase,

    y_top - y[n] <= ulp16(y_top) + ACC_TOL * (S_top + S[n]),

with ulp16 the spacing of binary16 numbers at |y_top| and ACC_TOL = 1e-4 (the
kernels' observed accumulation error is below 5e-5 * S; the element-wise bound
above is forty times wider).  Two such columns can round to the same binary16
value, or swap, without either side being wrong.  For a near-tied row the GPU's
argmax must still be one of the near-tied columns.  The near-tied rows are
returned, printed by the callers, and their number is bounded per call
(`max_near_tied`), so a rule that silently excused most rows would fail.
"""
from __future__ import annotations

import numpy as np

REL_TOL = 4e-3
ACC_TOL = 1e-4


def ulp16(v: np.ndarray) -> np.ndarray:
    """Spacing of IEEE binary16 numbers at magnitude |v| (subnormal spacing below 2^-14)."""
    a = np.maximum(np.abs(np.asarray(v, dtype=np.float64)), 2.0 ** -14)
    return 2.0 ** (np.floor(np.log2(a)) - 10)


def near_tied_sets(y: np.ndarray, s: np.ndarray):
    """Per row: the oracle's argmax and the boolean mask of columns it is near-tied with (itself included)."""
    rows = np.arange(y.shape[0])
    top = np.argmax(y, axis=1)
    y_top = y[rows, top][:, None]
    s_top = s[rows, top][:, None]
    slack = ulp16(y_top) + ACC_TOL * (s_top + s)
    return top, (y_top - y) <= slack


def check(gpu: np.ndarray, y: np.ndarray, s: np.ndarray, what: str = "", argmax: bool = True,
          max_near_tied: int | None = None):
    """Element-wise tolerance and the argmax rule.  max_near_tied: how many rows may be near-tied
    (default: an eighth of the rows, at least 2 -- a Gaussian row of a few thousand columns is near-tied
    with a probability of a few percent)."""
    g = np.asarray(gpu, dtype=np.float64)
    assert g.shape == y.shape, f"{what}: shape {g.shape} vs oracle {y.shape}"
    assert np.all(np.isfinite(g)), f"{what}: non-finite GPU output"
    err = np.abs(g - y)
    bound = REL_TOL * s
    bad = err > bound
    if bad.any():
        idx = np.unravel_index(np.argmax(np.where(bad, err - bound, -np.inf)), err.shape)
        raise AssertionError(
            f"{what}: {int(bad.sum())} of {bad.size} elements exceed 4e-3*S; worst at {idx}: "
            f"gpu={g[idx]!r} oracle={y[idx]!r} err={err[idx]:.3e} bound={bound[idx]:.3e}")
    worst = float(np.max(err / np.maximum(s, 1e-300)))
    info = {"worst_rel": worst, "argmax_rows_checked": 0, "near_tied_rows": []}
    if argmax and y.shape[1] > 1:
        top, tied = near_tied_sets(y, s)
        got = np.argmax(g, axis=1)
        rows = np.arange(y.shape[0])
        near = tied.sum(axis=1) > 1
        exact_bad = (~near) & (got != top)
        assert not exact_bad.any(), (
            f"{what}: argmax differs in rows {np.nonzero(exact_bad)[0][:8]} "
            f"(gpu {got[exact_bad][:8]}, oracle {top[exact_bad][:8]})")
        near_bad = near & ~tied[rows, got]
        assert not near_bad.any(), (
            f"{what}: argmax of near-tied rows {np.nonzero(near_bad)[0][:8]} is not among the tied columns "
            f"(gpu {got[near_bad][:8]}, oracle {top[near_bad][:8]})")
        limit = max(2, y.shape[0] // 8) if max_near_tied is None else max_near_tied
        info["argmax_rows_checked"] = int(y.shape[0])
        info["near_tied_rows"] = [int(r) for r in np.nonzero(near)[0]]
        assert len(info["near_tied_rows"]) <= limit, (
            f"{what}: {len(info['near_tied_rows'])} near-tied rows {info['near_tied_rows'][:8]} exceed the "
            f"limit of {limit}: the argmax rule would be excusing too much")
    return info
