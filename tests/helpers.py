"""Glue shared by the tests: workload dict -> oracle config, error norms and the closeness criteria."""
import dataclasses

import numpy as np

from oracle import ppll_oracle as O

# max |a - ref| may be this many times tol * max |ref|: for an error that is spread like noise with relative L2
# size tol, the largest of N element errors stands to the largest reference element roughly as tol itself (both
# are the same high quantile of their distributions); the factor leaves room for errors that grow with the value
# (bf16 rounding) and for references with lighter tails than the error.
MAX_ABS_FACTOR = 4.0


def oracle_cfg(wl: dict) -> O.BlockConfig:
    names = {f.name for f in dataclasses.fields(O.BlockConfig)}
    return O.BlockConfig(**{k: v for k, v in wl.items() if k in names})


def rel_l2(a, ref, floor_ref=None) -> float:
    """Per-tensor relative L2 error; absolute when the reference is ~0.  floor_ref: a companion tensor whose norm
    is a lower limit for the denominator (see assert_close)."""
    a = np.asarray(a, dtype=np.float64).reshape(-1)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1)
    nr = np.linalg.norm(ref)
    if floor_ref is not None:
        nr = max(nr, np.linalg.norm(np.asarray(floor_ref, dtype=np.float64)))
    d = np.linalg.norm(a - ref)
    return d if nr < 1e-12 else d / nr


def max_abs_ratio(a, ref, floor_ref=None) -> float:
    """Largest element error over the largest reference magnitude (absolute when the reference is ~0)."""
    a = np.asarray(a, dtype=np.float64).reshape(-1)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1)
    if a.size == 0:
        return 0.0
    d = np.abs(a - ref).max()
    m = np.abs(ref).max()
    if floor_ref is not None:
        m = max(m, np.abs(np.asarray(floor_ref, dtype=np.float64)).max())
    return d if m < 1e-12 else d / m


def worst_row_rel_l2(a, ref, row_len: int) -> float:
    """Largest relative L2 error of a row (a token's features, a pixel's channels).  A row is measured against
    its own norm, or against the root-mean-square row norm of the tensor where its own is smaller (rows that a
    ReLU has emptied, or nearly, have no scale of their own)."""
    a = np.asarray(a, dtype=np.float64).reshape(-1, row_len)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1, row_len)
    nr = np.linalg.norm(ref, axis=1)
    floor = np.sqrt(np.mean(nr ** 2))
    if floor < 1e-12:
        return float(np.linalg.norm(a - ref, axis=1).max())
    return float((np.linalg.norm(a - ref, axis=1) / np.maximum(nr, floor)).max())


def closeness(a, ref, row_len=None, floor_ref=None) -> dict:
    """The three distances the parity tests look at."""
    out = {"rel_l2": rel_l2(a, ref, floor_ref), "max_abs": max_abs_ratio(a, ref, floor_ref)}
    if row_len:
        out["row"] = worst_row_rel_l2(a, ref, row_len)
    return out


def assert_close(a, ref, tol, what, row_len=None, row_tol=None, max_tol=None, floor_ref=None) -> dict:
    """A tensor passes when (i) its relative L2 error is within tol, (ii) no single element is off by more than
    max_tol (default MAX_ABS_FACTOR * tol) times the largest reference magnitude, and (iii), when row_len is
    given, every row is within row_tol (default tol) in relative L2.  (ii) and (iii) are what a norm over a whole
    tensor cannot see: one wrong row among thousands, one wrong bias element.
    floor_ref: a companion reference tensor of the same kind (the scale gradient of a BatchNorm for its shift
    gradient) whose norm and largest magnitude are lower limits for the denominators of (i) and (ii): a
    reference that is a cancelling sum of the companion's own terms has no scale of its own."""
    a = np.asarray(a)
    ref = np.asarray(ref)
    assert a.size == ref.size, (what, "size", a.shape, ref.shape)
    assert np.all(np.isfinite(np.asarray(a, dtype=np.float64))), (what, "non-finite values")
    c = closeness(a, ref, row_len, floor_ref)
    assert c["rel_l2"] <= tol, (what, "relative L2", c["rel_l2"], "tolerance", tol)
    mt = max_tol if max_tol is not None else MAX_ABS_FACTOR * tol
    assert c["max_abs"] <= mt, (what, "largest element error / largest reference magnitude", c["max_abs"], "tolerance", mt)
    if row_len:
        rt = row_tol if row_tol is not None else tol
        assert c["row"] <= rt, (what, "worst row, relative L2", c["row"], "tolerance", rt)
    return c
