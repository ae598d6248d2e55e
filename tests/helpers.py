"""Glue shared by the tests: workload dict -> oracle config, error norms."""
import dataclasses

import numpy as np

from oracle import ppll_oracle as O


def oracle_cfg(wl: dict) -> O.BlockConfig:
    names = {f.name for f in dataclasses.fields(O.BlockConfig)}
    return O.BlockConfig(**{k: v for k, v in wl.items() if k in names})


def rel_l2(a, ref) -> float:
    """Per-tensor relative L2 error; absolute when the reference is ~0."""
    a = np.asarray(a, dtype=np.float64).reshape(-1)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1)
    nr = np.linalg.norm(ref)
    d = np.linalg.norm(a - ref)
    return d if nr < 1e-12 else d / nr
