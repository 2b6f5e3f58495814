"""Shared test helpers (no method arithmetic: fixture parsing and layout conversion only)."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def golden_values(name: str) -> dict:
    out = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, val, tol = line.split()
            out[key] = (float(val), float(tol))
    return out


def compact_from_paper_orientation(w_gate_df: np.ndarray, w_down_fd: np.ndarray) -> np.ndarray:
    """W_gate in R^{d x f} and W_down in R^{f x d} (Eq. 1 orientation) -> gd[f][2][d]."""
    d, f = w_gate_df.shape
    gd = np.empty((f, 2, d), dtype=np.float16)
    for j in range(f):
        gd[j, 0, :] = w_gate_df[:, j]
        gd[j, 1, :] = w_down_fd[j, :]
    return gd
