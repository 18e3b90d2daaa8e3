"""Distances between two evaluations of one tensor (numpy only; shared by the parity tests and
by the oracle-only script that writes the noise-floor fixtures).

frob    ||got - want||_F / ||want||_F over the whole tensor (the tolerance the workloads state);
row     max over rows (last axis = one token row) of ||got_r - want_r|| / ||want_r||: a single
        wrong row among thousands moves the Frobenius ratio by a fraction of a per cent and
        this one to ~1;
maxabs  max |got - want| / rms(want): a single wrong element.
"""
from __future__ import annotations

import numpy as np


def frob(got: np.ndarray, want: np.ndarray) -> float:
    want = np.asarray(want, dtype=np.float64)
    return float(np.linalg.norm(np.asarray(got, dtype=np.float64) - want) / max(np.linalg.norm(want), 1e-30))


def row(got: np.ndarray, want: np.ndarray) -> float:
    want = np.asarray(want, dtype=np.float64)
    diff = np.asarray(got, dtype=np.float64) - want
    w = want.reshape(-1, want.shape[-1])
    dn = np.linalg.norm(diff.reshape(w.shape), axis=1)
    wn = np.linalg.norm(w, axis=1)
    # rows of (near) zero norm are measured against the tensor's typical row
    floor = 1e-3 * max(float(np.sqrt(np.mean(wn * wn))), 1e-30)
    return float(np.max(dn / np.maximum(wn, floor)))


def maxabs(got: np.ndarray, want: np.ndarray) -> float:
    want = np.asarray(want, dtype=np.float64)
    rms = max(float(np.sqrt(np.mean(want * want))), 1e-30)
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - want)) / rms)


def all_three(got: np.ndarray, want: np.ndarray) -> dict:
    return {"frob": frob(got, want), "row": row(got, want), "maxabs": maxabs(got, want)}


def worst_element(got: np.ndarray, want: np.ndarray, count: int = 8):
    """[(index, got, want)] of the `count` elements with the largest absolute differences (for
    failure messages)."""
    want = np.asarray(want, dtype=np.float64)
    g = np.asarray(got, dtype=np.float64)
    diff = np.abs(g - want).ravel()
    top = np.argsort(diff)[::-1][:count]
    out = []
    for t in top:
        idx = np.unravel_index(int(t), want.shape)
        out.append((tuple(int(i) for i in idx), float(g[idx]), float(want[idx])))
    return out
