"""Oracle-side helpers for the GPU parity tests: feed the fp64 oracle the same seeded
inputs the library got.  Imports synth/ and oracle/ only."""
from __future__ import annotations

import numpy as np

import synth
from oracle import hmi_oracle as O


def weights_of(wl: synth.Workload, layer: int):
    names = [n for n, _, _ in synth.tensor_specs(wl)]
    shared = {n: a.astype(np.float64) for (n, _, _), a in zip(synth.shared_specs(wl), synth.shared_tensors(wl, layer))}
    cache = {}

    def get(t: int):
        if t not in cache:
            cache[t] = dict(shared)
            cache[t].update({n: a.astype(np.float64) for n, a in zip(names, synth.tenant_tensors(wl, t, layer))})
        return cache[t]
    return get


def oracle_forward(wl: synth.Workload, ids, lens, requests=None, batch: int = 0) -> np.ndarray:
    """All layers of the workload over the batch, fp64, for the given requests (default all).
    Rows of other requests are NaN."""
    R = len(ids)
    todo = list(range(R)) if requests is None else sorted(set(int(r) for r in requests))
    N = int(np.sum(lens))
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    X = np.full((N, wl.d_model), np.nan)
    for r in todo:
        X[off[r]:off[r + 1]] = synth.hidden_states(wl, r, int(lens[r]), batch).astype(np.float64)
    for layer in range(wl.n_layers):
        X = O.layer_forward(wl.block, X, ids, lens, weights_of(wl, layer), wl.n_heads, wl.ln_eps,
                            requests=todo)
    return X


def rows_of(lens, requests) -> np.ndarray:
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    return np.concatenate([np.arange(off[r], off[r + 1]) for r in requests]) if len(requests) else np.zeros(0, np.int64)


def compare(y_gpu: np.ndarray, y_ref: np.ndarray, rows, dtype: str):
    """-> (max_abs, rel_fro, ok) under the target's tolerances: bf16 max-abs 2e-2 and relative
    Frobenius 1e-2; fp32 1e-4 for both."""
    a, b = y_gpu[rows], y_ref[rows]
    assert np.isfinite(a).all() and np.isfinite(b).all()
    max_abs = float(np.abs(a - b).max()) if a.size else 0.0
    rel = float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30)) if a.size else 0.0
    tol_abs, tol_rel = (2e-2, 1e-2) if dtype == "bf16" else (1e-4, 1e-4)
    return max_abs, rel, (max_abs <= tol_abs and rel <= tol_rel)


def within_storage_rounding(y_gpu: np.ndarray, y_ref: np.ndarray, rows, budget: float = 2e-2) -> bool:
    """Element by element: |error| <= budget + half a bf16 ulp of the reference value, i.e. the flat max-abs bar
    applied to the value before it is stored.  Storing y as bf16 costs up to half an ulp by itself (0.0156 where
    4 <= |y| < 8), which the flat 2e-2 bar leaves only 0.0044 above.  Used next to the flat bars, for stacks of six
    layers, where the flat max-abs bar on the stored value is known to be out of reach of bf16 operands."""
    a, b = y_gpu[rows], y_ref[rows]
    mag = np.maximum(np.abs(b), 1e-30)
    half_ulp = 2.0 ** (np.floor(np.log2(mag)) - 8)
    return bool((np.abs(a - b) <= budget + half_ulp).all())
