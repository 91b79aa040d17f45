"""Seeded synthetic placement schedules and move records.

Inputs only: a schedule is one boolean per (layer, step, page) saying "this
page sits in HBM while the step runs".  Nothing here evaluates a schedule.
"""
from __future__ import annotations

import numpy as np

from .traces import Trace, _rng

OP_SET, OP_SWAP, OP_SHIFT = 0, 1, 2
MOVE_FIELDS = ("op", "layer", "page", "n1", "len", "layer2", "page2", "dsel")


def random_placements(tr: Trace, S: int, seed: int, *, density: float = 0.3,
                      flip_rate: float = 0.05, feasible: bool = True) -> np.ndarray:
    """[S][L][N][P] booleans with temporal coherence: each (layer, page) starts
    in HBM with probability `density` and toggles with probability `flip_rate`
    per step.  With `feasible`, pages are dropped (by a fixed random priority
    per schedule) at every step whose occupancy exceeds the HBM capacity."""
    rng = _rng(seed, 3)
    L, N, P = tr.L, tr.N, tr.P
    X = np.empty((S, L, N, P), dtype=np.uint8)
    al = tr.alive.astype(bool)
    for s in range(S):
        start = rng.random((L, 1, P)) < density
        flips = rng.random((L, N, P)) < flip_rate
        flips[:, 0, :] = False
        x = start ^ (np.cumsum(flips, axis=1) & 1).astype(bool)
        x &= al[None]
        if feasible:
            prio = rng.random((L, P))
            occ = x.sum(axis=(0, 2))
            for n in np.nonzero(occ > tr.cap_pages)[0]:
                on = x[:, n, :]
                pr = np.where(on, prio, np.inf).ravel()
                keep = np.argpartition(pr, tr.cap_pages)[: tr.cap_pages] if tr.cap_pages > 0 else []
                m = np.zeros(L * P, dtype=bool)
                m[keep] = True
                x[:, n, :] = on & m.reshape(L, P)
        X[s] = x
    return X


def edge_placements(tr: Trace, seed: int = 0) -> np.ndarray:
    """Empty, every alive page, every bit (also dead slots), checkerboards."""
    rng = _rng(seed, 4)
    L, N, P = tr.L, tr.N, tr.P
    al = np.broadcast_to(tr.alive[None], (L, N, P))
    out = [np.zeros((L, N, P), np.uint8), al.copy(), np.ones((L, N, P), np.uint8)]
    cb = (np.add.outer(np.add.outer(np.arange(L), np.arange(N)), np.arange(P)) & 1).astype(np.uint8)
    out.append(cb & al)
    out.append(cb)                       # also sets dead pages
    out.append(((rng.random((L, N, P)) < 0.5) & (al > 0)).astype(np.uint8))
    return np.stack(out)


def random_moves(tr: Trace, S: int, seed: int, max_len: int = 63) -> dict:
    """S raw move records (before any clipping): uniform layer, page, first
    step and length, a second (layer, page) and a shift selector."""
    rng = _rng(seed, 5)
    m = {
        "op": rng.choice([OP_SET, OP_SWAP, OP_SHIFT], size=S, p=[0.4, 0.4, 0.2]),
        "layer": rng.integers(0, tr.L, S),
        "page": rng.integers(0, tr.P, S),
        "n1": rng.integers(0, tr.N, S),
        "len": rng.integers(1, max_len + 1, S),
        "layer2": rng.integers(0, tr.L, S),
        "page2": rng.integers(0, tr.P, S),
        "dsel": rng.integers(0, 4, S),
    }
    return {k: v.astype(np.uint32) for k, v in m.items()}


def moves_to_records(m: dict) -> np.ndarray:
    """[S][8] uint32, field order MOVE_FIELDS."""
    return np.stack([m[k] for k in MOVE_FIELDS], axis=1).astype(np.uint32)
