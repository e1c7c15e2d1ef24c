"""k-means++ seeding of the k-means centroid mode, as an INPUT generator: it
returns prompt *positions* (init_pos) that both the CPU oracle and the GPU
library take as given.  fp64 D^2 sampling with numpy's Philox; the first centre
is drawn uniformly.  Kept apart from the oracle and from the GPU code: neither
implements it."""
from __future__ import annotations

import numpy as np


def kmeanspp_positions(X: np.ndarray, C: int, seed: int) -> np.ndarray:
    """X [n][dim] points -> int32 [C] distinct row indices chosen by D^2 sampling."""
    n = X.shape[0]
    assert 1 <= C <= n
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence([int(seed), 17, n, C])))
    X64 = X.astype(np.float64)
    xx = np.einsum("ij,ij->i", X64, X64)
    pos = np.empty(C, np.int64)
    pos[0] = rng.integers(0, n)
    d2 = np.maximum(xx - 2.0 * (X64 @ X64[pos[0]]) + xx[pos[0]], 0.0)
    d2[pos[0]] = 0.0
    for c in range(1, C):
        tot = d2.sum()
        if tot <= 0.0:                       # every point coincides with a centre: take unused rows in order
            unused = np.setdiff1d(np.arange(n), pos[:c])
            pos[c:] = unused[:C - c]
            break
        r = rng.random() * tot
        i = int(np.searchsorted(np.cumsum(d2), r, side="right"))
        i = min(i, n - 1)
        while d2[i] <= 0.0:                  # never pick a point that already is a centre
            i = (i + 1) % n
        pos[c] = i
        nd = np.maximum(xx - 2.0 * (X64 @ X64[i]) + xx[i], 0.0)
        d2 = np.minimum(d2, nd)
        d2[i] = 0.0
    return pos.astype(np.int32)


def kmeanspp_for_sequence(q_full: np.ndarray, g: int, C: int, seed: int) -> np.ndarray:
    """[s][h][d] prompt queries -> init_pos int32 [g][C] (points = per-position concatenation of a KV group's heads)."""
    s, h, d = q_full.shape
    G = h // g
    X = q_full.reshape(s, g, G * d)
    return np.stack([kmeanspp_positions(np.ascontiguousarray(X[:, kv, :]), C, seed * 131 + kv) for kv in range(g)])


def centroid_positions(mode: str, s: int, C: int, g: int, seed: int = 0) -> np.ndarray:
    """Prompt positions [g][C] of the queries kept as centroids under the four placements the
    paper compares (ablation on the position of the maintained centroids): "final" = the last C
    (the method's own choice, Algorithm 1 line 1), "init" = the first C, "equi" = evenly spaced,
    "random" = C distinct positions drawn with Philox(seed), sorted.  The same positions for
    every KV head."""
    if mode == "final":
        pos = np.arange(s - C, s)
    elif mode == "init":
        pos = np.arange(C)
    elif mode == "equi":
        pos = (np.arange(C, dtype=np.int64) * s) // C + (s // C) // 2
    elif mode == "random":
        rng = np.random.Generator(np.random.Philox(np.random.SeedSequence([int(seed), 23, s, C])))
        pos = np.sort(rng.choice(s, size=C, replace=False))
    else:
        raise KeyError(mode)
    return np.broadcast_to(pos.astype(np.int32), (g, C)).copy()
