"""Python face of the CPU oracle (``ctkvr_oracle.c``) -- TEST INFRASTRUCTURE.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It never imports the GPU package and the
GPU package never imports it.

The functions below only marshal numpy arrays into the C routines; the
arithmetic of the method lives in ``ctkvr_oracle.c`` where each routine cites
the lines of the paper's Algorithm 1 / Algorithm 2 it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ctkvr_oracle.c")
_LIB = os.path.join(_HERE, "libctkvr_oracle.so")

CFLAGS = ["-O2", "-mfma", "-mavx2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (contraction off: every fused multiply-add
    in it is an explicit ``fmaf``/``fma``)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *CFLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        ci = ctypes.c_int
        L.ctkvr_oracle_dot128.restype = ctypes.c_float
        L.ctkvr_oracle_dot128.argtypes = [fp, fp]
        L.ctkvr_oracle_inv_norm.restype = ctypes.c_float
        L.ctkvr_oracle_inv_norm.argtypes = [fp]
        L.ctkvr_oracle_exp.restype = ctypes.c_float
        L.ctkvr_oracle_exp.argtypes = [ctypes.c_float]
        L.ctkvr_oracle_log_fixed.restype = ctypes.c_double
        L.ctkvr_oracle_log_fixed.argtypes = [ctypes.c_uint64]
        L.ctkvr_oracle_build_lists.restype = None
        L.ctkvr_oracle_build_lists.argtypes = [fp, fp, ci, ci, ci, ci, ci, ctypes.c_float, ip, ci, ci, ci, ip, fp]
        L.ctkvr_oracle_inv_norms.restype = None
        L.ctkvr_oracle_inv_norms.argtypes = [fp, ci, fp]
        L.ctkvr_oracle_recall.restype = None
        L.ctkvr_oracle_recall.argtypes = [fp, fp, ci, ci, ci, ci, fp, ip]
        L.ctkvr_oracle_rerank_attend.restype = None
        L.ctkvr_oracle_rerank_attend.argtypes = [fp, fp, fp, ip, ip, ci, ci, ci, ci, ci, ci, ci, ctypes.c_float,
                                                 ip, ip, fp, ip, dp, dp]
        L.ctkvr_oracle_kmeans.restype = None
        L.ctkvr_oracle_kmeans.argtypes = [fp, ci, ci, fp, ci, ci, ci, ip, dp]
        L.ctkvr_oracle_num_threads.restype = ci
        L.ctkvr_oracle_set_threads.argtypes = [ci]
        _lib = L
    return _lib


def _f(a: np.ndarray):
    assert a.dtype == np.float32 and a.flags.c_contiguous
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _d(a: np.ndarray):
    assert a.dtype == np.float64 and a.flags.c_contiguous
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _i(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.dtype == np.int32 and a.flags.c_contiguous
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def default_scale(d: int = 128) -> np.float32:
    """1/sqrt(d) rounded once to fp32."""
    return np.float32(1.0 / np.sqrt(np.float64(d)))


# ---- primitives (exposed so the tests can pin them) ------------------------ #
def dot128(a: np.ndarray, b: np.ndarray) -> np.float32:
    a = np.ascontiguousarray(a, np.float32)
    b = np.ascontiguousarray(b, np.float32)
    assert a.shape == (128,) and b.shape == (128,)
    return np.float32(lib().ctkvr_oracle_dot128(_f(a), _f(b)))


def exp_c(x: float) -> np.float32:
    return np.float32(lib().ctkvr_oracle_exp(ctypes.c_float(x)))


def log_fixed(S: int) -> float:
    return float(lib().ctkvr_oracle_log_fixed(ctypes.c_uint64(S)))


def inv_norms(X: np.ndarray) -> np.ndarray:
    X = np.ascontiguousarray(X, np.float32)
    assert X.shape[-1] == 128
    out = np.empty(X.shape[:-1], np.float32)
    lib().ctkvr_oracle_inv_norms(_f(X), int(np.prod(X.shape[:-1])), _f(out))
    return out


# ---- Algorithm 1 ----------------------------------------------------------- #
def centroids_last_c(q_tail: np.ndarray, C: int) -> np.ndarray:
    """Algorithm 1 line 1: the last C prefill queries, as [h][C][d].
    ``q_tail`` is [n_tail >= C][h][d] ending at the last prompt position."""
    assert q_tail.shape[0] >= C
    return np.ascontiguousarray(np.transpose(q_tail[q_tail.shape[0] - C:], (1, 0, 2)), np.float32)


def build_lists(K: np.ndarray, Qc: np.ndarray, rho: int, scale: Optional[float] = None,
                pairs: Optional[np.ndarray] = None, return_keys: bool = False, n_init: int = 0, n_local: int = 0):
    """Algorithm 1 lines 2-4.  K [g][s][d], Qc [h][C][d] -> lists int32.
    With ``pairs`` ([n][2] of (kv head, centroid)) only those lists are built,
    returned as [n][rho]; otherwise [g][C][rho].  The first n_init and last n_local keys
    (the resident window of lines 5-6) are scored but never listed."""
    K = np.ascontiguousarray(K, np.float32)
    Qc = np.ascontiguousarray(Qc, np.float32)
    g, s, d = K.shape
    h, C, _ = Qc.shape
    assert d == 128 and h % g == 0 and n_init >= 0 and n_local >= 0 and 1 <= rho <= s - n_init - n_local
    scale = default_scale(d) if scale is None else np.float32(scale)
    if pairs is not None:
        pairs = np.ascontiguousarray(pairs, np.int32).reshape(-1, 2)
        n = pairs.shape[0]
        shape = (n, rho)
    else:
        n = g * C
        shape = (g, C, rho)
    lists = np.empty(shape, np.int32)
    keys = np.empty((n, s), np.float32) if return_keys else None
    lib().ctkvr_oracle_build_lists(_f(K), _f(Qc), h, g, s, C, rho, ctypes.c_float(scale), _i(pairs), n,
                                   int(n_init), int(n_local), _i(lists), _f(keys) if keys is not None else None)
    return (lists, keys) if return_keys else lists


# ---- Algorithm 2 ----------------------------------------------------------- #
def recall(q: np.ndarray, Qc: np.ndarray, g: int, n_probe: int) -> Tuple[np.ndarray, np.ndarray]:
    """Algorithm 2 lines 1-3.  q [h][d], Qc [h][C][d] -> (Cos_kv [g][C], I^Q [g][C'] ascending)."""
    q = np.ascontiguousarray(q, np.float32)
    Qc = np.ascontiguousarray(Qc, np.float32)
    h, C, d = Qc.shape
    assert q.shape == (h, d) and d == 128 and 1 <= n_probe <= C
    cos_kv = np.empty((g, C), np.float32)
    probe = np.empty((g, n_probe), np.int32)
    lib().ctkvr_oracle_recall(_f(q), _f(Qc), h, g, C, n_probe, _f(cos_kv), _i(probe))
    return cos_kv, probe


@dataclass
class DecodeResult:
    cos_kv: np.ndarray      # [g][C] fp32
    probe: np.ndarray       # [g][C'] int32 ascending
    cand: list              # per kv head: int32 array of the L recalled key ids, ascending
    ncand: np.ndarray       # [g] int32
    rerank_key: list        # per kv head: fp32 [L] max-over-group log-softmax over the recalled set
    sel: np.ndarray         # [g][top_k] int32 ascending, -1 padded
    out: np.ndarray         # [h][d] fp64
    lse: np.ndarray         # [h] fp64


def rerank_attend(q, K, V, lists, probe, top_k, scale=None):
    """Algorithm 2 lines 4-9 given the probed centroid ids."""
    q = np.ascontiguousarray(q, np.float32)
    K = np.ascontiguousarray(K, np.float32)
    V = np.ascontiguousarray(V, np.float32)
    lists = np.ascontiguousarray(lists, np.int32)
    probe = np.ascontiguousarray(probe, np.int32)
    g, s, d = K.shape
    h = q.shape[0]
    _, C, rho = lists.shape
    n_probe = probe.shape[1]
    scale = default_scale(d) if scale is None else np.float32(scale)
    Lmax = min(s, n_probe * rho)
    cand = np.full((g, Lmax), -1, np.int32)
    ncand = np.zeros(g, np.int32)
    rkey = np.zeros((g, Lmax), np.float32)
    sel = np.empty((g, top_k), np.int32)
    out = np.empty((h, d), np.float64)
    lse = np.empty(h, np.float64)
    lib().ctkvr_oracle_rerank_attend(_f(q), _f(K), _f(V), _i(lists), _i(probe), h, g, s, C, rho, n_probe, top_k,
                                     ctypes.c_float(scale), _i(cand), _i(ncand), _f(rkey), _i(sel), _d(out), _d(lse))
    return cand, ncand, rkey, sel, out, lse


def decode_step(q, K, V, Qc, lists, n_probe, top_k, scale=None) -> DecodeResult:
    """Algorithm 2 lines 1-9 for one sequence and one decode query."""
    g = K.shape[0]
    cos_kv, probe = recall(q, Qc, g, n_probe)
    cand, ncand, rkey, sel, out, lse = rerank_attend(q, K, V, lists, probe, top_k, scale)
    return DecodeResult(cos_kv, probe, [cand[i, :ncand[i]].copy() for i in range(g)], ncand,
                        [rkey[i, :ncand[i]].copy() for i in range(g)], sel, out, lse)


def window_attention(q, K, V, n_init: int, s_index: int, n_local: int, scale=None):
    """Attention of every query head over the resident window (Algorithm 2 line 10): the first
    n_init keys and the keys from s_index - n_local to the end of K (the local window grows with
    the tokens decoded since the index was built).  fp64.  Returns (out [h][d], lse [h]);
    an empty window gives zeros and -inf."""
    q = np.asarray(q, np.float64)
    g, s_cur, d = K.shape
    h = q.shape[0]
    G = h // g
    scale = float(default_scale(d) if scale is None else scale)
    rows = np.concatenate([np.arange(0, n_init), np.arange(s_index - n_local, s_cur)])
    out = np.zeros((h, d), np.float64)
    lse = np.full(h, -np.inf, np.float64)
    if len(rows) == 0:
        return out, lse
    for head in range(h):
        kv = head // G
        z = (np.asarray(K[kv, rows], np.float64) @ q[head]) * scale
        m = z.max()
        e = np.exp(z - m)
        out[head] = (e / e.sum()) @ np.asarray(V[kv, rows], np.float64)
        lse[head] = m + np.log(e.sum())
    return out, lse


def merge_attention(out_a, lse_a, out_b, lse_b):
    """Algorithm 2 line 11: two attention outputs over disjoint key sets combined into the
    attention over their union, through their log-sum-exps."""
    m = np.maximum(lse_a, lse_b)
    m = np.where(np.isfinite(m), m, 0.0)
    wa, wb = np.exp(lse_a - m), np.exp(lse_b - m)
    den = wa + wb
    out = (out_a * wa[:, None] + out_b * wb[:, None]) / den[:, None]
    return out, m + np.log(den)


def decode_step_window(q, K, V, Qc, lists, n_probe, top_k, s_index: int, n_init: int, n_local: int, scale=None) -> DecodeResult:
    """Algorithm 2 lines 1-11 with a resident window: retrieval and sparse attention over the
    s_index keys the index was built on (its lists hold no window keys), attention over the
    window -- K and V may have grown beyond s_index by the decoded tokens -- and the merge."""
    r = decode_step(q, K[:, :s_index], V[:, :s_index], Qc, lists, n_probe, top_k, scale)
    out_w, lse_w = window_attention(q, K, V, n_init, s_index, n_local, scale)
    r.out, r.lse = merge_attention(r.out, r.lse, out_w, lse_w)
    return r


def centroid_update(q, Qc, lists, res: DecodeResult, n_updates: int) -> int:
    """Algorithm 2 line 12 (dynamic centroid update), in place, after the decode step `res` of
    query q: the query becomes the centroid of FIFO slot n_updates mod C for every query head,
    and that slot's list becomes the rho keys with the largest rerank score A'_kv (the same
    score line 6 ranks by, over the recalled set), ties to the lowest key id, stored ascending.
    The oldest mapping goes first: slot 0 holds the earliest prompt query.  Should fewer than rho
    keys have been recalled the last one is repeated (a list always has rho entries).
    Returns the slot written."""
    q = np.asarray(q, np.float32)
    g, C, rho = lists.shape
    slot = int(n_updates) % C
    for kv in range(g):
        key = np.asarray(res.rerank_key[kv], np.float32)
        cand = np.asarray(res.cand[kv], np.int32)
        L = len(cand)
        if L == 0:
            continue
        n = min(rho, L)
        order = np.lexsort((cand, -key.astype(np.float64)))   # score descending, then key id ascending
        top = np.sort(cand[order[:n]])
        lists[kv, slot, :n] = top
        lists[kv, slot, n:] = top[-1]
    Qc[:, slot, :] = q
    return slot


# ---- k-means centroid mode -------------------------------------------------- #
def group_points(q_full: np.ndarray, g: int) -> np.ndarray:
    """[s][h][d] prompt queries -> [g][s][G*d]: a point is the concatenation of the G
    query-head vectors of a KV group at one position."""
    s, h, d = q_full.shape
    G = h // g
    return np.ascontiguousarray(q_full.reshape(s, g, G * d).transpose(1, 0, 2), np.float32)


def kmeans_centroids(q_full: np.ndarray, g: int, init_pos: np.ndarray, iters: int, dtype: str = "bf16"):
    """Lloyd iterations from the centres at prompt positions init_pos [g][C].
    Returns (Qc [h][C][d], assign [g][s], inertia [g][iters+1])."""
    s, h, d = q_full.shape
    G = h // g
    C = init_pos.shape[1]
    X = group_points(q_full, g)
    Qc = np.empty((h, C, d), np.float32)
    assign = np.empty((g, s), np.int32)
    inertia = np.empty((g, iters + 1), np.float64)
    for kv in range(g):
        cent = np.ascontiguousarray(X[kv][init_pos[kv]], np.float32)
        lib().ctkvr_oracle_kmeans(_f(X[kv]), s, G * d, _f(cent), C, iters, int(dtype == "bf16"), _i(assign[kv]),
                                  _d(inertia[kv]))
        Qc[kv * G:(kv + 1) * G] = cent.reshape(C, G, d).transpose(1, 0, 2)
    return Qc, assign, inertia


def kmeans_from_centres(q_full: np.ndarray, g: int, Qc0: np.ndarray, iters: int, dtype: str = "bf16"):
    """The same Lloyd iterations started from explicit centres Qc0 [h][C][d] (per KV head the
    concatenation of its G heads' rows) instead of prompt positions.  Same returns as
    kmeans_centroids."""
    s, h, d = q_full.shape
    G = h // g
    C = Qc0.shape[1]
    X = group_points(q_full, g)
    Qc = np.empty((h, C, d), np.float32)
    assign = np.empty((g, s), np.int32)
    inertia = np.empty((g, iters + 1), np.float64)
    for kv in range(g):
        cent = np.ascontiguousarray(np.asarray(Qc0[kv * G:(kv + 1) * G], np.float32).transpose(1, 0, 2).reshape(C, G * d))
        lib().ctkvr_oracle_kmeans(_f(X[kv]), s, G * d, _f(cent), C, iters, int(dtype == "bf16"), _i(assign[kv]),
                                  _d(inertia[kv]))
        Qc[kv * G:(kv + 1) * G] = cent.reshape(C, G, d).transpose(1, 0, 2)
    return Qc, assign, inertia


def num_threads() -> int:
    return int(lib().ctkvr_oracle_num_threads())


def set_threads(n: int) -> None:
    lib().ctkvr_oracle_set_threads(int(n))
