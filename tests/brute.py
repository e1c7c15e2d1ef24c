"""Brute-force fp64 definitions written straight from the paper's formulas with
numpy.  Used only to pin the oracle; shares nothing with oracle/ or the GPU
package."""
import numpy as np


def softmax64(z, axis=-1):
    z = np.asarray(z, np.float64)
    z = z - z.max(axis=axis, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=axis, keepdims=True)


def dense_attention(q, K, V, scale):
    """Textbook softmax(q K^T scale) V with grouped-query heads.  q [h,d], K,V [g,s,d]."""
    h, d = q.shape
    g = K.shape[0]
    G = h // g
    out = np.empty((h, d), np.float64)
    lse = np.empty(h, np.float64)
    for head in range(h):
        kv = head // G
        z = (K[kv].astype(np.float64) @ q[head].astype(np.float64)) * np.float64(scale)
        m = z.max()
        e = np.exp(z - m)
        out[head] = (e / e.sum()) @ V[kv].astype(np.float64)
        lse[head] = m + np.log(e.sum())
    return out, lse


def group_softmax_max(qs, Kset, scale):
    """max over the query heads of a KV group of softmax(q_h . K^set): qs [G,d], Kset [L,d] -> [L]."""
    z = (qs.astype(np.float64) @ Kset.astype(np.float64).T) * np.float64(scale)   # [G, L]
    return softmax64(z, axis=1).max(axis=0)


def top_ids(score, ids, n):
    """ids of the n largest scores, ties to the lowest id, returned ascending."""
    score = np.asarray(score)
    ids = np.asarray(ids)
    order = np.lexsort((ids, -score))
    return np.sort(ids[order[:n]])


def check_topn_within_band(chosen, score64, ids, n, rel_band):
    """`chosen` must hold n ids and agree with the exact top-n of score64 except
    for ids whose score lies within rel_band of the n-th largest score."""
    chosen = np.asarray(chosen)
    ids = np.asarray(ids)
    n = min(n, len(ids))
    assert len(chosen) == n
    assert np.all(np.diff(chosen) > 0), "not strictly ascending"
    assert np.all(np.isin(chosen, ids))
    if n == len(ids):
        return 0
    srt = np.sort(score64)[::-1]
    kth = srt[n - 1]
    lo, hi = kth - abs(kth) * rel_band, kth + abs(kth) * rel_band
    must_in = ids[score64 > hi]
    must_out = ids[score64 < lo]
    assert np.all(np.isin(must_in, chosen)), "a clearly better id was left out"
    assert not np.any(np.isin(must_out, chosen)), "a clearly worse id was chosen"
    return int(np.sum((score64 >= lo) & (score64 <= hi))) - 1   # others within the band of the n-th
