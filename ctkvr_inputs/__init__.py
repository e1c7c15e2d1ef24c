"""Seeded synthetic inputs for the CTkvr decode/build path.

This module only *generates data*: Gaussian keys and values, random-walk
queries, rotary position embedding of the generated vectors, bf16 rounding of
the generated values, and the physical paging of a KV cache.  It contains none
of the retrieval method's arithmetic (no scores, no selections, no softmax), so
that both the CPU oracle's tests and the GPU tests can draw the very same
inputs from it without sharing any of the computation under test.

Recipe (per sequence, seed ``sigma``; all draws from ``numpy.random.Philox``):

* keys      ``k_t ~ N(0, I_d)`` per KV head, rotated by RoPE at position ``t``;
* values    ``v_t ~ N(0, I_d)`` per KV head, no RoPE;
* queries   per *query* head a Gaussian random walk ``w_t = w_{t-1} + step * N(0, I)``
            with ``w_0 ~ N(0, I)``; the post-RoPE query at position ``t`` is
            ``RoPE(w_t, t)``.  Adjacent positions are therefore similar, which is
            the property of real post-RoPE queries the method relies on
            (Observation 1 of the paper).  Decode queries continue the same walk
            at positions ``s, s+1, ...``.
* RoPE      rotate-half pairing ``(i, i + d/2)``, ``theta_i = base**(-2 i / d)``,
            angle ``pos * theta_i``, evaluated in fp64.
* rounding  fp64 -> fp32 (round to nearest even) and, for bf16 workloads,
            fp32 -> bf16 (round to nearest even on the bit pattern).
* paging    the tokens of every sequence are cut into ``page_size``-token pages
            (last page possibly partial) and the pages of all sequences are
            scattered over the physical page pool by a seeded permutation.

bf16 arrays are carried as ``uint16`` bit patterns on the numpy side.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

ROPE_BASE = 10000.0
WALK_STEP = 0.05


# --------------------------------------------------------------------------- #
# dtype helpers (data representation only)
# --------------------------------------------------------------------------- #
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest even), returned as uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    # no generated value comes near the top of the exponent range, so the 32-bit sum cannot wrap
    u = u + np.uint32(0x7FFF) + lsb
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


def round_to_dtype(x64: np.ndarray, dtype: str) -> np.ndarray:
    """fp64 -> the workload's storage dtype, returned as fp32 *values*."""
    x32 = x64.astype(np.float32)
    if dtype == "f32":
        return x32
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(x32))
    raise ValueError(dtype)


# --------------------------------------------------------------------------- #
# RoPE (applied to generated vectors; the library itself takes post-RoPE data)
# --------------------------------------------------------------------------- #
def rope_tables(pos: np.ndarray, d: int, base: float = ROPE_BASE):
    """cos and sin of the rotation angles of positions ``pos`` for head dimension ``d`` (fp64)."""
    half = d // 2
    theta = base ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = np.asarray(pos, dtype=np.float64)[..., None] * theta
    return np.cos(ang), np.sin(ang)


def rope(x: np.ndarray, pos: np.ndarray, base: float = ROPE_BASE, tables=None) -> np.ndarray:
    """Rotate ``x[..., d]`` (fp64) by the angles of positions ``pos`` (broadcast
    against the leading axes of ``x``), rotate-half pairing.  ``tables`` may carry
    ``rope_tables(pos, d)`` computed once for many calls at the same positions."""
    half = x.shape[-1] // 2
    c, s = rope_tables(pos, x.shape[-1], base) if tables is None else tables
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


# --------------------------------------------------------------------------- #
# one sequence
# --------------------------------------------------------------------------- #
@dataclass
class Sequence:
    """One synthetic sequence.  All arrays hold fp32 *values* that are exactly
    representable in ``dtype``."""
    seed: int
    dtype: str
    s: int                      # context length
    K: np.ndarray               # [g, s, d]
    V: np.ndarray               # [g, s, d]
    q_tail: np.ndarray          # [n_tail, h, d] post-RoPE prefill queries at positions s-n_tail .. s-1
    q_decode: np.ndarray        # [n_decode, h, d] post-RoPE decode queries at positions s, s+1, ...
    q_full: Optional[np.ndarray] = None   # [s, h, d] all prefill queries (only if asked for)


class _Done:
    """Result holder for work run in place (short sequences need no thread pool)."""
    def __init__(self, value):
        self.value = value

    def result(self):
        return self.value


def gen_sequence(seed: int, s: int, h: int, g: int, d: int, n_tail: int, n_decode: int,
                 dtype: str = "bf16", full_walk: bool = False,
                 walk_step: float = WALK_STEP) -> Sequence:
    """Draw one sequence.

    With ``full_walk=False`` the walk state at position ``s - n_tail`` is drawn
    from its exact marginal ``N(0, (1 + walk_step^2 (s - n_tail)) I)`` and only
    the last ``n_tail`` prefill positions plus the decode positions are walked:
    this is the same process restricted to the positions the last-C index needs.
    With ``full_walk=True`` every prefill position is generated.
    """
    assert 0 < n_tail <= s and n_decode >= 0
    root = np.random.SeedSequence([int(seed), s, h, g, d])
    ss_k, ss_v, ss_q = root.spawn(3)
    rk = np.random.Generator(np.random.Philox(ss_k))
    rv = np.random.Generator(np.random.Philox(ss_v))
    rq = np.random.Generator(np.random.Philox(ss_q))

    # The draws are taken in a fixed order (keys and values head by head, then the walk of every
    # query head); rotating and rounding a head's draws does not touch the generators and runs on
    # a small thread pool for long sequences.
    from concurrent.futures import ThreadPoolExecutor
    pool = ThreadPoolExecutor(max_workers=4) if s * d >= (1 << 22) else None
    run = pool.submit if pool else (lambda f, *a: _Done(f(*a)))
    pos = np.arange(s)
    ktab = rope_tables(pos, d)
    K = np.empty((g, s, d), dtype=np.float32)
    V = np.empty((g, s, d), dtype=np.float32)

    def put_kv(j, kraw, vraw):
        K[j] = round_to_dtype(rope(kraw, pos, tables=ktab), dtype)
        V[j] = round_to_dtype(vraw, dtype)

    jobs = []
    for j in range(g):
        jobs.append(run(put_kv, j, rk.standard_normal((s, d)), rv.standard_normal((s, d))))
        if len(jobs) >= 6:
            jobs.pop(0).result()

    start = 0 if full_walk else s - n_tail
    n_pos = s + n_decode - start
    qpos = np.arange(start, s + n_decode)
    qtab = rope_tables(qpos, d)
    q_all = np.empty((n_pos, h, d), dtype=np.float32)

    def put_q(i, inc):
        inc[0] *= np.sqrt(1.0 + walk_step * walk_step * start)
        inc[1:] *= walk_step
        w = np.cumsum(inc, axis=0)
        q_all[:, i, :] = round_to_dtype(rope(w, qpos, tables=qtab), dtype)

    for i in range(h):
        jobs.append(run(put_q, i, rq.standard_normal((n_pos, d))))
        if len(jobs) >= 6:
            jobs.pop(0).result()
    for j in jobs:
        j.result()
    if pool:
        pool.shutdown()
    n_pref = s - start
    q_pref = q_all[:n_pref]
    return Sequence(seed=seed, dtype=dtype, s=s, K=K, V=V,
                    q_tail=np.ascontiguousarray(q_pref[n_pref - n_tail:]),
                    q_decode=np.ascontiguousarray(q_all[n_pref:]),
                    q_full=np.ascontiguousarray(q_pref) if full_walk else None)


def gen_lattice_sequence(seed: int, s: int, h: int, g: int, d: int, n_tail: int, n_decode: int,
                         denom: int = 8, span: int = 8) -> Sequence:
    """Inputs on the lattice ``{k/denom : |k| <= span}``: every product and every
    partial sum of a 128-term dot product is exactly representable in fp32, so
    a dot product has one value whatever the summation order."""
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence([int(seed), 7, s, h, g, d])))
    def lat(shape):
        return (rng.integers(-span, span + 1, size=shape).astype(np.float32) / np.float32(denom))
    K, V = lat((g, s, d)), lat((g, s, d))
    q_tail, q_dec = lat((n_tail, h, d)), lat((n_decode, h, d))
    return Sequence(seed=seed, dtype="bf16", s=s, K=K, V=V, q_tail=q_tail, q_decode=q_dec)


# --------------------------------------------------------------------------- #
# paging (pure data movement)
# --------------------------------------------------------------------------- #
@dataclass
class PagedKV:
    k_pages: np.ndarray         # [num_pages, g, page_size, d] fp32 values
    v_pages: np.ndarray
    block_table: np.ndarray     # int32 [batch, max_pages], unused entries -1
    ctx_lens: np.ndarray        # int32 [batch]
    page_size: int


def paginate(seqs: List[Sequence], page_size: int = 16, seed: int = 0, spare_pages: int = 3) -> PagedKV:
    """Scatter the tokens of ``seqs`` over a physical page pool.  The physical
    order of the pages is a seeded permutation, so logically adjacent pages are
    not adjacent in memory; ``spare_pages`` unused pages (filled with a large
    sentinel value) are mixed in so that a wrong page lookup is visible."""
    g, _, d = seqs[0].K.shape
    n_pages_seq = [(q.s + page_size - 1) // page_size for q in seqs]
    total = sum(n_pages_seq) + spare_pages
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence([int(seed), 11, total])))
    perm = rng.permutation(total).astype(np.int32)
    k_pages = np.full((total, g, page_size, d), 3.0e4, dtype=np.float32)
    v_pages = np.full((total, g, page_size, d), 3.0e4, dtype=np.float32)
    max_pages = max(n_pages_seq)
    bt = np.full((len(seqs), max_pages), -1, dtype=np.int32)
    at = 0
    for b, q in enumerate(seqs):
        npg = n_pages_seq[b]
        phys = perm[at:at + npg]
        at += npg
        bt[b, :npg] = phys
        pad = npg * page_size - q.s
        Kp = np.pad(q.K, ((0, 0), (0, pad), (0, 0))) if pad else q.K
        Vp = np.pad(q.V, ((0, 0), (0, pad), (0, 0))) if pad else q.V
        # [g, npg, page, d] -> [npg, g, page, d]
        k_pages[phys] = Kp.reshape(g, npg, page_size, d).transpose(1, 0, 2, 3)
        v_pages[phys] = Vp.reshape(g, npg, page_size, d).transpose(1, 0, 2, 3)
    return PagedKV(k_pages=k_pages, v_pages=v_pages, block_table=bt,
                   ctx_lens=np.array([q.s for q in seqs], dtype=np.int32), page_size=page_size)


# --------------------------------------------------------------------------- #
# the named workloads
# --------------------------------------------------------------------------- #
@dataclass
class Workload:
    name: str
    dtype: str
    h: int
    g: int
    d: int
    ctx_lens: List[int]
    seeds: List[int]
    n_centroids: int            # C; 0 => per sequence ctx_len // centroid_div
    centroid_div: int
    n_probe: int                # C'
    list_len: int               # rho
    top_k: int                  # rho'
    n_decode: int
    page_size: int = 16
    page_seed: int = 0

    def centroids_of(self, s: int) -> int:
        return self.n_centroids if self.n_centroids > 0 else s // self.centroid_div

    @property
    def batch(self) -> int:
        return len(self.ctx_lens)


def _ragged_lengths(seed: int, n: int, lo: int, hi: int) -> List[int]:
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence([int(seed), 13])))
    return [int(x) for x in rng.integers(lo, hi + 1, size=n)]


def workload(name: str) -> Workload:
    """The five benchmark configurations (list length rho = top_k in all of them) and the paper's operating point."""
    if name == "cfg1":   # tiny fp32, GQA 8/2
        return Workload("cfg1", "f32", 8, 2, 128, [4096], [1], 64, 0, 8, 256, 256, 4)
    if name == "cfg2":   # Llama-3-8B-shaped layer, 32K
        return Workload("cfg2", "bf16", 32, 8, 128, [32768], [2], 512, 0, 32, 1024, 1024, 256, page_seed=2)
    if name == "cfg3":   # 128K, batch 4
        return Workload("cfg3", "bf16", 32, 8, 128, [131072] * 4, [30, 31, 32, 33], 2048, 0, 64, 2048, 2048, 128,
                        page_seed=3)
    if name == "cfg4":   # ragged batch of 16
        lens = _ragged_lengths(4, 16, 8192, 65536)
        return Workload("cfg4", "bf16", 32, 8, 128, lens, list(range(40, 56)), 0, 64, 32, 1024, 1024, 64,
                        page_seed=4)
    if name == "cfg5":   # index build only, 128K
        return Workload("cfg5", "bf16", 32, 8, 128, [131072], [5], 2048, 0, 64, 2048, 2048, 0, page_seed=5)
    # The paper's own operating point (experimental setup of the evaluation section): C = min(2048, s/16),
    # C' = 4, rho = 2.5 rho', rho' in {512, 1024}; Llama-3-8B (32/8 heads) and Yi-9B (32/4 heads) shapes.
    if name == "paper_llama":
        return Workload("paper_llama", "bf16", 32, 8, 128, [32768], [61], 2048, 0, 4, 2560, 1024, 64, page_seed=61)
    if name == "paper_yi":
        return Workload("paper_yi", "bf16", 32, 4, 128, [32768], [62], 2048, 0, 4, 1280, 512, 64, page_seed=62)
    # The dynamic budget of the appendix comparison at equal sparsity: rho' = 4 % of the context, rho = 2.5 rho'.
    if name == "paper_budget4":
        return Workload("paper_budget4", "bf16", 32, 8, 128, [32768], [63], 2048, 0, 4, 3277, 1311, 64, page_seed=63)
    raise KeyError(name)


@dataclass
class Batch:
    wl: Workload
    seqs: List[Sequence]
    paged: PagedKV
    extra: Dict[str, object] = field(default_factory=dict)


def gen_batch(wl: Workload, n_decode: Optional[int] = None, full_walk: bool = False) -> Batch:
    nd = wl.n_decode if n_decode is None else n_decode
    seqs = [gen_sequence(seed, s, wl.h, wl.g, wl.d, wl.centroids_of(s), nd, wl.dtype, full_walk=full_walk)
            for seed, s in zip(wl.seeds, wl.ctx_lens)]
    return Batch(wl=wl, seqs=seqs, paged=paginate(seqs, wl.page_size, wl.page_seed))


def small_workload(name: str = "small", dtype: str = "bf16", h: int = 8, g: int = 2, ctx_lens=(1000,),
                   seeds=(100,), n_centroids: int = 24, centroid_div: int = 0, n_probe: int = 4,
                   list_len: int = 96, top_k: int = 64, n_decode: int = 3, page_size: int = 16) -> Workload:
    """Free-form small workloads for tests."""
    return Workload(name, dtype, h, g, 128, list(ctx_lens), list(seeds), n_centroids, centroid_div, n_probe,
                    list_len, top_k, n_decode, page_size=page_size, page_seed=int(seeds[0]))
