"""Glue for the GPU parity tests: moves the seeded inputs to the device, builds
the oracle's index and runs both sides on the same inputs.  No arithmetic of
the method lives here."""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional

import numpy as np

import oracle
from ctkvr_inputs import Batch, Workload, f32_to_bf16_bits
from ctkvr_inputs.device import (DeviceBatch, device_batch, device_full_queries, params_of, to_dev,  # noqa: F401
                                 torch_dtype)

REL_TOL = 2e-3   # max relative error of the attention output (bf16 inputs, fp32 accumulation)


@dataclass
class OracleIndex:
    Qc: List[np.ndarray]        # per sequence [h][C_i][d]
    lists: List[np.ndarray]     # per sequence [g][C_i][rho]

    def padded(self, wl: Workload):
        """[B][h][C_max][d] centroid table (storage dtype) and [B][g][C_max][rho] lists, zero padded."""
        c_max = max(q.shape[1] for q in self.Qc)
        cen = np.zeros((len(self.Qc), wl.h, c_max, wl.d), np.float32)
        lst = np.zeros((len(self.Qc), wl.g, c_max, wl.list_len), np.int32)
        for b, (q, l) in enumerate(zip(self.Qc, self.lists)):
            cen[b, :, :q.shape[1]] = q
            lst[b, :, :l.shape[1]] = l
        return (f32_to_bf16_bits(cen) if wl.dtype == "bf16" else cen), lst


def oracle_index(bt: Batch) -> OracleIndex:
    wl = bt.wl
    Qc = [oracle.centroids_last_c(sq.q_tail, wl.centroids_of(sq.s)) for sq in bt.seqs]
    lists = [oracle.build_lists(sq.K, q, wl.list_len) for sq, q in zip(bt.seqs, Qc)]
    return OracleIndex(Qc, lists)


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """Per output row (one query head): max |got - ref| / max |ref|; returns the worst row."""
    got = got.reshape(-1, got.shape[-1]).astype(np.float64)
    ref = ref.reshape(-1, ref.shape[-1]).astype(np.float64)
    return float(np.max(np.max(np.abs(got - ref), axis=1) / np.max(np.abs(ref), axis=1)))


def run_decode_parity(bt: Batch, oi: OracleIndex, idx, db: DeviceBatch, steps: Optional[List[int]] = None,
                      check_candidates: bool = True, update: bool = False) -> dict:
    """Run decode steps on the GPU index `idx` and on the oracle with index `oi`;
    assert bit-equal integers and outputs within REL_TOL.  With update=True both sides
    apply the dynamic centroid update after every step (`oi` is changed in place).
    Returns statistics."""
    import torch
    import paper_2512_15550_amd as ck
    wl = bt.wl
    B, h, g, d = wl.batch, wl.h, wl.g, wl.d
    steps = list(range(bt.seqs[0].q_decode.shape[0])) if steps is None else steps
    out = torch.empty((B, h, d), dtype=torch.float32, device="cuda")
    lse = torch.empty((B, h), dtype=torch.float32, device="cuda")
    sel = torch.empty((B, g, wl.top_k), dtype=torch.int32, device="cuda")
    ncand = torch.empty((B, g), dtype=torch.int32, device="cuda")
    probe = torch.empty((B, g, wl.n_probe), dtype=torch.int32, device="cuda")
    worst, worst_lse, alphas = 0.0, 0.0, []
    n_updates = 0
    for st in steps:
        q = np.stack([sq.q_decode[st] for sq in bt.seqs])
        q_dev = to_dev(q, wl)
        ck.ctkvr_decode_step(idx, q_dev, db.k_pages, db.v_pages, db.block_table, out, lse, sel, ncand, probe)
        torch.cuda.synchronize()
        g_out, g_lse = out.cpu().numpy(), lse.cpu().numpy()
        g_sel, g_ncand, g_probe = sel.cpu().numpy(), ncand.cpu().numpy(), probe.cpu().numpy()
        g_cand = ck.ctkvr_index_last_candidates(idx) if check_candidates else None
        for b, sq in enumerate(bt.seqs):
            r = oracle.decode_step(q[b], sq.K, sq.V, oi.Qc[b], oi.lists[b], wl.n_probe, wl.top_k)
            tag = f"step {st} seq {b}"
            assert np.array_equal(g_probe[b], r.probe), f"{tag}: probed centroids differ"
            assert np.array_equal(g_ncand[b], r.ncand), f"{tag}: L differs {g_ncand[b]} vs {r.ncand}"
            if check_candidates:
                for kv in range(g):
                    assert np.array_equal(g_cand[b, kv, :r.ncand[kv]], r.cand[kv]), f"{tag} kv {kv}: recalled ids differ"
            assert np.array_equal(g_sel[b], r.sel), f"{tag}: selected ids differ ({int(np.sum(g_sel[b] != r.sel))} slots)"
            e = rel_err(g_out[b], r.out)
            assert e <= REL_TOL, f"{tag}: output relative error {e:.3e} > {REL_TOL}"
            worst = max(worst, e)
            el = float(np.max(np.abs(g_lse[b] - r.lse) / np.maximum(1.0, np.abs(r.lse))))
            assert el <= 1e-4, f"{tag}: lse error {el:.3e}"
            worst_lse = max(worst_lse, el)
            alphas.append(float(np.mean(r.ncand)) / (wl.n_probe * wl.list_len))
            if update:
                oracle.centroid_update(q[b], oi.Qc[b], oi.lists[b], r, n_updates)
        if update:
            ck.ctkvr_centroid_update(idx, q_dev)
            n_updates += 1
    ck.ctkvr_index_check(idx)
    return {"max_rel_err": worst, "max_lse_err": worst_lse, "alpha": float(np.mean(alphas))}


def run_sampled_parity(bt: Batch, idx, db: DeviceBatch, steps: List[int], n_list_samples: int = 32, seed: int = 0,
                       say=print) -> dict:
    """Full-size parity where the oracle cannot afford the whole index: the GPU
    builds its own index; the oracle (a) rebuilds a random sample of its lists
    and (b) for the given decode steps rebuilds exactly the lists the step
    probes, then runs Algorithm 2 on them.  Every integer must be bit-equal
    (probed centroids, the probed lists themselves, L, selected ids), outputs
    within REL_TOL."""
    import torch
    import paper_2512_15550_amd as ck
    wl = bt.wl
    B, h, g, d = wl.batch, wl.h, wl.g, wl.d
    gl = ck.ctkvr_index_lists(idx)                     # [B][g][C_max][rho]
    Qc = [oracle.centroids_last_c(sq.q_tail, wl.centroids_of(sq.s)) for sq in bt.seqs]
    rng = np.random.Generator(np.random.Philox(seed))
    n_checked = 0
    for b, sq in enumerate(bt.seqs):
        Cb = wl.centroids_of(sq.s)
        n = max(1, n_list_samples // B)
        pairs = np.stack([rng.integers(0, g, n), rng.integers(0, Cb, n)], axis=1).astype(np.int32)
        built = oracle.build_lists(sq.K, Qc[b], wl.list_len, pairs=pairs)
        for (kv, j), row in zip(pairs, built):
            assert np.array_equal(gl[b, kv, j], row), f"list (seq {b}, kv {kv}, centroid {j}) differs from the oracle"
        n_checked += n
    say(f"  {n_checked} sampled lists bit-equal")
    out = torch.empty((B, h, d), dtype=torch.float32, device="cuda")
    lse = torch.empty((B, h), dtype=torch.float32, device="cuda")
    sel = torch.empty((B, g, wl.top_k), dtype=torch.int32, device="cuda")
    ncand = torch.empty((B, g), dtype=torch.int32, device="cuda")
    probe = torch.empty((B, g, wl.n_probe), dtype=torch.int32, device="cuda")
    worst, alphas = 0.0, []
    for st in steps:
        q = np.stack([sq.q_decode[st] for sq in bt.seqs])
        q_dev = to_dev(q, wl)
        ck.ctkvr_decode_step(idx, q_dev, db.k_pages, db.v_pages, db.block_table, out, lse, sel, ncand, probe)
        torch.cuda.synchronize()
        g_out, g_lse = out.cpu().numpy(), lse.cpu().numpy()
        g_sel, g_ncand, g_probe = sel.cpu().numpy(), ncand.cpu().numpy(), probe.cpu().numpy()
        for b, sq in enumerate(bt.seqs):
            tag = f"step {st} seq {b}"
            Cb = wl.centroids_of(sq.s)
            _, pr = oracle.recall(q[b], Qc[b], g, wl.n_probe)
            assert np.array_equal(g_probe[b], pr), f"{tag}: probed centroids differ"
            pairs = np.array([[kv, j] for kv in range(g) for j in pr[kv]], np.int32)
            built = oracle.build_lists(sq.K, Qc[b], wl.list_len, pairs=pairs)
            lst = np.zeros((g, Cb, wl.list_len), np.int32)
            for (kv, j), row in zip(pairs, built):
                assert np.array_equal(gl[b, kv, j], row), f"{tag}: probed list (kv {kv}, centroid {j}) differs"
                lst[kv, j] = row
            cand, nc, _, o_sel, o_out, o_lse = oracle.rerank_attend(q[b], sq.K, sq.V, lst, pr, wl.top_k)
            assert np.array_equal(g_ncand[b], nc), f"{tag}: L differs {g_ncand[b]} vs {nc}"
            assert np.array_equal(g_sel[b], o_sel), f"{tag}: selected ids differ ({int(np.sum(g_sel[b] != o_sel))} slots)"
            e = rel_err(g_out[b], o_out)
            assert e <= REL_TOL, f"{tag}: output relative error {e:.3e}"
            worst = max(worst, e)
            assert float(np.max(np.abs(g_lse[b] - o_lse) / np.maximum(1.0, np.abs(o_lse)))) <= 1e-4, f"{tag}: lse"
            alphas.append(float(np.mean(nc)) / (wl.n_probe * wl.list_len))
        say(f"  step {st}: all {B} sequences bit-equal, worst rel err so far {worst:.2e}")
    ck.ctkvr_index_check(idx)
    return {"max_rel_err": worst, "alpha": float(np.mean(alphas)), "lists_checked": n_checked}


def run_sampled_parity_next(bt: Batch, idx, db: DeviceBatch, steps: List[int], n_init: int = 0, n_local: int = 0,
                            update: bool = False, say=print) -> dict:
    """run_sampled_parity for the rows that follow the core path, at sizes where the oracle cannot
    afford the whole index: the resident window (index built with n_init / n_local; the step attends
    over the window too) and the dynamic centroid update after every step.  The oracle keeps the
    lists it knows -- those it has rebuilt because a step probed them, and those an update wrote --
    and every one of them must equal the GPU's list at the moment it is probed; after the last
    step the GPU's centroid table and all known lists are compared once more."""
    import torch
    import paper_2512_15550_amd as ck
    wl = bt.wl
    B, h, g, d = wl.batch, wl.h, wl.g, wl.d
    Qc = [oracle.centroids_last_c(sq.q_tail, wl.centroids_of(sq.s)).copy() for sq in bt.seqs]
    Qc0 = [q.copy() for q in Qc]                       # the prompt's centroids: what unknown lists are rebuilt from
    lists = [np.zeros((g, wl.centroids_of(sq.s), wl.list_len), np.int32) for sq in bt.seqs]
    known = [np.zeros((g, wl.centroids_of(sq.s)), bool) for sq in bt.seqs]
    out = torch.empty((B, h, d), dtype=torch.float32, device="cuda")
    lse = torch.empty((B, h), dtype=torch.float32, device="cuda")
    sel = torch.empty((B, g, wl.top_k), dtype=torch.int32, device="cuda")
    ncand = torch.empty((B, g), dtype=torch.int32, device="cuda")
    probe = torch.empty((B, g, wl.n_probe), dtype=torch.int32, device="cuda")
    worst, n_updates, n_built = 0.0, 0, 0
    gl = ck.ctkvr_index_lists(idx)
    for st in steps:
        q = np.stack([sq.q_decode[st] for sq in bt.seqs])
        q_dev = to_dev(q, wl)
        ck.ctkvr_decode_step(idx, q_dev, db.k_pages, db.v_pages, db.block_table, out, lse, sel, ncand, probe)
        torch.cuda.synchronize()
        g_out, g_lse = out.cpu().numpy(), lse.cpu().numpy()
        g_sel, g_ncand, g_probe = sel.cpu().numpy(), ncand.cpu().numpy(), probe.cpu().numpy()
        for b, sq in enumerate(bt.seqs):
            tag = f"step {st} seq {b}"
            _, pr = oracle.recall(q[b], Qc[b], g, wl.n_probe)
            assert np.array_equal(g_probe[b], pr), f"{tag}: probed centroids differ"
            need = np.array([[kv, j] for kv in range(g) for j in pr[kv] if not known[b][kv, j]], np.int32).reshape(-1, 2)
            if len(need):   # never probed before and not written by an update: still the prompt's list
                built = oracle.build_lists(sq.K, Qc0[b], wl.list_len, pairs=need, n_init=n_init, n_local=n_local)
                for (kv, j), row in zip(need, built):
                    lists[b][kv, j] = row
                    known[b][kv, j] = True
                n_built += len(need)
            for kv in range(g):
                for j in pr[kv]:
                    assert np.array_equal(gl[b, kv, j], lists[b][kv, j]), f"{tag}: probed list (kv {kv}, centroid {j}) differs"
            if n_init + n_local:
                r = oracle.decode_step_window(q[b], sq.K, sq.V, Qc[b], lists[b], wl.n_probe, wl.top_k, sq.s, n_init, n_local)
            else:
                r = oracle.decode_step(q[b], sq.K, sq.V, Qc[b], lists[b], wl.n_probe, wl.top_k)
            assert np.array_equal(g_ncand[b], r.ncand), f"{tag}: L differs {g_ncand[b]} vs {r.ncand}"
            assert np.array_equal(g_sel[b], r.sel), f"{tag}: selected ids differ ({int(np.sum(g_sel[b] != r.sel))} slots)"
            e = rel_err(g_out[b], r.out)
            assert e <= REL_TOL, f"{tag}: output relative error {e:.3e}"
            worst = max(worst, e)
            assert float(np.max(np.abs(g_lse[b] - r.lse) / np.maximum(1.0, np.abs(r.lse)))) <= 1e-4, f"{tag}: lse"
            if update:
                slot = oracle.centroid_update(q[b], Qc[b], lists[b], r, n_updates)
                known[b][:, slot] = True
        if update:
            ck.ctkvr_centroid_update(idx, q_dev)
            n_updates += 1
            gl = ck.ctkvr_index_lists(idx)
        say(f"  step {st}: all {B} sequences bit-equal, worst rel err so far {worst:.2e}, {n_built} lists rebuilt so far")
    if update:
        cen = ck.ctkvr_index_centroids(idx)
        for b, sq in enumerate(bt.seqs):
            Cb = wl.centroids_of(sq.s)
            ref = f32_to_bf16_bits(Qc[b]) if wl.dtype == "bf16" else Qc[b]
            assert np.array_equal(cen[b, :, :Cb], ref), f"centroid table of sequence {b} differs after {n_updates} updates"
            assert np.array_equal(gl[b, :, :Cb][known[b]], lists[b][known[b]]), f"known lists of sequence {b} differ at the end"
    ck.ctkvr_index_check(idx)
    return {"max_rel_err": worst, "lists_rebuilt": n_built, "updates": n_updates}
