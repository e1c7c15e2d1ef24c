"""GPU parity of the dynamic centroid update (Algorithm 2 line 12): decode steps with an
update after each, on the GPU through the C ABI and in the oracle, from the same index.
Every step's integers must stay bit-equal (so a wrong slot, list or centroid shows up in the
next step's probe), and at the end the two indexes must hold the same lists and centroids."""
import numpy as np
import pytest

from ctkvr_inputs import gen_batch, small_workload
from tests import harness as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ck():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2512_15550_amd as ck
    ck.load_library()
    return ck


CASES = [
    # name, dtype, h, g, ctx_lens, C, div, C', rho, rho', steps
    ("same_budget", "bf16", 8, 2, (1000,), 24, 0, 4, 64, 64, 6),
    ("wraps_around", "bf16", 4, 2, (800,), 5, 0, 2, 48, 48, 12),        # more updates than slots
    ("list_longer", "bf16", 8, 2, (1500,), 16, 0, 4, 120, 50, 5),       # rho > rho': second ranking with budget rho
    ("list_shorter", "f32", 4, 2, (1200,), 12, 0, 3, 40, 90, 5),        # rho < rho'
    ("ragged_batch", "bf16", 8, 2, (700, 1333, 2049), 0, 100, 3, 80, 80, 9),   # C_i = 7, 13, 20: slots differ per sequence
    ("multi_tile", "bf16", 16, 4, (9000,), 96, 0, 12, 700, 300, 3),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_update_keeps_gpu_and_oracle_indexes_equal(ck, case):
    name, dtype, h, g, lens, C, div, n_probe, rho, top_k, steps = case
    wl = small_workload(name, dtype, h, g, lens, tuple(range(700, 700 + len(lens))), C, div, n_probe, rho, top_k, steps)
    print(f"[dcu {name}] generating", flush=True)
    bt = gen_batch(wl)
    oi = H.oracle_index(bt)
    db = H.device_batch(bt)
    cen, lst = oi.padded(wl)
    idx = ck.ctkvr_index_load(H.params_of(wl), db.ctx_lens, cen, lst)
    print(f"[dcu {name}] {steps} steps with update", flush=True)
    st = H.run_decode_parity(bt, oi, idx, db, update=True)
    ref_cen, ref_lst = oi.padded(wl)
    got_lst, got_cen = ck.ctkvr_index_lists(idx), ck.ctkvr_index_centroids(idx)
    for b, sq in enumerate(bt.seqs):
        Cb = wl.centroids_of(sq.s)
        assert np.array_equal(got_lst[b, :, :Cb], ref_lst[b, :, :Cb]), f"lists of sequence {b} differ after the updates"
        assert np.array_equal(got_cen[b, :, :Cb], ref_cen[b, :, :Cb]), f"centroids of sequence {b} differ after the updates"
    assert not np.array_equal(ref_lst, lst), "the updates changed nothing"
    print(f"[dcu {name}] ok {st}", flush=True)
    ck.ctkvr_free(idx)


def test_update_at_full_size_32k(ck):
    """cfg2 (32K context, C = 512, C' = 32, rho = rho' = 1024) in the launch shape bench.py times."""
    from ctkvr_inputs import workload
    wl = workload("cfg2")
    print("[dcu cfg2] generating", flush=True)
    bt = gen_batch(wl, n_decode=6)
    oi = H.oracle_index(bt)
    db = H.device_batch(bt)
    cen, lst = oi.padded(wl)
    idx = ck.ctkvr_index_load(H.params_of(wl), db.ctx_lens, cen, lst)
    print("[dcu cfg2] 6 steps with update", flush=True)
    st = H.run_decode_parity(bt, oi, idx, db, update=True, check_candidates=False)
    ref_cen, ref_lst = oi.padded(wl)
    assert np.array_equal(ck.ctkvr_index_lists(idx), ref_lst)
    assert np.array_equal(ck.ctkvr_index_centroids(idx), ref_cen)
    print(f"[dcu cfg2] ok {st}", flush=True)
    ck.ctkvr_free(idx)


def test_update_needs_a_decode_step_first(ck):
    import torch
    wl = small_workload("dcu_err", "bf16", 4, 2, (300,), (1,), 8, 0, 2, 32, 16, 1)
    bt = gen_batch(wl)
    oi = H.oracle_index(bt)
    db = H.device_batch(bt)
    cen, lst = oi.padded(wl)
    idx = ck.ctkvr_index_load(H.params_of(wl), db.ctx_lens, cen, lst)
    q = H.to_dev(np.stack([sq.q_decode[0] for sq in bt.seqs]), wl)
    with pytest.raises(ck.CtkvrError) as ei:
        ck.ctkvr_centroid_update(idx, q)
    assert ei.value.code == -1
    out = torch.empty((wl.batch, wl.h, wl.d), dtype=torch.float32, device="cuda")
    ck.ctkvr_decode_step(idx, q, db.k_pages, db.v_pages, db.block_table, out)
    ck.ctkvr_centroid_update(idx, q)
    with pytest.raises(ck.CtkvrError):
        ck.ctkvr_centroid_update(idx, q)     # one update per step
    torch.cuda.synchronize()
    ck.ctkvr_free(idx)
