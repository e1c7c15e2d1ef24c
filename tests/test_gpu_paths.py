"""The two ways a decode step is launched -- one launch per stage, or the whole step as one launch
whose blocks walk the stages together (Algorithm 2 lines 1-9 either way) -- must give the same
integers bit for bit, both equal to the oracle's, and outputs within the tolerance; the single
launch must give the same bits in every run (no atomic decides an order) and report no expired wait."""
import numpy as np
import pytest

from ctkvr_inputs import gen_batch, small_workload, workload
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
    # name, dtype, h, g, ctx_lens, seeds, C, div, C', rho, rho', steps
    ("one_unit", "bf16", 4, 1, (5000,), (501,), 64, 0, 8, 200, 150, 3),
    ("three_units_g1", "bf16", 3, 3, (2000,), (502,), 40, 0, 6, 100, 64, 2),          # units not a multiple of 8
    ("eight_units", "bf16", 16, 4, (3000, 1111), (503, 504), 48, 0, 6, 128, 100, 2),  # a unit's blocks on one XCD
    ("g8_f32", "f32", 8, 1, (2600,), (505,), 30, 0, 5, 90, 80, 2),
    ("ragged_div", "bf16", 8, 2, (900, 4000, 2500), (506, 507, 508), 0, 50, 4, 96, 64, 2),
    ("many_units", "bf16", 8, 8, tuple([700] * 9), tuple(range(510, 519)), 16, 0, 4, 64, 48, 1),   # 72 units, 3 blocks each
    ("more_picks_than_recalled", "bf16", 8, 2, (1500,), (520,), 24, 0, 3, 40, 500, 2),  # rho' >= L: everything is picked
    ("top1", "bf16", 8, 2, (1500,), (521,), 24, 0, 4, 64, 1, 2),
    ("rho_not_multiple_of_4", "bf16", 8, 2, (1800,), (522,), 24, 0, 5, 77, 50, 2),
    ("many_centroids", "bf16", 8, 2, (6000,), (523,), 2500, 0, 40, 64, 128, 2),        # 8 keys per thread in the probe select
    ("few_probes", "bf16", 8, 2, (5000,), (524,), 1500, 0, 4, 160, 100, 2),            # the extraction route, 2 keys per thread
    ("two_chunks", "bf16", 8, 8, tuple([20000] * 8), tuple(range(560, 568)), 64, 0, 40, 1000, 1000, 1),   # 64 units, 4 blocks each: shares above 4096 ranks
]


def _run(ck, case, path):
    name, dtype, h, g, lens, seeds, C, div, n_probe, rho, top_k, steps = case
    wl = small_workload(name, dtype, h, g, lens, seeds, C, div, n_probe, rho, top_k, steps)
    bt = gen_batch(wl)
    db = H.device_batch(bt)
    oi = H.oracle_index(bt)
    cen, lst = oi.padded(wl)
    idx = ck.ctkvr_index_load(H.params_of(wl), db.ctx_lens, cen, lst)
    ck.ctkvr_index_set_decode_path(idx, path)
    assert ck.ctkvr_index_decode_path(idx) == path
    st = H.run_decode_parity(bt, oi, idx, db)
    ck.ctkvr_index_check(idx)
    ck.ctkvr_free(idx)
    return st


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_single_launch_step_matches_the_oracle(ck, case):
    print(f"[paths {case[0]}] single launch", flush=True)
    st = _run(ck, case, ck.PATH_FUSED)
    print(f"[paths {case[0]}] ok {st}", flush=True)


@pytest.mark.parametrize("case", CASES[:5], ids=[c[0] for c in CASES[:5]])
def test_staged_step_matches_the_oracle(ck, case):
    print(f"[paths {case[0]}] staged", flush=True)
    _run(ck, case, ck.PATH_STAGED)


SPLIT_CASES = CASES[:5] + [CASES[5], CASES[6], CASES[11]] + [
    # recalled ids far apart (L / s about 1 %): a block's ranks spread over several passes of 64 bitmap words
    ("sparse_recall", "bf16", 8, 2, (60000,), (530,), 32, 0, 2, 300, 100, 2),
    ("ragged_sparse", "bf16", 8, 2, (40000, 3000, 17000), (531, 532, 533), 0, 200, 3, 150, 100, 2),
]


@pytest.mark.parametrize("by_rank", [0, 1])
@pytest.mark.parametrize("case", SPLIT_CASES, ids=[c[0] for c in SPLIT_CASES])
def test_both_ways_of_splitting_the_recalled_ids_over_blocks_match_the_oracle(ck, case, by_rank, monkeypatch):
    """The scoring launch gives a unit's blocks equal id ranges or equal numbers of ranks, chosen per batch; here each
    is forced in turn (read when the index is created)."""
    monkeypatch.setenv("CTKVR_SCORE_BY_RANK", str(by_rank))
    print(f"[paths {case[0]}] split by {'rank' if by_rank else 'id range'}", flush=True)
    _run(ck, case, ck.PATH_STAGED)


XCD_CASES = [
    # (sequence, KV head) units a multiple of 8: 8, 16 (ragged), 8 with a group of one head
    ("xcd_8_units", "bf16", 32, 8, (9000,), (560,), 128, 0, 16, 256, 256, 3),
    ("xcd_16_units_ragged", "bf16", 16, 8, (5000, 2100), (561, 562), 0, 100, 6, 120, 90, 3),
    ("xcd_8_units_g1", "f32", 4, 4, (1500, 3000), (563, 564), 24, 0, 5, 100, 70, 2),
]


@pytest.mark.parametrize("one_xcd", [0, 1])
@pytest.mark.parametrize("case", XCD_CASES, ids=[c[0] for c in XCD_CASES])
def test_units_spread_over_the_xcds_or_each_on_one_match_the_oracle(ck, case, one_xcd, monkeypatch):
    """With a multiple of 8 units the blocks of a unit can be given linear ids that all land on one XCD, in every
    kernel of a step (chosen for small batches); here both mappings are forced in turn (read when the index is
    created).  (The same with the resident window's blocks in the scoring launch: tests/test_gpu_window.py.)"""
    monkeypatch.setenv("CTKVR_XCD_UNITS", str(one_xcd))
    print(f"[paths {case[0]}] units {'each on one XCD' if one_xcd else 'spread'}", flush=True)
    _run(ck, case, ck.PATH_STAGED)


@pytest.mark.parametrize("merged", [0, 1])
@pytest.mark.parametrize("case", SPLIT_CASES, ids=[c[0] for c in SPLIT_CASES])
def test_key_histogram_and_classification_as_one_launch_or_two_match_the_oracle(ck, case, merged, monkeypatch):
    """Small batches take the ranking keys' histogram and the classification pass in one launch (every block takes its
    unit's whole histogram itself), large ones in two chip-wide launches; here each form is forced in turn."""
    monkeypatch.setenv("CTKVR_KEYCLASS", str(merged))
    print(f"[paths {case[0]}] keys + classification in {'one launch' if merged else 'two launches'}", flush=True)
    _run(ck, case, ck.PATH_STAGED)


def test_exact_ties_through_the_single_launch(ck):
    """Duplicated keys and centroids (planted exact ties) and lattice inputs crowd the deciding
    bucket: the unit's first block then selects alone (the histogram-free route)."""
    import torch
    from ctkvr_inputs import Batch, gen_lattice_sequence, paginate
    wl = small_workload("paths_lattice", "bf16", 8, 2, (3000,), (530,), 32, 0, 6, 150, 100, 2)
    sq = gen_lattice_sequence(530, 3000, 8, 2, 128, 32, 2)
    sq.K[:, 1000:1400] = sq.K[:, 100:500]          # exact duplicates: equal scores, lowest id wins
    bt = Batch(wl=wl, seqs=[sq], paged=paginate([sq], wl.page_size, 530))
    db = H.device_batch(bt)
    oi = H.oracle_index(bt)
    cen, lst = oi.padded(wl)
    for path in (ck.PATH_FUSED, ck.PATH_STAGED):
        idx = ck.ctkvr_index_load(H.params_of(wl), db.ctx_lens, cen, lst)
        ck.ctkvr_index_set_decode_path(idx, path)
        H.run_decode_parity(bt, oi, idx, db)
        ck.ctkvr_index_check(idx)
        ck.ctkvr_free(idx)


def test_single_launch_gives_the_same_bits_every_run_and_under_graph_replay(ck):
    import torch
    wl = small_workload("paths_repeat", "bf16", 32, 8, (9000,), (540,), 128, 0, 16, 256, 256, 3)
    bt = gen_batch(wl)
    db = H.device_batch(bt)
    idx = ck.ctkvr_build_index(H.params_of(wl), db.q_prefill, db.cu_seqlens, True, db.k_pages, db.block_table, db.ctx_lens)
    ck.ctkvr_index_set_decode_path(idx, ck.PATH_FUSED)
    B, h, g, d = wl.batch, wl.h, wl.g, wl.d
    qs = [H.to_dev(np.stack([sq.q_decode[i] for sq in bt.seqs]), wl) for i in range(3)]
    outs = [torch.zeros((B, h, d), dtype=torch.float32, device="cuda") for _ in range(3)]
    sels = [torch.zeros((B, g, wl.top_k), dtype=torch.int32, device="cuda") for _ in range(3)]

    def steps():
        for i in range(3):
            ck.ctkvr_decode_step(idx, qs[i], db.k_pages, db.v_pages, db.block_table, outs[i], out_sel=sels[i])

    steps()
    torch.cuda.synchronize()
    ref_out, ref_sel = [o.clone() for o in outs], [s.clone() for s in sels]
    for rep in range(5):
        steps()
        torch.cuda.synchronize()
        for i in range(3):
            assert torch.equal(outs[i], ref_out[i]) and torch.equal(sels[i], ref_sel[i]), f"run {rep} step {i} differs"
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            steps()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for rep in range(4):
        for o in outs:
            o.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for i in range(3):
            assert torch.equal(outs[i], ref_out[i]) and torch.equal(sels[i], ref_sel[i]), f"replay {rep} step {i} differs"
        ck.ctkvr_decode_step(idx, qs[rep % 3], db.k_pages, db.v_pages, db.block_table, outs[0])   # eager work in between
        torch.cuda.synchronize()
        assert torch.equal(outs[0], ref_out[rep % 3])
    # and the staged path selects the same keys
    ck.ctkvr_index_set_decode_path(idx, ck.PATH_STAGED)
    steps()
    torch.cuda.synchronize()
    for i in range(3):
        assert torch.equal(sels[i], ref_sel[i])
        assert float((outs[i] - ref_out[i]).abs().max()) <= 1e-4 * float(ref_out[i].abs().max())
    ck.ctkvr_index_check(idx)
    ck.ctkvr_free(idx)


def test_path_selection_errors(ck):
    wl = small_workload("paths_err", "bf16", 4, 2, (300,), (550,), 8, 0, 2, 32, 16, 1)
    bt = gen_batch(wl)
    db = H.device_batch(bt)
    idx = ck.ctkvr_build_index(H.params_of(wl), db.q_prefill, db.cu_seqlens, True, db.k_pages, db.block_table, db.ctx_lens)
    with pytest.raises(ck.CtkvrError):
        ck.ctkvr_index_set_decode_path(idx, 7)
    ck.ctkvr_index_set_decode_path(idx, ck.PATH_STAGED)
    assert ck.ctkvr_index_decode_path(idx) == ck.PATH_STAGED
    ck.ctkvr_index_set_decode_path(idx, ck.PATH_AUTO)
    assert ck.ctkvr_index_decode_path(idx) == ck.PATH_STAGED      # the default: one launch per stage
    ck.ctkvr_index_set_decode_path(idx, ck.PATH_FUSED)            # 2 units: the single launch fits
    assert ck.ctkvr_index_decode_path(idx) == ck.PATH_FUSED
    assert ck.ctkvr_measure_dispatch_floor(50) > 0.0
    ck.ctkvr_free(idx)


@pytest.mark.parametrize("groups", [2, 3, 5])
def test_groups_of_sequences_side_by_side_match_the_oracle_eager_and_replayed(ck, groups, monkeypatch):
    """The sequences of a batch split into groups whose steps are issued side by side (forked from and joined
    into the caller's stream): same integers as the oracle, same bits as the unsplit step, also when the
    forked step is captured into a graph and replayed."""
    import torch
    wl = small_workload("paths_groups", "bf16", 8, 2, (900, 2500, 1300, 3100, 700), (570, 571, 572, 573, 574), 0, 50, 4, 96, 64, 3)
    bt = gen_batch(wl)
    db = H.device_batch(bt)
    oi = H.oracle_index(bt)
    cen, lst = oi.padded(wl)
    monkeypatch.setenv("CTKVR_DECODE_GROUPS", "1")
    one = ck.ctkvr_index_load(H.params_of(wl), db.ctx_lens, cen, lst)
    monkeypatch.setenv("CTKVR_DECODE_GROUPS", str(groups))
    idx = ck.ctkvr_index_load(H.params_of(wl), db.ctx_lens, cen, lst)
    monkeypatch.delenv("CTKVR_DECODE_GROUPS")
    H.run_decode_parity(bt, oi, idx, db)
    B, h, g, d = wl.batch, wl.h, wl.g, wl.d
    qs = [H.to_dev(np.stack([sq.q_decode[i] for sq in bt.seqs]), wl) for i in range(3)]
    outs = [torch.zeros((B, h, d), dtype=torch.float32, device="cuda") for _ in range(3)]
    sels = [torch.zeros((B, g, wl.top_k), dtype=torch.int32, device="cuda") for _ in range(3)]
    ref = torch.zeros((B, h, d), dtype=torch.float32, device="cuda")

    def steps():
        for i in range(3):
            ck.ctkvr_decode_step(idx, qs[i], db.k_pages, db.v_pages, db.block_table, outs[i], out_sel=sels[i])

    steps()
    torch.cuda.synchronize()
    ref_out, ref_sel = [o.clone() for o in outs], [s.clone() for s in sels]
    for i in range(3):
        ck.ctkvr_decode_step(one, qs[i], db.k_pages, db.v_pages, db.block_table, ref)
        torch.cuda.synchronize()
        assert torch.equal(ref, ref_out[i]), f"step {i}: the split step differs from the unsplit one"
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            steps()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for rep in range(4):
        for o in outs:
            o.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for i in range(3):
            assert torch.equal(outs[i], ref_out[i]) and torch.equal(sels[i], ref_sel[i]), f"replay {rep} step {i} differs"
        ck.ctkvr_decode_step(idx, qs[rep % 3], db.k_pages, db.v_pages, db.block_table, outs[0])   # eager work in between
        torch.cuda.synchronize()
        assert torch.equal(outs[0], ref_out[rep % 3])
    ck.ctkvr_free(idx)
    ck.ctkvr_free(one)
