"""A decode step captured in a HIP graph must give on every replay what the eager launches give:
the step allocates nothing, records no memset and keeps its counters on the device."""
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


@pytest.mark.parametrize("window", [False, True], ids=["plain", "window"])
def test_graph_replays_equal_eager_steps(ck, window):
    import torch
    n_steps = 4
    wl = small_workload("graph", "bf16", 8, 2, (3000, 1700), (810, 811), 32, 0, 5, 128, 96, n_steps)
    bt = gen_batch(wl)
    db = H.device_batch(bt)
    kw = dict(n_init=8, n_local=100) if window else {}
    idx = ck.ctkvr_build_index(H.params_of(wl, **kw), db.q_prefill, db.cu_seqlens, True, db.k_pages, db.block_table,
                               db.ctx_lens)
    B, h, g, d = wl.batch, wl.h, wl.g, wl.d
    qs = [H.to_dev(np.stack([sq.q_decode[i] for sq in bt.seqs]), wl) for i in range(n_steps)]
    outs = [torch.zeros((B, h, d), dtype=torch.float32, device="cuda") for _ in range(n_steps)]
    sels = [torch.zeros((B, g, wl.top_k), dtype=torch.int32, device="cuda") for _ in range(n_steps)]

    def steps():
        for i in range(n_steps):
            ck.ctkvr_decode_step(idx, qs[i], db.k_pages, db.v_pages, db.block_table, outs[i], out_sel=sels[i])

    steps()
    torch.cuda.synchronize()
    ref_out = [o.clone() for o in outs]
    ref_sel = [s.clone() for s in sels]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            steps()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for rep in range(4):
        for o, s in zip(outs, sels):
            o.zero_()
            s.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for i in range(n_steps):
            assert torch.equal(sels[i], ref_sel[i]), f"replay {rep} step {i}: selected ids differ from the eager run"
            assert torch.equal(outs[i], ref_out[i]), f"replay {rep} step {i}: output differs from the eager run"
        # eager work of the program's own between replays: a step with another query order
        ck.ctkvr_decode_step(idx, qs[(rep + 1) % n_steps], db.k_pages, db.v_pages, db.block_table, outs[0])
        torch.cuda.synchronize()
        assert torch.equal(outs[0], ref_out[(rep + 1) % n_steps])
    ck.ctkvr_free(idx)


def test_graph_with_centroid_updates_tracks_an_eager_twin(ck):
    """Steps followed by the dynamic centroid update, captured once and replayed: the FIFO position
    lives on the device, so every replay continues where the last one stopped -- exactly like a
    second, eagerly driven index that is given the same sequence of steps."""
    import torch
    n_steps = 3
    wl = small_workload("graph_dcu", "bf16", 8, 2, (2500,), (820,), 6, 0, 3, 64, 64, n_steps)
    bt = gen_batch(wl)
    db = H.device_batch(bt)

    def build():
        return ck.ctkvr_build_index(H.params_of(wl), db.q_prefill, db.cu_seqlens, True, db.k_pages, db.block_table,
                                    db.ctx_lens)

    eager, graphed = build(), build()
    B, h, g, d = wl.batch, wl.h, wl.g, wl.d
    qs = [H.to_dev(np.stack([sq.q_decode[i] for sq in bt.seqs]), wl) for i in range(n_steps)]
    outs_e = [torch.zeros((B, h, d), dtype=torch.float32, device="cuda") for _ in range(n_steps)]
    outs_g = [torch.zeros((B, h, d), dtype=torch.float32, device="cuda") for _ in range(n_steps)]

    def steps(idx, outs):
        for i in range(n_steps):
            ck.ctkvr_decode_step(idx, qs[i], db.k_pages, db.v_pages, db.block_table, outs[i])
            ck.ctkvr_centroid_update(idx, qs[i])

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            steps(graphed, outs_g)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for rep in range(3):      # 9 updates on 6 slots: the FIFO wraps
        steps(eager, outs_e)
        graph.replay()
        torch.cuda.synchronize()
        for i in range(n_steps):
            assert torch.equal(outs_g[i], outs_e[i]), f"replay {rep} step {i}: output differs from the eager twin"
        assert np.array_equal(ck.ctkvr_index_lists(graphed), ck.ctkvr_index_lists(eager)), f"replay {rep}: lists differ"
        assert np.array_equal(ck.ctkvr_index_centroids(graphed), ck.ctkvr_index_centroids(eager))
    ck.ctkvr_free(eager)
    ck.ctkvr_free(graphed)
