"""GPU parity of the resident window (Algorithm 1 lines 5-6, Algorithm 2 lines 10-11): lists
built without the initial and local keys, attention over the window -- which grows with the
tokens decoded after the build -- merged with the sparse attention, against the oracle."""
import numpy as np
import pytest

import oracle
from ctkvr_inputs import Batch, gen_sequence, paginate, small_workload
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
    # name, dtype, h, g, ctx_lens (indexed prefix), C, C', rho, rho', n_init, n_local, grow, steps
    ("g4_bf16", "bf16", 8, 2, (1000,), 24, 4, 96, 64, 8, 40, 5, 4),
    ("g2_f32", "f32", 4, 2, (1500,), 20, 5, 100, 70, 4, 17, 3, 3),
    ("g8_long_window", "bf16", 8, 1, (2100,), 32, 6, 128, 100, 130, 700, 9, 3),   # several runs of 64 rows per block
    ("ragged_batch", "bf16", 8, 2, (700, 1333, 2049), 12, 4, 120, 90, 4, 64, 6, 4),
    ("grown_only", "bf16", 8, 2, (900,), 12, 3, 60, 50, 0, 0, 7, 4),              # no window at build: decoded tokens only
    ("init_only", "bf16", 4, 2, (640,), 8, 3, 64, 64, 16, 0, 0, 2),
]


def _random_window_case(seed):
    r = np.random.Generator(np.random.Philox(seed))
    g = int(r.choice([1, 2, 4]))
    G = int(r.choice([1, 2, 4, 8]))
    B = int(r.integers(1, 4))
    lens = tuple(int(x) for x in r.integers(200, 2500, size=B))
    smin = min(lens)
    n_init = int(r.integers(0, 40))
    n_local = int(r.integers(0, 120))
    C = int(r.integers(2, 30))
    n_probe = int(r.integers(1, C + 1))
    rho = int(r.integers(1, min(150, smin - n_init - n_local) + 1))
    top_k = int(r.integers(1, 200))
    grow = int(r.integers(0, 12))
    dtype = "f32" if r.random() < 0.25 else "bf16"
    return (f"rnd{seed}", dtype, G * g, g, lens, C, n_probe, rho, top_k, n_init, n_local, grow, 3)


CASES += [_random_window_case(s) for s in range(9100, 9108)]


def _setup(ck, case):
    name, dtype, h, g, lens, C, n_probe, rho, top_k, n_init, n_local, grow, steps = case
    wl = small_workload(name, dtype, h, g, lens, tuple(range(900, 900 + len(lens))), C, 0, n_probe, rho, top_k, steps)
    seqs = [gen_sequence(seed, s + grow, h, g, 128, C, steps, dtype) for seed, s in zip(wl.seeds, lens)]
    bt = Batch(wl=wl, seqs=seqs, paged=paginate(seqs, wl.page_size, wl.page_seed))
    db = H.device_batch(bt)
    db.ctx_lens = np.asarray(lens, np.int32)          # the index covers the prefix only
    Qc = [oracle.centroids_last_c(sq.q_tail, C) for sq in seqs]
    lists = [oracle.build_lists(sq.K[:, :s], q, rho, n_init=n_init, n_local=n_local) for sq, s, q in zip(seqs, lens, Qc)]
    return wl, bt, db, Qc, lists


XCD_CASES = [
    ("units_8", "bf16", 32, 8, (1500,), 24, 4, 96, 64, 8, 100, 5, 3),
    ("units_16_ragged", "bf16", 16, 8, (900, 1700), 16, 4, 80, 60, 4, 64, 3, 3),
]


@pytest.mark.parametrize("one_xcd", [0, 1])
@pytest.mark.parametrize("case", XCD_CASES, ids=[c[0] for c in XCD_CASES])
def test_window_with_units_spread_over_the_xcds_or_each_on_one(ck, case, one_xcd, monkeypatch):
    """A multiple of 8 (sequence, KV head) units: both block-to-unit mappings forced in turn, the window's blocks
    riding in the scoring launch."""
    monkeypatch.setenv("CTKVR_XCD_UNITS", str(one_xcd))
    test_window_build_and_decode_match_the_oracle(ck, case)


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_window_build_and_decode_match_the_oracle(ck, case):
    import torch
    name, dtype, h, g, lens, C, n_probe, rho, top_k, n_init, n_local, grow, steps = case
    print(f"[window {name}] generating", flush=True)
    wl, bt, db, Qc, lists = _setup(ck, case)
    print(f"[window {name}] building on the GPU", flush=True)
    idx = ck.ctkvr_build_index(H.params_of(wl, n_init=n_init, n_local=n_local), db.q_prefill, db.cu_seqlens, True,
                               db.k_pages, db.block_table, db.ctx_lens)
    got = ck.ctkvr_index_lists(idx)
    for b in range(wl.batch):
        assert np.array_equal(got[b], lists[b]), f"lists of sequence {b} differ"
        if n_init + n_local:
            assert got[b].min() >= n_init and got[b].max() < lens[b] - n_local
    B, d = wl.batch, wl.d
    out = torch.empty((B, h, d), dtype=torch.float32, device="cuda")
    lse = torch.empty((B, h), dtype=torch.float32, device="cuda")
    sel = torch.empty((B, g, top_k), dtype=torch.int32, device="cuda")
    ncand = torch.empty((B, g), dtype=torch.int32, device="cuda")
    probe = torch.empty((B, g, n_probe), dtype=torch.int32, device="cuda")
    worst = 0.0
    for st in range(steps):
        cur = np.array([s + min(st + 1, grow) for s in lens], np.int32)
        q = np.stack([sq.q_decode[st] for sq in bt.seqs])
        print(f"[window {name}] step {st} cur {cur.tolist()}", flush=True)
        if grow == 0 and st == steps - 1:      # the plain entry point on a window index: cur = ctx_len
            ck.ctkvr_decode_step(idx, H.to_dev(q, wl), db.k_pages, db.v_pages, db.block_table, out, lse, sel, ncand, probe)
        else:
            ck.ctkvr_decode_step_window(idx, H.to_dev(q, wl), db.k_pages, db.v_pages, db.block_table,
                                        torch.from_numpy(cur).cuda(), out, lse, sel, ncand, probe)
        torch.cuda.synchronize()
        g_out, g_lse, g_sel = out.cpu().numpy(), lse.cpu().numpy(), sel.cpu().numpy()
        g_ncand, g_probe = ncand.cpu().numpy(), probe.cpu().numpy()
        for b, sq in enumerate(bt.seqs):
            r = oracle.decode_step_window(q[b], sq.K[:, :cur[b]], sq.V[:, :cur[b]], Qc[b], lists[b], n_probe, top_k,
                                          lens[b], n_init, n_local)
            tag = f"step {st} seq {b}"
            assert np.array_equal(g_probe[b], r.probe), f"{tag}: probed centroids differ"
            assert np.array_equal(g_ncand[b], r.ncand), f"{tag}: L differs"
            assert np.array_equal(g_sel[b], r.sel), f"{tag}: selected ids differ"
            e = H.rel_err(g_out[b], r.out)
            assert e <= H.REL_TOL, f"{tag}: output relative error {e:.3e}"
            el = float(np.max(np.abs(g_lse[b] - r.lse) / np.maximum(1.0, np.abs(r.lse))))
            assert el <= 1e-4, f"{tag}: lse error {el:.3e}"
            worst = max(worst, e)
    print(f"[window {name}] ok, max rel err {worst:.2e}", flush=True)
    ck.ctkvr_free(idx)


def test_window_leaves_too_few_keys_is_an_error(ck):
    case = ("err", "bf16", 4, 2, (300,), 8, 2, 32, 16, 200, 80, 0, 1)
    wl, bt, db, Qc, lists = None, None, None, None, None
    name, dtype, h, g, lens, C, n_probe, rho, top_k, n_init, n_local, grow, steps = case
    wl = small_workload(name, dtype, h, g, lens, (1,), C, 0, n_probe, rho, top_k, steps)
    seqs = [gen_sequence(1, lens[0], h, g, 128, C, steps, dtype)]
    bt = Batch(wl=wl, seqs=seqs, paged=paginate(seqs, wl.page_size, wl.page_seed))
    db = H.device_batch(bt)
    with pytest.raises(ck.CtkvrError) as ei:
        ck.ctkvr_build_index(H.params_of(wl, n_init=n_init, n_local=n_local), db.q_prefill, db.cu_seqlens, True,
                             db.k_pages, db.block_table, db.ctx_lens)
    assert ei.value.code == -1
