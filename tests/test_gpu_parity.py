"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Integers (probed centroids, recalled ids, selected ids,
list contents) must be bit-equal; attention outputs within 2e-3 relative."""
import numpy as np
import pytest

import oracle
from ctkvr_inputs import gen_batch, gen_lattice_sequence, paginate, small_workload, workload, Batch
from tests import harness as H
from tests.bands import key_band

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ck():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2512_15550_amd as ck
    ck.load_library()
    return ck


def _say(msg):
    print(msg, flush=True)


def test_both_forms_of_the_fixed_point_exponential_agree_on_every_input(ck):
    # the form written after the definition and the straight-line form the kernels use: all 1.1e9 fp32 values in [-32, 0]
    assert ck.ctkvr_selftest_exp() == 0


SMALL = [
    # name, dtype, h, g, ctx_lens, C, div, C', rho, rho'
    ("g4_bf16", "bf16", 8, 2, (1000,), 24, 0, 4, 96, 64),
    ("g1_bf16", "bf16", 2, 2, (777,), 16, 0, 3, 80, 50),
    ("g2_f32", "f32", 4, 2, (1500,), 20, 0, 5, 100, 70),
    ("g8_bf16", "bf16", 8, 1, (2100,), 32, 0, 6, 128, 100),
    ("ragged_batch", "bf16", 8, 2, (700, 1333, 2049, 5000), 0, 50, 4, 120, 90),
    ("rerank_off", "bf16", 8, 2, (900,), 12, 0, 3, 60, 180),          # rho' >= L: every recalled key is kept
    ("all_probed", "bf16", 4, 1, (640,), 8, 0, 8, 640, 640),           # C' = C, rho = s: dense attention
    ("multi_tile", "bf16", 16, 4, (9000,), 96, 0, 12, 700, 300),       # L spans many 256-id tiles, ragged tail
]


@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
def test_decode_matches_oracle_on_shared_index(ck, case):
    name, dtype, h, g, lens, C, div, n_probe, rho, top_k = case
    wl = small_workload(name, dtype, h, g, lens, tuple(range(200, 200 + len(lens))), C, div, n_probe, rho, top_k, 3)
    _say(f"[case {name}] generating")
    bt = gen_batch(wl)
    oi = H.oracle_index(bt)
    db = H.device_batch(bt)
    cen, lst = oi.padded(wl)
    idx = ck.ctkvr_index_load(H.params_of(wl), db.ctx_lens, cen, lst)
    _say(f"[case {name}] decode parity")
    st = H.run_decode_parity(bt, oi, idx, db)
    _say(f"[case {name}] ok {st}")
    ck.ctkvr_free(idx)


EDGE = [
    # name, dtype, h, g, ctx_lens, C, C', rho, rho'
    ("s33_one_pick", "bf16", 2, 1, (33,), 2, 1, 5, 1),
    ("single_head", "f32", 1, 1, (64,), 3, 2, 9, 4),
    ("every_query_a_centroid", "bf16", 4, 2, (100,), 100, 7, 10, 10),
    ("list_is_everything", "bf16", 8, 2, (257,), 4, 1, 257, 100),
    ("tiny_and_long", "bf16", 8, 2, (17, 4097), 5, 2, 16, 12),
]


@pytest.mark.parametrize("case", EDGE, ids=[c[0] for c in EDGE])
def test_edge_shapes(ck, case):
    name, dtype, h, g, lens, C, n_probe, rho, top_k = case
    wl = small_workload(name, dtype, h, g, lens, tuple(range(260, 260 + len(lens))), C, 0, n_probe, rho, top_k, 2)
    bt = gen_batch(wl)
    oi = H.oracle_index(bt)
    db = H.device_batch(bt)
    idx = ck.ctkvr_build_index(H.params_of(wl), db.q_prefill, db.cu_seqlens, True, db.k_pages, db.block_table,
                               db.ctx_lens)
    for b in range(wl.batch):
        assert np.array_equal(ck.ctkvr_index_lists(idx)[b], oi.lists[b])
    st = H.run_decode_parity(bt, oi, idx, db)
    _say(f"[edge {name}] ok {st}")
    ck.ctkvr_free(idx)


def _random_case(seed):
    """A valid small configuration drawn from a seed: shapes, budgets and batch all vary."""
    r = np.random.Generator(np.random.Philox(seed))
    g = int(r.choice([1, 2, 4]))
    G = int(r.choice([1, 2, 4, 8]))
    B = int(r.integers(1, 4))
    lens = tuple(int(x) for x in r.integers(40, 3000, size=B))
    smin = min(lens)
    C = int(r.integers(1, min(40, smin) + 1))
    n_probe = int(r.integers(1, C + 1))
    rho = int(r.integers(1, min(200, smin) + 1))
    top_k = int(r.integers(1, 300))
    dtype = "f32" if r.random() < 0.25 else "bf16"
    page = int(r.choice([8, 16, 32]))
    return dtype, G * g, g, lens, C, n_probe, rho, top_k, page


@pytest.mark.parametrize("seed", list(range(9000, 9016)))
def test_random_shapes(ck, seed):
    dtype, h, g, lens, C, n_probe, rho, top_k, page = _random_case(seed)
    _say(f"[random {seed}] {dtype} h={h} g={g} lens={lens} C={C} C'={n_probe} rho={rho} rho'={top_k} page={page}")
    wl = small_workload(f"rnd{seed}", dtype, h, g, lens, tuple(range(seed * 10, seed * 10 + len(lens))), C, 0, n_probe, rho,
                        top_k, 2, page_size=page)
    bt = gen_batch(wl)
    oi = H.oracle_index(bt)
    db = H.device_batch(bt)
    idx = ck.ctkvr_build_index(H.params_of(wl), db.q_prefill, db.cu_seqlens, True, db.k_pages, db.block_table,
                               db.ctx_lens)
    got = ck.ctkvr_index_lists(idx)
    for b in range(wl.batch):
        assert np.array_equal(got[b], oi.lists[b]), f"lists of sequence {b} differ"
    st = H.run_decode_parity(bt, oi, idx, db, update=(seed % 2 == 0))
    _say(f"[random {seed}] ok {st}")
    ck.ctkvr_free(idx)


@pytest.mark.parametrize("page_size", [1, 4, 64, 256])
def test_other_page_sizes(ck, page_size):
    """The KV layout is a parameter: pages of 1 token (every row its own block-table entry), of a
    few tokens, and pages larger than a 32-id bitmap word."""
    wl = small_workload(f"page{page_size}", "bf16", 8, 2, (2300, 999), (250, 251), 20, 0, 4, 100, 64, 2,
                        page_size=page_size)
    bt = gen_batch(wl)
    oi = H.oracle_index(bt)
    db = H.device_batch(bt)
    idx = ck.ctkvr_build_index(H.params_of(wl), db.q_prefill, db.cu_seqlens, True, db.k_pages, db.block_table,
                               db.ctx_lens)
    for b in range(wl.batch):
        assert np.array_equal(ck.ctkvr_index_lists(idx)[b], oi.lists[b])
    st = H.run_decode_parity(bt, oi, idx, db)
    _say(f"[page {page_size}] ok {st}")
    ck.ctkvr_free(idx)


@pytest.mark.parametrize("case", SMALL[:5], ids=[c[0] for c in SMALL[:5]])
def test_exact_build_matches_oracle_lists(ck, case):
    name, dtype, h, g, lens, C, div, n_probe, rho, top_k = case
    wl = small_workload(name, dtype, h, g, lens, tuple(range(300, 300 + len(lens))), C, div, n_probe, rho, top_k, 1)
    bt = gen_batch(wl)
    oi = H.oracle_index(bt)
    db = H.device_batch(bt)
    _say(f"[build {name}] building on the GPU")
    idx = ck.ctkvr_build_index(H.params_of(wl), db.q_prefill, db.cu_seqlens, True, db.k_pages, db.block_table,
                               db.ctx_lens)
    lists = ck.ctkvr_index_lists(idx)
    cen = ck.ctkvr_index_centroids(idx)
    ref_cen, ref_lst = oi.padded(wl)
    assert np.array_equal(cen, ref_cen), "centroid table differs from the last C prompt queries"
    for b, sq in enumerate(bt.seqs):
        Cb = wl.centroids_of(sq.s)
        assert np.array_equal(lists[b, :, :Cb], oi.lists[b]), f"lists of sequence {b} differ"
    info = ck.ctkvr_index_info(idx)
    assert info["index_bytes"] == wl.batch * wl.g * info["c_max"] * wl.list_len * 4
    st = H.run_decode_parity(bt, oi, idx, db)   # decode on the GPU-built index
    _say(f"[build {name}] ok {st}")
    ck.ctkvr_free(idx)


def test_exact_ties_duplicated_keys_and_centroids(ck):
    wl = small_workload("ties", "bf16", 4, 2, (512,), (400,), 8, 0, 3, 64, 40, 2)
    bt = gen_batch(wl)
    sq = bt.seqs[0]
    sq.K[:, 256:512] = sq.K[:, 0:256]
    sq.V[:, 256:512] = sq.V[:, 0:256]
    sq.q_tail[4:8] = sq.q_tail[0:4]
    bt = Batch(wl=wl, seqs=[sq], paged=paginate([sq], wl.page_size, 9))
    oi = H.oracle_index(bt)
    db = H.device_batch(bt)
    idx = ck.ctkvr_build_index(H.params_of(wl), db.q_prefill, db.cu_seqlens, True, db.k_pages, db.block_table,
                               db.ctx_lens)
    assert np.array_equal(ck.ctkvr_index_lists(idx)[0], oi.lists[0])
    H.run_decode_parity(bt, oi, idx, db)
    ck.ctkvr_free(idx)


@pytest.mark.parametrize("C,n_dup,n_probe", [(300, 200, 12), (1500, 1400, 40), (600, 90, 20)])
def test_many_equal_cosines_take_the_lowest_centroid_ids(ck, C, n_dup, n_probe):
    """n_dup of the C centroids are one and the same vector, so their cosines tie exactly, far more of them than are
    probed: the probed ids must be the oracle's (ties to the lowest id), with 2 and with 8 keys per thread in the
    selection."""
    wl = small_workload(f"dupcos{C}", "bf16", 4, 2, (2000,), (430,), C, 0, n_probe, 48, 40, 2)
    bt = gen_batch(wl)
    sq = bt.seqs[0]
    n_tail = sq.q_tail.shape[0]
    sq.q_tail[n_tail - C + 5:n_tail - C + 5 + n_dup] = sq.q_tail[n_tail - 1]    # the newest query, copied over older centroids
    bt = Batch(wl=wl, seqs=[sq], paged=paginate([sq], wl.page_size, 9))
    oi = H.oracle_index(bt)
    db = H.device_batch(bt)
    cen, lst = oi.padded(wl)
    idx = ck.ctkvr_index_load(H.params_of(wl), db.ctx_lens, cen, lst)
    st = H.run_decode_parity(bt, oi, idx, db)
    _say(f"[dupcos C={C} dup={n_dup}] ok {st}")
    ck.ctkvr_free(idx)


def test_lattice_inputs_all_scores_exact(ck):
    wl = small_workload("lattice", "bf16", 8, 2, (1200,), (500,), 16, 0, 4, 90, 60, 3)
    sq = gen_lattice_sequence(500, 1200, 8, 2, 128, 16, 3)
    bt = Batch(wl=wl, seqs=[sq], paged=paginate([sq], wl.page_size, 5))
    oi = H.oracle_index(bt)
    db = H.device_batch(bt)
    idx = ck.ctkvr_build_index(H.params_of(wl), db.q_prefill, db.cu_seqlens, True, db.k_pages, db.block_table,
                               db.ctx_lens)
    assert np.array_equal(ck.ctkvr_index_lists(idx)[0], oi.lists[0])
    H.run_decode_parity(bt, oi, idx, db)
    ck.ctkvr_free(idx)


def test_cfg1_tiny_fp32_end_to_end(ck):
    wl = workload("cfg1")
    bt = gen_batch(wl)
    oi = H.oracle_index(bt)
    db = H.device_batch(bt)
    idx = ck.ctkvr_build_index(H.params_of(wl), db.q_prefill, db.cu_seqlens, True, db.k_pages, db.block_table,
                               db.ctx_lens)
    assert np.array_equal(ck.ctkvr_index_lists(idx)[0], oi.lists[0])
    st = H.run_decode_parity(bt, oi, idx, db)
    _say(f"[cfg1] {st}")
    ck.ctkvr_free(idx)


def test_cfg2_32k_decode_on_oracle_index(ck):
    wl = workload("cfg2")
    _say("[cfg2] generating inputs")
    bt = gen_batch(wl, n_decode=6)
    _say("[cfg2] oracle index build (CPU)")
    oi = H.oracle_index(bt)
    db = H.device_batch(bt)
    cen, lst = oi.padded(wl)
    idx = ck.ctkvr_index_load(H.params_of(wl), db.ctx_lens, cen, lst)
    _say("[cfg2] decode parity")
    st = H.run_decode_parity(bt, oi, idx, db)
    _say(f"[cfg2] ok {st}")
    ck.ctkvr_free(idx)
    _say("[cfg2] GPU exact build vs oracle lists")
    idx2 = ck.ctkvr_build_index(H.params_of(wl), db.q_prefill, db.cu_seqlens, True, db.k_pages, db.block_table,
                                db.ctx_lens)
    assert np.array_equal(ck.ctkvr_index_lists(idx2)[0], oi.lists[0])
    ck.ctkvr_free(idx2)


def test_bad_max_pages_is_an_error_not_a_fault(ck):
    import torch
    wl = small_workload("err", "bf16", 4, 2, (300,), (1,), 8, 0, 2, 32, 16, 1)
    bt = gen_batch(wl)
    db = H.device_batch(bt)
    oi = H.oracle_index(bt)
    cen, lst = oi.padded(wl)
    idx = ck.ctkvr_index_load(H.params_of(wl), db.ctx_lens, cen, lst)
    out = torch.empty((1, 4, 128), dtype=torch.float32, device="cuda")
    short = db.block_table[:, :5].contiguous()
    with pytest.raises(ck.CtkvrError):
        ck.ctkvr_decode_step(idx, H.to_dev(bt.seqs[0].q_decode[:1], wl), db.k_pages, db.v_pages, short, out)
    bad = lst.copy()
    bad[0, 0, 0, 0] = 300
    with pytest.raises(ck.CtkvrError):
        ck.ctkvr_index_load(H.params_of(wl), db.ctx_lens, cen, bad)
    ck.ctkvr_free(idx)


def _full_size(ck, name, steps, n_decode):
    wl = workload(name)
    _say(f"[{name}] generating inputs")
    bt = gen_batch(wl, n_decode=n_decode)
    db = H.device_batch(bt)
    _say(f"[{name}] GPU index build")
    idx = ck.ctkvr_build_index(H.params_of(wl), db.q_prefill, db.cu_seqlens, True, db.k_pages, db.block_table,
                               db.ctx_lens)
    _say(f"[{name}] sampled parity against the oracle")
    st = H.run_sampled_parity(bt, idx, db, steps, say=_say)
    _say(f"[{name}] ok {st}")
    ck.ctkvr_free(idx)


def test_cfg3_128k_batch4_sampled(ck):
    """Full size, launch configuration of the benchmark: sampled lists and two decode steps."""
    _full_size(ck, "cfg3", steps=[0, 5], n_decode=6)


def test_cfg4_ragged_batch16_sampled(ck):
    _full_size(ck, "cfg4", steps=[0, 3], n_decode=4)


def test_paper_operating_point_llama_shape_sampled(ck):
    """C = 2048, C' = 4, rho = 2.5 rho' = 2560, rho' = 1024 at 32K (the evaluation section's set-up), 32/8 heads."""
    _full_size(ck, "paper_llama", steps=[0, 3], n_decode=4)


def test_paper_operating_point_yi_shape_sampled(ck):
    """The same operating point with rho' = 512 on the 32/4-head shape (G = 8)."""
    _full_size(ck, "paper_yi", steps=[0, 3], n_decode=4)


def test_dynamic_budget_four_percent_of_the_context_sampled(ck):
    """rho' = 0.04 s = 1311 and rho = 2.5 rho' = 3277 at 32K (the budget of the appendix's equal-sparsity comparison):
    neither is a power of two or a multiple of a tile."""
    _full_size(ck, "paper_budget4", steps=[0, 3], n_decode=4)


# --------------------------------------------------------------------------- #
# matrix-core list build (Algorithm 1 lines 2-4 with the dot products on MFMA)
# --------------------------------------------------------------------------- #
# The matrix-core route differs from the fixed-order route only in how the 128 products of a logit are summed;
# tests/bands.py derives from that how far from the rho-th key the two may disagree.
def _check_lists_within_band(gpu_lists, sq, Qc, wl, pairs=None, exact_dots=False, n_init=0, n_local=0):
    """GPU lists may differ from the oracle's only in ids whose (oracle) key lies within key_band of the rho-th.
    Returns (ids that differ, largest such distance as a fraction of the band that allowed it, the distance)."""
    ref, keys = oracle.build_lists(sq.K, Qc, wl.list_len, pairs=pairs, return_keys=True, n_init=n_init, n_local=n_local)
    g, C = wl.g, Qc.shape[1]
    G = wl.h // g
    scale = oracle.default_scale(Qc.shape[2])
    if pairs is None:
        pairs = np.array([[kv, j] for kv in range(g) for j in range(C)], np.int32)
        ref = ref.reshape(-1, wl.list_len)
    n_diff, worst, worst_abs = 0, 0.0, 0.0
    for (kv, j), r, key in zip(pairs, ref, keys):
        got = gpu_lists[kv, j]
        assert np.all(np.diff(got) > 0) and got[0] >= 0 and got[-1] < sq.s
        if np.array_equal(got, r):
            continue
        band = key_band(Qc[kv * G:(kv + 1) * G, j], sq.K[kv], scale, exact_dots=exact_dots)
        key = key[n_init:len(key) - n_local]       # the resident window is never listed
        got, r = got - n_init, r - n_init
        kth = np.sort(key)[::-1][wl.list_len - 1]
        odd = np.setxor1d(got, r)
        dist = float(np.abs(key[odd] - kth).max())
        assert dist <= band, f"list (kv {kv}, centroid {j}) differs {dist:.3g} from the rho-th key, band {band:.3g}"
        worst, worst_abs = max(worst, dist / band), max(worst_abs, dist)
        n_diff += len(odd) // 2
    return n_diff, worst, worst_abs


def test_mfma_build_on_lattice_inputs_differs_only_through_the_denominators(ck):
    """Dot products that are exact in fp32: both routes see the same logits and maxima, and only the way the
    softmax denominators are summed separates them (a band of a few 1e-5 instead of one that scales with the norms)."""
    wl = small_workload("lattice_mfma", "bf16", 8, 2, (2500,), (510,), 70, 0, 4, 120, 60, 2)
    sq = gen_lattice_sequence(510, 2500, 8, 2, 128, 70, 2)
    bt = Batch(wl=wl, seqs=[sq], paged=paginate([sq], wl.page_size, 6))
    oi = H.oracle_index(bt)
    db = H.device_batch(bt)
    idx = ck.ctkvr_build_index(H.params_of(wl, build_algo=ck.BUILD_MFMA), db.q_prefill, db.cu_seqlens, True, db.k_pages,
                               db.block_table, db.ctx_lens)
    got = ck.ctkvr_index_lists(idx)[0]
    n_diff, worst, worst_abs = _check_lists_within_band(got, sq, oi.Qc[0], wl, exact_dots=True)
    _say(f"[mfma lattice] ids that differ: {n_diff}; farthest from the rho-th key {worst_abs:.3g} = {worst:.3f} of the band")
    assert n_diff <= 0.001 * got.size
    if n_diff == 0:      # the same index as the oracle's: the decode step on it must then agree as well
        H.run_decode_parity(bt, oi, idx, db)
    ck.ctkvr_free(idx)


@pytest.mark.parametrize("s,h,g", [(2500, 8, 2), (2501, 4, 2), (1999, 8, 1)])
def test_mfma_build_without_the_resident_window_on_lattice_inputs(ck, s, h, g):
    """Lists that leave out the initial and local keys (Algorithm 1 lines 5-6), by the matrix-core route: row lengths
    that do and do not allow the 16-byte key stores, window edges inside a group of four keys, group sizes 4, 2, 8."""
    n_init, n_local = 7, 45
    wl = small_workload("lattice_mfma_win", "bf16", h, g, (s,), (511,), 70, 0, 4, 120, 60, 1)
    sq = gen_lattice_sequence(511 + s, s, h, g, 128, 70, 1)
    bt = Batch(wl=wl, seqs=[sq], paged=paginate([sq], wl.page_size, 7))
    Qc = oracle.centroids_last_c(sq.q_tail, 70)
    db = H.device_batch(bt)
    idx = ck.ctkvr_build_index(H.params_of(wl, build_algo=ck.BUILD_MFMA, n_init=n_init, n_local=n_local), db.q_prefill,
                               db.cu_seqlens, True, db.k_pages, db.block_table, db.ctx_lens)
    got = ck.ctkvr_index_lists(idx)[0]
    assert got.min() >= n_init and got.max() < s - n_local
    n_diff, worst, worst_abs = _check_lists_within_band(got, sq, Qc, wl, exact_dots=True, n_init=n_init, n_local=n_local)
    _say(f"[mfma lattice window] ids that differ: {n_diff}; farthest from the rho-th key {worst_abs:.3g} = {worst:.3f} of the band")
    assert n_diff <= 0.001 * got.size
    ck.ctkvr_free(idx)


@pytest.mark.parametrize("case", [SMALL[0], SMALL[1], SMALL[3], SMALL[4], SMALL[7]],
                         ids=[SMALL[i][0] for i in (0, 1, 3, 4, 7)])
def test_mfma_build_matches_oracle_up_to_ties(ck, case):
    name, dtype, h, g, lens, C, div, n_probe, rho, top_k = case
    wl = small_workload(name, dtype, h, g, lens, tuple(range(600, 600 + len(lens))), C, div, n_probe, rho, top_k, 1)
    bt = gen_batch(wl)
    db = H.device_batch(bt)
    idx = ck.ctkvr_build_index(H.params_of(wl, build_algo=ck.BUILD_MFMA), db.q_prefill, db.cu_seqlens, True, db.k_pages,
                               db.block_table, db.ctx_lens)
    lists = ck.ctkvr_index_lists(idx)
    n_diff, worst, worst_abs = 0, 0.0, 0.0
    for b, sq in enumerate(bt.seqs):
        Cb = wl.centroids_of(sq.s)
        n, w, wa = _check_lists_within_band(lists[b, :, :Cb], sq, oracle.centroids_last_c(sq.q_tail, Cb), wl)
        n_diff, worst, worst_abs = n_diff + n, max(worst, w), max(worst_abs, wa)
    _say(f"[mfma {name}] ids that differ inside the derived band: {n_diff}; farthest from the rho-th key "
         f"{worst_abs:.3g} = {worst:.3f} of the band")
    ck.ctkvr_free(idx)


@pytest.mark.parametrize("name,h,g,s,rho,expect_redo", [
    ("cand_ok", 8, 2, 6000, 400, False),         # about 2 rho + 256 = 1056 candidates per unit: within [rho, 4 rho]
    ("cand_all_equal", 8, 2, 2500, 40, True),    # every key the same vector: all s keys tie with the threshold and cannot all be candidates: handed back, same lists
    ("cand_g1", 2, 2, 6100, 400, False),         # one head per group: a wave's two work items are two sub-tiles
    ("cand_g2", 4, 2, 5900, 400, False),
    ("cand_g8", 8, 1, 6200, 400, False),         # four head pairs meet in shared memory
])
def test_mfma_build_from_candidates_gives_the_lists_of_the_route_that_ranks_every_key(ck, name, h, g, s, rho, expect_redo, monkeypatch):
    """The candidate route (threshold from a sample of the positions, exact selection among the keys above it) and
    its hand-back when a unit has too few or too many candidates: bit-equal lists either way, since both rank the
    same matrix-core keys; and within the derived band of the oracle's."""
    wl = small_workload(name, "bf16", h, g, (s, s - 777), (620, 621), 40, 0, 4, rho, 60, 1)
    bt = gen_batch(wl)
    if name == "cand_all_equal":
        for sq in bt.seqs:
            sq.K[:] = sq.K[:, :1]
        bt = Batch(wl=wl, seqs=bt.seqs, paged=paginate(bt.seqs, wl.page_size, 11))
    db = H.device_batch(bt)
    lists = {}
    for forced in ("0", "1", "redo"):
        monkeypatch.setenv("CTKVR_BUILD_CANDIDATES", "0" if forced == "0" else "1")
        if forced == "redo":
            monkeypatch.setenv("CTKVR_BUILD_CANDIDATES_REDO", "1")
        idx = ck.ctkvr_build_index(H.params_of(wl, build_algo=ck.BUILD_MFMA), db.q_prefill, db.cu_seqlens, True, db.k_pages,
                                   db.block_table, db.ctx_lens)
        monkeypatch.delenv("CTKVR_BUILD_CANDIDATES_REDO", raising=False)
        by_cand, redone = ck.ctkvr_index_build_route(idx)
        assert by_cand == (forced != "0")
        if forced == "1":
            assert (redone > 0) == expect_redo, f"{redone} chunks handed back"
        if forced == "redo":
            assert redone > 0
        lists[forced] = ck.ctkvr_index_lists(idx)
        ck.ctkvr_free(idx)
    assert np.array_equal(lists["0"], lists["1"]) and np.array_equal(lists["0"], lists["redo"])
    for b, sq in enumerate(bt.seqs):
        n, w, wa = _check_lists_within_band(lists["1"][b, :, :40], sq, oracle.centroids_last_c(sq.q_tail, 40), wl)
        _say(f"[mfma {name}] sequence {b}: ids that differ inside the derived band: {n}; farthest {wa:.3g} = {w:.3f} of the band")


def test_scratch_kept_between_candidate_builds_changes_no_list(ck, monkeypatch):
    """The candidate route keeps its device scratch between builds: a build that finds the scratch of a larger,
    different build (its contents still there), one that has to grow it, and one after ctkvr_release_scratch give
    the lists of a build with a scratch of its own."""
    shapes = {"large": (16, 2, 12000, 300), "small": (8, 2, 9000, 256), "larger": (16, 4, 14000, 320)}
    dbs, wls = {}, {}
    for name, (h, g, s, rho) in shapes.items():
        wls[name] = small_workload("scratch_" + name, "bf16", h, g, (s, s - 500), (630, 631), 40, 0, 4, rho, 60, 1)
        dbs[name] = H.device_batch(gen_batch(wls[name]))

    def build(name):
        wl, db = wls[name], dbs[name]
        idx = ck.ctkvr_build_index(H.params_of(wl, build_algo=ck.BUILD_MFMA), db.q_prefill, db.cu_seqlens, True, db.k_pages,
                                   db.block_table, db.ctx_lens)
        assert ck.ctkvr_index_build_route(idx)[0]
        lists = ck.ctkvr_index_lists(idx)
        ck.ctkvr_free(idx)
        return lists

    monkeypatch.setenv("CTKVR_BUILD_CANDIDATES", "1")
    ck.ctkvr_release_scratch()
    monkeypatch.setenv("CTKVR_BUILD_SCRATCH_CACHE", "0")
    own = {name: build(name) for name in shapes}
    monkeypatch.setenv("CTKVR_BUILD_SCRATCH_CACHE", "1")
    for name in ("large", "small", "small", "larger", "large"):
        assert np.array_equal(build(name), own[name]), name
    ck.ctkvr_release_scratch()
    ck.ctkvr_release_scratch()          # nothing kept: still fine
    assert np.array_equal(build("small"), own["small"])


def test_two_host_threads_building_at_once_each_get_their_lists(ck, monkeypatch):
    """Only one build at a time can hold the kept scratch; a build on another host thread that finds it taken
    allocates its own.  Two threads build different indices side by side, several times."""
    import threading
    import torch
    monkeypatch.setenv("CTKVR_BUILD_CANDIDATES", "1")
    shapes = {"a": (16, 2, 12000, 300), "b": (8, 2, 9000, 256)}
    wls = {n: small_workload("threads_" + n, "bf16", h, g, (s,), (640 + i,), 40, 0, 4, rho, 60, 1)
           for i, (n, (h, g, s, rho)) in enumerate(shapes.items())}
    dbs = {n: H.device_batch(gen_batch(wls[n])) for n in shapes}

    def build(name, stream=None):
        wl, db = wls[name], dbs[name]
        idx = ck.ctkvr_build_index(H.params_of(wl, build_algo=ck.BUILD_MFMA), db.q_prefill, db.cu_seqlens, True, db.k_pages,
                                   db.block_table, db.ctx_lens)
        lists = ck.ctkvr_index_lists(idx)
        ck.ctkvr_free(idx)
        return lists

    want = {n: build(n) for n in shapes}
    got, errors = {n: [] for n in shapes}, []

    def worker(name):
        try:
            torch.cuda.set_device(0)
            for _ in range(4):
                got[name].append(build(name))
        except Exception as e:      # noqa: BLE001  (reported below, in the test's own thread)
            errors.append((name, repr(e)))

    threads = [threading.Thread(target=worker, args=(n,)) for n in shapes]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for n in shapes:
        assert len(got[n]) == 4 and all(np.array_equal(x, want[n]) for x in got[n]), n


def test_mfma_build_from_candidates_leaves_the_resident_window_out(ck, monkeypatch):
    n_init, n_local = 9, 300
    wl = small_workload("cand_window", "bf16", 8, 2, (7000,), (622,), 33, 0, 4, 300, 60, 1)
    bt = gen_batch(wl)
    db = H.device_batch(bt)
    got = {}
    for forced in ("0", "1"):
        monkeypatch.setenv("CTKVR_BUILD_CANDIDATES", forced)
        idx = ck.ctkvr_build_index(H.params_of(wl, build_algo=ck.BUILD_MFMA, n_init=n_init, n_local=n_local), db.q_prefill,
                                   db.cu_seqlens, True, db.k_pages, db.block_table, db.ctx_lens)
        got[forced] = ck.ctkvr_index_lists(idx)[0]
        if forced == "1":
            assert ck.ctkvr_index_build_route(idx) == (True, 0)
        ck.ctkvr_free(idx)
    assert got["1"].min() >= n_init and got["1"].max() < 7000 - n_local
    assert np.array_equal(got["0"], got["1"])


def test_mfma_build_cfg2_and_128k_sampled(ck):
    for name, n_pairs in (("cfg2", 96), ("cfg5", 48)):
        wl = workload(name)
        _say(f"[mfma {name}] generating")
        bt = gen_batch(wl, n_decode=1)
        db = H.device_batch(bt)
        idx = ck.ctkvr_build_index(H.params_of(wl, build_algo=ck.BUILD_MFMA), db.q_prefill, db.cu_seqlens, True,
                                   db.k_pages, db.block_table, db.ctx_lens)
        lists = ck.ctkvr_index_lists(idx)
        sq = bt.seqs[0]
        C = wl.centroids_of(sq.s)
        rng = np.random.Generator(np.random.Philox(77))
        pairs = np.stack([rng.integers(0, wl.g, n_pairs), rng.integers(0, C, n_pairs)], axis=1).astype(np.int32)
        assert ck.ctkvr_index_build_route(idx) == (True, 0)     # long sequences: the candidate route, nothing handed back
        n_diff, worst, worst_abs = _check_lists_within_band(lists[0], sq, oracle.centroids_last_c(sq.q_tail, C), wl,
                                                            pairs=pairs)
        _say(f"[mfma {name}] {n_pairs} sampled lists agree; ids inside the derived band: {n_diff}; farthest from "
             f"the rho-th key {worst_abs:.3g} = {worst:.3f} of the band")
        ck.ctkvr_free(idx)
