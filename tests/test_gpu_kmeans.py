"""k-means centroid mode on the GPU (matrix-core assignment, fixed-point sums)
against the oracle's Lloyd iterations from the same seeded start positions.
Bit-exact where the arithmetic is exact (lattice inputs, first update); beyond
that a tie in the assignment may resolve differently and the runs drift:
compared through inertia, and through the argmin property: iteration T of the GPU
must be one exact Lloyd step of the oracle from the GPU's own centres after
iteration T-1, except for the centres that a near-tie (brute force, fp64) touches."""
import numpy as np
import pytest

import oracle
from ctkvr_inputs import Batch, bf16_bits_to_f32, gen_batch, paginate, small_workload, Sequence
from ctkvr_inputs.kmeans_init import kmeanspp_for_sequence
from tests import harness as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ck():
    import torch
    assert torch.cuda.is_available()
    import paper_2512_15550_amd as ck
    ck.load_library()
    return ck


def _gpu_kmeans(ck, bt, init_pos, iters, algo=None):
    import torch
    wl = bt.wl
    if "dev" not in bt.extra:      # one upload per batch, however many builds follow
        bt.extra["dev"] = (H.device_batch(bt),) + tuple(H.device_full_queries(bt))
    db, qf, cu = bt.extra["dev"]
    p = H.params_of(wl, centroid_mode=ck.KMEANS, kmeans_iters=iters)
    if algo is not None:
        p.build_algo = algo
    ip = torch.from_numpy(np.ascontiguousarray(init_pos, np.int32)).cuda()
    idx = ck.ctkvr_build_index(p, qf, cu, False, db.k_pages, db.block_table, db.ctx_lens, init_pos=ip)
    cen = bf16_bits_to_f32(ck.ctkvr_index_centroids(idx))     # [B][h][C][d]
    return idx, db, cen


def _inertia_of(q_full, g, Qc):
    """Sum over positions of the squared distance to the nearest of the given centres [h][C][d],
    per KV head, by brute force in fp64 (nothing of the oracle or the GPU path is involved)."""
    s, h, d = q_full.shape
    G = h // g
    out = []
    for kv in range(g):
        X = q_full[:, kv * G:(kv + 1) * G].reshape(s, G * d).astype(np.float64)
        M = Qc[kv * G:(kv + 1) * G].transpose(1, 0, 2).reshape(Qc.shape[1], G * d).astype(np.float64)
        d2 = (X * X).sum(1)[:, None] - 2.0 * (X @ M.T) + (M * M).sum(1)[None, :]
        out.append(np.maximum(d2.min(axis=1), 0.0).sum())
    return np.array(out)


def _lattice_batch(seed, s, h, g, C, rho, n_probe, top_k):
    r = np.random.Generator(np.random.Philox(seed))
    lat = lambda shape: (r.integers(-8, 9, size=shape) / 8.0).astype(np.float32)
    sq = Sequence(seed=seed, dtype="bf16", s=s, K=lat((g, s, 128)), V=lat((g, s, 128)), q_tail=None,
                  q_decode=lat((2, h, 128)), q_full=lat((s, h, 128)))
    sq.q_tail = sq.q_full[s - C:]
    wl = small_workload("km_lattice", "bf16", h, g, (s,), (seed,), C, 0, n_probe, rho, top_k, 2)
    return Batch(wl=wl, seqs=[sq], paged=paginate([sq], wl.page_size, seed))


@pytest.mark.parametrize("h,g", [(8, 2), (2, 2), (8, 1)])
def test_first_update_on_lattice_inputs_is_bit_exact_and_decodes_like_the_oracle(ck, h, g):
    s, C = 1500, 40
    bt = _lattice_batch(700 + h + g, s, h, g, C, 64, 4, 48)
    sq = bt.seqs[0]
    init = kmeanspp_for_sequence(sq.q_full, g, C, seed=5)
    Qc, _, _ = oracle.kmeans_centroids(sq.q_full, g, init, iters=1)
    idx, db, cen = _gpu_kmeans(ck, bt, init[None], 1)
    assert np.array_equal(cen[0], Qc), "centres after the first update differ"
    lists = oracle.build_lists(sq.K, Qc, bt.wl.list_len)
    assert np.array_equal(ck.ctkvr_index_lists(idx)[0], lists)
    H.run_decode_parity(bt, H.OracleIndex([Qc], [lists]), idx, db)
    ck.ctkvr_free(idx)


def test_first_update_with_large_magnitudes_is_bit_exact(ck):
    """Queries of magnitude up to 2048 (still exact products and sums): the update's fixed-point sums leave
    the 32-bit range of its fast rounding path, mixed with members that stay inside it."""
    s, C, h, g = 1100, 24, 8, 2
    bt = _lattice_batch(731, s, h, g, C, 48, 3, 32)
    sq = bt.seqs[0]
    big = np.random.Generator(np.random.Philox(732)).random(s) < 0.3
    sq.q_full[big] *= np.float32(2048.0)
    sq.q_tail = sq.q_full[s - C:]
    init = kmeanspp_for_sequence(sq.q_full, g, C, seed=6)
    Qc, _, _ = oracle.kmeans_centroids(sq.q_full, g, init, iters=1)
    idx, db, cen = _gpu_kmeans(ck, bt, init[None], 1)
    assert np.array_equal(cen[0], Qc), "centres after the first update differ"
    ck.ctkvr_free(idx)


def test_zero_iterations_is_the_start_positions(ck):
    wl = small_workload("km0", "bf16", 8, 2, (900,), (710,), 24, 0, 4, 64, 32, 1)
    bt = gen_batch(wl, full_walk=True)
    sq = bt.seqs[0]
    init = kmeanspp_for_sequence(sq.q_full, 2, 24, seed=1)
    idx, _, cen = _gpu_kmeans(ck, bt, init[None], 0)
    G = 4
    for kv in range(2):
        for hh in range(G):
            assert np.array_equal(cen[0, kv * G + hh], sq.q_full[init[kv], kv * G + hh])
    ck.ctkvr_free(idx)


@pytest.mark.parametrize("mode", ["final", "init", "equi", "random"])
def test_centroid_position_modes_build_and_decode_like_the_oracle(ck, mode):
    """The paper's ablation on where the C kept queries sit (final / random / init / equi): zero
    Lloyd iterations from the chosen positions.  "final" must reproduce the default build."""
    from ctkvr_inputs.kmeans_init import centroid_positions
    s, h, g, C = 1200, 8, 2, 20
    wl = small_workload("pos_" + mode, "bf16", h, g, (s,), (720,), C, 0, 4, 64, 40, 2)
    bt = gen_batch(wl, full_walk=True)
    sq = bt.seqs[0]
    pos = centroid_positions(mode, s, C, g, seed=9)
    assert pos.shape == (g, C) and pos.min() >= 0 and pos.max() < s and np.all(np.diff(pos, axis=1) > 0)
    G = h // g
    Qc = np.stack([sq.q_full[pos[head // G], head] for head in range(h)])      # [h][C][d]
    lists = oracle.build_lists(sq.K, Qc, wl.list_len)
    idx, db, cen = _gpu_kmeans(ck, bt, pos[None], 0)
    assert np.array_equal(cen[0], Qc)
    assert np.array_equal(ck.ctkvr_index_lists(idx)[0], lists)
    if mode == "final":
        assert np.array_equal(Qc, oracle.centroids_last_c(sq.q_tail, C))
    H.run_decode_parity(bt, H.OracleIndex([Qc], [lists]), idx, db)
    ck.ctkvr_free(idx)


def test_gaussian_inputs_inertia_tracks_the_oracle_and_never_increases(ck):
    wl = small_workload("km_gauss", "bf16", 8, 2, (3000, 1700), (720, 721), 0, 50, 4, 96, 64, 1)
    bt = gen_batch(wl, full_walk=True)
    c_max = max(wl.centroids_of(s) for s in wl.ctx_lens)
    inits = [kmeanspp_for_sequence(sq.q_full, 2, wl.centroids_of(sq.s), seed=3 + b) for b, sq in enumerate(bt.seqs)]
    init_pad = np.zeros((2, 2, c_max), np.int32)
    for b, ip in enumerate(inits):
        init_pad[b, :, :ip.shape[1]] = ip
    prev = None
    for iters in (0, 1, 2, 5):
        idx, _, cen = _gpu_kmeans(ck, bt, init_pad, iters)
        ck.ctkvr_free(idx)
        cur = []
        for b, sq in enumerate(bt.seqs):
            Cb = wl.centroids_of(sq.s)
            gi = _inertia_of(sq.q_full, 2, cen[b, :, :Cb])
            _, _, oi = oracle.kmeans_centroids(sq.q_full, 2, inits[b], iters=iters)
            assert np.all(np.abs(gi - oi[:, -1]) <= 1e-3 * oi[:, -1]), (iters, b, gi, oi[:, -1])
            cur.append(gi)
        cur = np.concatenate(cur)
        if prev is not None:
            assert np.all(cur <= prev * (1 + 1e-3))
        prev = cur


def test_one_centre_is_the_mean_and_s_centres_give_zero_inertia(ck):
    wl = small_workload("km_one", "bf16", 4, 2, (64,), (730,), 1, 0, 1, 16, 8, 1)
    bt = gen_batch(wl, full_walk=True)
    sq = bt.seqs[0]
    idx, _, cen = _gpu_kmeans(ck, bt, np.zeros((1, 2, 1), np.int32), 1)
    Qc, _, _ = oracle.kmeans_centroids(sq.q_full, 2, np.zeros((2, 1), np.int32), iters=1)
    assert np.array_equal(cen[0], Qc)          # one cluster: no assignment to disagree on
    ck.ctkvr_free(idx)
    wl2 = small_workload("km_all", "bf16", 4, 2, (64,), (731,), 64, 0, 4, 16, 8, 1)
    bt2 = gen_batch(wl2, full_walk=True)
    init = np.tile(np.arange(64, dtype=np.int32), (1, 2, 1))
    idx, _, cen = _gpu_kmeans(ck, bt2, init, 2)
    assert np.all(_inertia_of(bt2.seqs[0].q_full, 2, cen[0]) <= 1e-6)   # every position is its own centre
    ck.ctkvr_free(idx)


def test_kmeans_argument_errors(ck):
    import torch
    wl = small_workload("km_err", "bf16", 4, 2, (200,), (740,), 8, 0, 2, 16, 8, 1)
    bt = gen_batch(wl, full_walk=True)
    db = H.device_batch(bt)
    qf, cu = H.device_full_queries(bt)
    p = H.params_of(wl, centroid_mode=ck.KMEANS, kmeans_iters=1)
    with pytest.raises(ck.CtkvrError):       # needs init_pos
        ck.ctkvr_build_index(p, qf, cu, False, db.k_pages, db.block_table, db.ctx_lens)
    ip = torch.zeros((1, 2, 8), dtype=torch.int32, device="cuda")
    with pytest.raises(ck.CtkvrError):       # needs all prompt queries
        ck.ctkvr_build_index(p, db.q_prefill, db.cu_seqlens, True, db.k_pages, db.block_table, db.ctx_lens, init_pos=ip)


# --------------------------------------------------------------------------- #
# more than one tile of 128 centres, a ragged last tile, every group size; full size
# --------------------------------------------------------------------------- #
def _touched_centres(X, M, rel=1e-5, chunk=8192):
    """Brute force in fp64: which centres could a point's assignment move to or from when the
    scores x.m - |m|^2/2 carry an error of up to rel * (|x| |m|_max + |m|_max^2 / 2)?  (The
    matrix cores accumulate n = 512..1024 exact bf16 products in fp32: the expected rounding is
    sqrt(n) 2^-24 ~ 2e-6 of |x||m|, the worst case n 2^-24 ~ 6e-5; 1e-5 sits between.)
    Returns (touched [C] bool, number of ambiguous points, inertia)."""
    X = np.asarray(X, np.float64)
    M = np.asarray(M, np.float64)
    m2 = (M * M).sum(1)
    mmax = float(np.sqrt(m2.max()))
    touched = np.zeros(M.shape[0], bool)
    n_amb, inertia = 0, 0.0
    for i0 in range(0, X.shape[0], chunk):
        x = X[i0:i0 + chunk]
        sc = x @ M.T - 0.5 * m2
        best = sc.max(1)
        x2 = (x * x).sum(1)
        near = sc >= (best - rel * (np.sqrt(x2) * mmax + 0.5 * mmax * mmax))[:, None]
        amb = near.sum(1) >= 2
        n_amb += int(amb.sum())
        touched |= near[amb].any(0)
        inertia += float(np.maximum(x2 - 2.0 * best, 0.0).sum())
    return touched, n_amb, inertia


def _flat(Qc, kv, G):
    """[h][C][d] -> the G*d-dimensional centres of KV head kv, [C][G*d]."""
    return Qc[kv * G:(kv + 1) * G].transpose(1, 0, 2).reshape(Qc.shape[1], -1)


def _check_one_lloyd_step(q_full, g, cen_prev, cen_next, tag, max_touched=0.25):
    """cen_next must be the oracle's Lloyd step from cen_prev for every centre no near-tie touches."""
    s, h, d = q_full.shape
    G = h // g
    ref, _, _ = oracle.kmeans_from_centres(q_full, g, cen_prev, iters=1)
    stats = []
    for kv in range(g):
        X = q_full[:, kv * G:(kv + 1) * G].reshape(s, G * d)
        touched, n_amb, in_prev = _touched_centres(X, _flat(cen_prev, kv, G))
        same = np.all(_flat(cen_next, kv, G) == _flat(ref, kv, G), axis=1)
        bad = np.flatnonzero(~same & ~touched)
        assert bad.size == 0, f"{tag} kv {kv}: centres {bad[:8].tolist()} differ from the oracle's step with no near-tie in reach"
        frac = float(touched.mean())
        assert frac <= max_touched, f"{tag} kv {kv}: {frac:.2%} of the centres lie within the tie band: the check has no teeth"
        _, _, in_next = _touched_centres(X, _flat(cen_next, kv, G))
        assert in_next <= in_prev * (1 + 1e-3), f"{tag} kv {kv}: inertia rose {in_prev} -> {in_next}"
        stats.append((n_amb, int(touched.sum()), int((~same).sum())))
    return stats


def _random_positions(seed, s, g, C):
    r = np.random.Generator(np.random.Philox(seed))
    return np.stack([np.sort(r.choice(s, size=C, replace=False)) for _ in range(g)]).astype(np.int32)


@pytest.mark.parametrize("h,g,C", [(2, 2, 300), (8, 2, 300), (8, 1, 300), (8, 2, 1100), (8, 1, 1100), (4, 4, 1100)])
def test_many_centres_first_update_on_lattice_inputs_is_bit_exact(ck, h, g, C):
    """300 and 1100 centres: three and nine tiles of 128 in the assignment kernel, the last one
    ragged (44 and 76 centres); group sizes 1, 4 and 8."""
    s = 6000
    bt = _lattice_batch(800 + h + g + C, s, h, g, C, 64, 4, 48)
    sq = bt.seqs[0]
    init = _random_positions(801 + C, s, g, C)
    print(f"[kmeans lattice h{h} g{g} C{C}] oracle", flush=True)
    Qc, _, _ = oracle.kmeans_centroids(sq.q_full, g, init, iters=1)
    print(f"[kmeans lattice h{h} g{g} C{C}] GPU", flush=True)
    idx, db, cen = _gpu_kmeans(ck, bt, init[None], 1)
    ck.ctkvr_free(idx)
    assert np.array_equal(cen[0], Qc), "centres after the first update differ"
    assert not np.array_equal(cen[0], np.stack([sq.q_full[init[head // (h // g)], head] for head in range(h)]))


@pytest.mark.parametrize("h,g,C", [(8, 2, 300), (8, 1, 1100), (2, 2, 1100)])
def test_many_centres_every_iteration_is_a_lloyd_step_of_the_previous_centres(ck, h, g, C):
    """Gaussian random-walk queries: iterations 1, 2 and 5 of the GPU, each checked as ONE oracle step
    from the GPU's own previous centres (the argmin property, with a band for near-ties)."""
    s = 6000
    wl = small_workload(f"km_many_{h}_{g}_{C}", "bf16", h, g, (s,), (760 + C + h,), C, 0, 4, 64, 48, 1)
    bt = gen_batch(wl, full_walk=True)
    sq = bt.seqs[0]
    init = _random_positions(761 + C, s, g, C)
    cen = {}
    for iters in (0, 1, 2, 4, 5):
        idx, _, c = _gpu_kmeans(ck, bt, init[None], iters)
        ck.ctkvr_free(idx)
        cen[iters] = c[0]
    for a, b in ((0, 1), (1, 2), (4, 5)):
        st = _check_one_lloyd_step(sq.q_full, g, cen[a], cen[b], f"h{h} g{g} C{C} iteration {b}")
        print(f"[kmeans many h{h} g{g} C{C}] iteration {b}: (ambiguous points, touched centres, differing centres) per KV head {st}", flush=True)


def test_cfg5_full_size_lloyd_iterations_sampled(ck):
    """The index-build benchmark configuration at full size (131072 positions, 32/8 heads, 2048 centres,
    10 Lloyd iterations), in the launch shape bench.py times.  One KV head is checked on the oracle:
    the first iteration from the shared start positions, and the tenth as a Lloyd step from the GPU's
    own centres after nine; the inertia of the GPU's centres tracks the oracle's."""
    from ctkvr_inputs import workload
    wl = workload("cfg5")
    print("[kmeans cfg5] generating all prompt queries", flush=True)
    bt = gen_batch(wl, n_decode=1, full_walk=True)
    sq = bt.seqs[0]
    g, G, C, s = wl.g, wl.h // wl.g, wl.n_centroids, sq.s
    init = _random_positions(55, s, g, C)
    cen = {}
    for iters in (0, 1, 9, 10):
        print(f"[kmeans cfg5] GPU build with {iters} iterations", flush=True)
        idx, _, c = _gpu_kmeans(ck, bt, init[None], iters, algo=ck.BUILD_MFMA)
        ck.ctkvr_free(idx)
        cen[iters] = c[0]
    kv = 5
    qh = np.ascontiguousarray(sq.q_full[:, kv * G:(kv + 1) * G])
    sl = slice(kv * G, (kv + 1) * G)
    assert np.array_equal(cen[0][sl], np.stack([sq.q_full[init[kv], kv * G + hh] for hh in range(G)]))
    print("[kmeans cfg5] oracle: first iteration of one KV head", flush=True)
    st = _check_one_lloyd_step(qh, 1, cen[0][sl], cen[1][sl], "cfg5 iteration 1")
    print(f"[kmeans cfg5] iteration 1: (ambiguous points, touched centres, differing centres) {st}", flush=True)
    _, _, o_in = oracle.kmeans_centroids(qh, 1, init[kv:kv + 1], iters=1)
    _, _, g_in = _touched_centres(qh.reshape(s, -1), _flat(cen[1][sl], 0, G))
    assert abs(g_in - o_in[0, 1]) <= 1e-3 * o_in[0, 1], (g_in, o_in)
    print("[kmeans cfg5] oracle: tenth iteration of the same head from the GPU's ninth", flush=True)
    st = _check_one_lloyd_step(qh, 1, cen[9][sl], cen[10][sl], "cfg5 iteration 10")
    print(f"[kmeans cfg5] iteration 10: (ambiguous points, touched centres, differing centres) {st}", flush=True)
    _, _, in10 = _touched_centres(qh.reshape(s, -1), _flat(cen[10][sl], 0, G))
    assert in10 < 0.9 * g_in, "ten iterations should have lowered the inertia well below the first"
