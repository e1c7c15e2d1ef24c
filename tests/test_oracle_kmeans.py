"""Pins for the oracle's k-means centroid mode (the benchmark's index-build
configuration; not in the paper).  CPU only."""
import numpy as np
import pytest
from scipy.cluster.vq import kmeans2

import oracle
from ctkvr_inputs import bf16_bits_to_f32, f32_to_bf16_bits, gen_sequence
from ctkvr_inputs.kmeans_init import kmeanspp_for_sequence, kmeanspp_positions


def _seq(seed, s, h, g, dtype="f32"):
    return gen_sequence(seed, s, h, g, 128, s, 1, dtype, full_walk=True)


def test_points_are_the_groups_heads_concatenated():
    sq = _seq(1, 50, 4, 2)
    X = oracle.group_points(sq.q_full, 2)
    assert X.shape == (2, 50, 256)
    assert np.array_equal(X[1, 7, :128], sq.q_full[7, 2]) and np.array_equal(X[1, 7, 128:], sq.q_full[7, 3])


def test_one_centre_becomes_the_mean():
    sq = _seq(2, 300, 4, 2)
    Qc, assign, inertia = oracle.kmeans_centroids(sq.q_full, 2, np.zeros((2, 1), np.int32), iters=1, dtype="f32")
    X = oracle.group_points(sq.q_full, 2)
    for kv in range(2):
        mean = X[kv].astype(np.float64).mean(axis=0)
        got = Qc[kv * 2:(kv + 1) * 2, 0].reshape(-1)
        assert np.max(np.abs(got - mean)) <= 2e-6 * max(1.0, np.max(np.abs(mean)))
        assert np.all(assign[kv] == 0)
        assert inertia[kv, 1] <= inertia[kv, 0]
        assert abs(inertia[kv, 1] - np.sum((X[kv] - mean) ** 2)) <= 1e-6 * inertia[kv, 1]


def test_every_point_its_own_centre_gives_zero_inertia():
    sq = _seq(3, 40, 2, 1)
    init = np.arange(40, dtype=np.int32)[None, :]
    Qc, assign, inertia = oracle.kmeans_centroids(sq.q_full, 1, init, iters=2, dtype="f32")
    assert np.all(inertia < 1e-6) and np.array_equal(assign[0], np.arange(40))
    # fp32 data is summed on a 2^-20 grid: equal up to that resolution (bf16 data would be exact)
    assert np.max(np.abs(Qc.transpose(1, 0, 2).reshape(40, -1) - oracle.group_points(sq.q_full, 1)[0])) <= 2.0 ** -20


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_inertia_never_increases(dtype):
    sq = _seq(4, 600, 4, 2, dtype)
    init = kmeanspp_for_sequence(sq.q_full, 2, 12, seed=9)
    _, _, inertia = oracle.kmeans_centroids(sq.q_full, 2, init, iters=8, dtype=dtype)
    slack = 1e-3 if dtype == "bf16" else 1e-7        # bf16 centres are rounded after every update
    assert np.all(inertia[:, 1:] <= inertia[:, :-1] * (1 + slack))
    assert np.all(inertia[:, -1] < 0.9 * inertia[:, 0])


def test_one_lloyd_step_equals_scipy():
    sq = _seq(5, 500, 2, 1)
    X = oracle.group_points(sq.q_full, 1)[0]
    init = kmeanspp_positions(X, 8, seed=3)[None, :]
    Qc, assign, _ = oracle.kmeans_centroids(sq.q_full, 1, init, iters=1, dtype="f32")
    ref_c, ref_lab = kmeans2(X.astype(np.float64), X[init[0]].astype(np.float64), iter=1, minit="matrix")
    got = Qc.transpose(1, 0, 2).reshape(8, -1)
    assert np.max(np.abs(got - ref_c)) <= 2e-6 * np.max(np.abs(ref_c))
    # assign is measured on the updated centres, scipy's labels on the initial ones: compare through a second call
    _, assign0, _ = oracle.kmeans_centroids(sq.q_full, 1, init, iters=0, dtype="f32")
    assert np.array_equal(assign0[0], ref_lab)


def test_lattice_points_exact_mean_and_bf16_rounding():
    r = np.random.default_rng(0)
    s, h, g = 200, 2, 1
    q = (r.integers(-8, 9, size=(s, h, 128)) / 8.0).astype(np.float32)
    init = np.array([[0, 1, 2]], np.int32)
    Qc, _, _ = oracle.kmeans_centroids(q, g, init, iters=1, dtype="bf16")
    _, assign0, _ = oracle.kmeans_centroids(q, g, init, iters=0, dtype="bf16")
    X = q.reshape(s, 256).astype(np.float64)
    for c in range(3):
        mean = X[assign0[0] == c].mean(axis=0).astype(np.float32)
        want = bf16_bits_to_f32(f32_to_bf16_bits(mean))
        assert np.array_equal(Qc.transpose(1, 0, 2).reshape(3, -1)[c], want)


def test_kmeanspp_positions_are_distinct_and_seeded():
    sq = _seq(6, 400, 4, 2)
    a = kmeanspp_for_sequence(sq.q_full, 2, 16, seed=1)
    b = kmeanspp_for_sequence(sq.q_full, 2, 16, seed=1)
    c = kmeanspp_for_sequence(sq.q_full, 2, 16, seed=2)
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    assert all(len(set(row.tolist())) == 16 for row in a)


def test_tied_centres_send_points_to_the_lowest_id():
    """Two start positions naming the SAME point give two identical centres: every point is
    exactly as far from both, and the assignment must go to the lower centre id (a `>=` in the
    scan would send all of them to the higher one).  The higher one then has no members."""
    sq = _seq(7, 120, 2, 1)
    init = np.array([[5, 5, 60]], np.int32)          # centres 0 and 1 coincide
    _, assign0, _ = oracle.kmeans_centroids(sq.q_full, 1, init, iters=0, dtype="f32")
    assert not np.any(assign0[0] == 1)
    assert np.any(assign0[0] == 0) and np.any(assign0[0] == 2)
    X = oracle.group_points(sq.q_full, 1)[0].astype(np.float64)
    d0 = np.sum((X - X[5]) ** 2, axis=1)
    d2 = np.sum((X - X[60]) ** 2, axis=1)
    assert np.array_equal(assign0[0], np.where(d2 < d0, 2, 0))       # brute force, ties to the lower id
    # the same with the duplicate in the highest slots: the lower of the two still wins
    init = np.array([[60, 5, 5]], np.int32)
    _, assign0, _ = oracle.kmeans_centroids(sq.q_full, 1, init, iters=0, dtype="f32")
    assert not np.any(assign0[0] == 2)
    assert np.array_equal(assign0[0], np.where(d2 < d0, 0, 1))


def test_a_centre_without_members_keeps_its_position():
    """The duplicate centre of the case above receives no point; after an update it must still be
    where it started (not zero, not NaN, not moved to a mean), while its twin has moved to the mean
    of its members; and it stays there over further iterations as long as it stays empty."""
    sq = _seq(8, 150, 2, 1)
    init = np.array([[9, 9, 100]], np.int32)
    X = oracle.group_points(sq.q_full, 1)[0]
    for iters in (1, 3):
        Qc, assign, inertia = oracle.kmeans_centroids(sq.q_full, 1, init, iters=iters, dtype="f32")
        cent = Qc.transpose(1, 0, 2).reshape(3, -1)
        assert np.all(np.isfinite(cent))
        if not np.any(assign[0] == 1):                    # still empty on the final centres
            assert np.array_equal(cent[1], X[9])
        assert not np.array_equal(cent[0], X[9])          # the twin took the members and moved
        assert np.all(inertia[:, 1:] <= inertia[:, :-1] * (1 + 1e-7))
    _, assign0, _ = oracle.kmeans_centroids(sq.q_full, 1, init, iters=0, dtype="f32")
    Qc1, _, _ = oracle.kmeans_centroids(sq.q_full, 1, init, iters=1, dtype="f32")
    cent1 = Qc1.transpose(1, 0, 2).reshape(3, -1)
    assert np.array_equal(cent1[1], X[9])                 # one update: the empty centre has not moved at all
    mean0 = X[assign0[0] == 0].astype(np.float64).mean(axis=0)
    assert np.max(np.abs(cent1[0] - mean0)) <= 2e-6 * max(1.0, np.max(np.abs(mean0)))


def test_starting_from_explicit_centres_equals_starting_from_their_positions():
    sq = _seq(9, 400, 4, 2, "bf16")
    init = kmeanspp_for_sequence(sq.q_full, 2, 10, seed=4)
    a = oracle.kmeans_centroids(sq.q_full, 2, init, iters=3)
    Qc0 = np.stack([sq.q_full[init[head // 2], head] for head in range(4)])
    b = oracle.kmeans_from_centres(sq.q_full, 2, Qc0, iters=3)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert np.allclose(a[2], b[2], rtol=1e-12, atol=0)    # the inertia is a threaded fp64 sum: order may differ
    # and two iterations then one more equal three in one go (the centres are the whole state)
    mid = oracle.kmeans_from_centres(sq.q_full, 2, Qc0, iters=2)[0]
    assert np.array_equal(oracle.kmeans_from_centres(sq.q_full, 2, mid, iters=1)[0], a[0])
