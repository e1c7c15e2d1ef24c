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
