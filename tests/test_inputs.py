"""The seeded input generators: determinism, RoPE as a rotation, paging as a
pure permutation of rows.  CPU only."""
import numpy as np

from ctkvr_inputs import (bf16_bits_to_f32, f32_to_bf16_bits, gen_batch, gen_sequence, paginate, rope,
                          small_workload, workload)


def test_bf16_roundtrip_and_rounding():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -2.5, 0.0, 3.0e38], np.float32)
    b = bf16_bits_to_f32(f32_to_bf16_bits(x))
    assert b[0] == 1.0 and b[1] == 1.0                    # halfway case rounds to even
    assert b[2] == 1.0 + 2 ** -7 and b[3] == 1.0 + 2 ** -6
    assert np.array_equal(bf16_bits_to_f32(f32_to_bf16_bits(b)), b)


def test_rope_is_a_rotation_and_relative():
    r = np.random.default_rng(0)
    x, y = r.standard_normal((5, 128)), r.standard_normal((5, 128))
    px, py = np.arange(5) * 7 + 3, np.arange(5) * 11
    rx, ry = rope(x, px), rope(y, py)
    assert np.allclose(np.linalg.norm(rx, axis=1), np.linalg.norm(x, axis=1))
    # <R_a x, R_b y> depends on b - a only
    rx2, ry2 = rope(x, px + 100), rope(y, py + 100)
    assert np.allclose(np.sum(rx * ry, 1), np.sum(rx2 * ry2, 1))
    assert np.allclose(rope(x, np.zeros(5)), x)


def test_sequences_are_reproducible_and_walk_is_smooth():
    a = gen_sequence(7, 512, 8, 2, 128, 32, 4, "bf16")
    b = gen_sequence(7, 512, 8, 2, 128, 32, 4, "bf16")
    assert np.array_equal(a.K, b.K) and np.array_equal(a.q_tail, b.q_tail) and np.array_equal(a.q_decode, b.q_decode)
    c = gen_sequence(8, 512, 8, 2, 128, 32, 4, "bf16")
    assert not np.array_equal(a.K, c.K)
    assert a.q_tail.shape == (32, 8, 128) and a.q_decode.shape == (4, 8, 128) and a.K.shape == (2, 512, 128)
    # values are exactly representable in bf16
    assert np.array_equal(bf16_bits_to_f32(f32_to_bf16_bits(a.K)), a.K)
    full = gen_sequence(7, 512, 8, 2, 128, 32, 4, "f32", full_walk=True)
    assert full.q_full.shape == (512, 8, 128) and np.array_equal(full.q_full[-32:], full.q_tail)


def test_paging_is_a_permutation_of_rows():
    wl = small_workload(ctx_lens=(100, 37, 64), seeds=(1, 2, 3), n_centroids=8)
    bt = gen_batch(wl, n_decode=1)
    pg = bt.paged
    assert pg.block_table.shape == (3, 7) and list(pg.ctx_lens) == [100, 37, 64]
    used = pg.block_table[pg.block_table >= 0]
    assert len(set(used.tolist())) == len(used) == 7 + 3 + 4
    for b, sq in enumerate(bt.seqs):
        for t in (0, 1, 15, 16, sq.s - 1):
            page = pg.block_table[b, t // 16]
            assert np.array_equal(pg.k_pages[page, :, t % 16], sq.K[:, t])
            assert np.array_equal(pg.v_pages[page, :, t % 16], sq.V[:, t])


def test_named_workloads_match_the_configurations():
    w2, w3, w4 = workload("cfg2"), workload("cfg3"), workload("cfg4")
    assert (w2.h, w2.g, w2.ctx_lens, w2.n_centroids, w2.n_probe, w2.top_k, w2.n_decode) == (32, 8, [32768], 512, 32, 1024, 256)
    assert w3.batch == 4 and w3.ctx_lens[0] == 131072 and w3.n_centroids == 2048 and w3.n_probe == 64
    assert w4.batch == 16 and all(8192 <= s <= 65536 for s in w4.ctx_lens) and w4.centroids_of(8192) == 128
    assert workload("cfg1").dtype == "f32"
