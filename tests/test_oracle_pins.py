"""Pins for the CPU oracle: every check here compares the oracle with something
other than itself -- brute-force fp64 definitions (tests/brute.py), library
exp/log/sort, closed forms, and the values the paper prints
(tests/golden/paper_values.txt).  CPU only."""
import math
import os

import numpy as np
import pytest

import oracle
from ctkvr_inputs import gen_lattice_sequence, gen_sequence
from tests import brute

SCALE = np.float32(1.0 / math.sqrt(128.0))
GOLD = {}
with open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")) as fh:
    for line in fh:
        if line.strip() and not line.startswith("#"):
            name, value, _ = [x.strip() for x in line.split("|", 2)]
            GOLD[name] = value


def _rng(seed):
    return np.random.Generator(np.random.Philox(seed))


# --------------------------------------------------------------------------- #
# fixed arithmetic primitives against library routines
# --------------------------------------------------------------------------- #
def test_dot128_close_to_exact_and_exact_on_lattice():
    r = _rng(1)
    for _ in range(200):
        a = r.standard_normal(128).astype(np.float32)
        b = r.standard_normal(128).astype(np.float32)
        exact = float(np.dot(a.astype(np.float64), b.astype(np.float64)))
        bound = 12 * 2.0 ** -24 * float(np.sum(np.abs(a.astype(np.float64) * b.astype(np.float64))))
        assert abs(float(oracle.dot128(a, b)) - exact) <= bound
    for _ in range(200):   # lattice k/8: all partial sums are exact, so the result is THE dot product
        a = (r.integers(-8, 9, 128) / 8.0).astype(np.float32)
        b = (r.integers(-8, 9, 128) / 8.0).astype(np.float32)
        assert float(oracle.dot128(a, b)) == float(np.dot(a.astype(np.float64), b.astype(np.float64)))


def test_dot128_uses_every_element_once():
    # e_i . e_j = delta_ij, and a weighted basis picks out single coordinates
    w = np.arange(1, 129, dtype=np.float32)
    for i in range(128):
        e = np.zeros(128, np.float32)
        e[i] = 1.0
        assert float(oracle.dot128(e, w)) == float(w[i])
        assert float(oracle.dot128(w, e)) == float(w[i])


def test_exp_series_against_libm():
    xs = np.concatenate([np.linspace(-30.0, 0.0, 20001), -np.logspace(-8, 1.4, 500)]).astype(np.float32)
    for x in xs:
        got = float(oracle.exp_c(float(x)))
        ref = math.exp(float(x))
        assert abs(got - ref) <= 2.5e-7 * ref, (x, got, ref)
    assert float(oracle.exp_c(0.0)) == 1.0
    assert float(oracle.exp_c(-30.5)) == 0.0
    assert float(oracle.exp_c(-1e30)) == 0.0
    assert float(oracle.exp_c(float("-inf"))) == 0.0


def test_log_fixed_against_libm():
    r = _rng(2)
    vals = [1, 2, 3, 1 << 40, (1 << 40) + 1, (1 << 57) - 1, 1 << 57, (1 << 63) + 12345]
    vals += [int(v) for v in r.integers(1, 1 << 62, 2000)]
    vals += [int((1 << 40) * math.sqrt(2.0) * (1 + d)) for d in (-1e-9, 0.0, 1e-9)]
    for S in vals:
        ref = math.log(S) - 40 * math.log(2.0)
        assert abs(oracle.log_fixed(S) - ref) <= 4e-15 * max(1.0, abs(ref)), S


def test_inv_norm_against_numpy():
    r = _rng(3)
    X = r.standard_normal((64, 128)).astype(np.float32) * 3
    ref = 1.0 / np.linalg.norm(X.astype(np.float64), axis=1)
    got = oracle.inv_norms(X)
    assert np.all(np.abs(got - ref) <= 3e-7 * ref)
    assert oracle.inv_norms(np.zeros((1, 128), np.float32))[0] == 0.0


# --------------------------------------------------------------------------- #
# Algorithm 1: inverted lists against the definition, brute force, tiny inputs
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("seed,h,g", [(11, 4, 2), (12, 8, 2), (13, 3, 3), (14, 4, 1)])
def test_lists_equal_bruteforce_definition(seed, h, g):
    s, C, rho = 64, 4, 8
    sq = gen_sequence(seed, s, h, g, 128, C, 1, "bf16")
    Qc = oracle.centroids_last_c(sq.q_tail, C)
    # line 1: the centroids are the last C prompt queries, verbatim
    for j in range(C):
        assert np.array_equal(Qc[:, j, :], sq.q_tail[sq.q_tail.shape[0] - C + j])
    lists = oracle.build_lists(sq.K, Qc, rho, SCALE)
    assert lists.shape == (g, C, rho) and lists.dtype == np.int32
    G = h // g
    in_band = 0
    for kv in range(g):
        for j in range(C):
            A_kv = brute.group_softmax_max(Qc[kv * G:(kv + 1) * G, j, :], sq.K[kv], SCALE)   # lines 2-3
            in_band += brute.check_topn_within_band(lists[kv, j], A_kv, np.arange(s), rho, 1e-5)   # line 4
            if in_band == 0:
                assert np.array_equal(lists[kv, j], brute.top_ids(A_kv, np.arange(s), rho))
    assert in_band == 0   # seeds chosen without near-ties at the list boundary


def test_lists_on_lattice_inputs_are_exact_and_ties_go_to_lowest_id():
    s, C, rho, h, g = 96, 3, 10, 4, 2
    sq = gen_lattice_sequence(21, s, h, g, 128, C, 1)
    K = sq.K.copy()
    K[:, 40:48] = K[:, 8:16]          # exact duplicate keys => exact score ties
    Qc = oracle.centroids_last_c(sq.q_tail, C)
    lists, keys = oracle.build_lists(K, Qc, rho, SCALE, return_keys=True)
    keys = keys.reshape(g, C, s)
    assert np.array_equal(keys[:, :, 40:48], keys[:, :, 8:16])
    for kv in range(g):
        for j in range(C):
            assert np.array_equal(lists[kv, j], brute.top_ids(keys[kv, j], np.arange(s), rho))
            A = brute.group_softmax_max(Qc[kv * 2:(kv + 1) * 2, j], K[kv], SCALE)
            assert np.allclose(np.exp(keys[kv, j].astype(np.float64)), A, rtol=2e-6, atol=0)
    # all keys identical: every score ties, so each list is the rho lowest ids
    K2 = np.tile(K[:, :1], (1, s, 1))           # all keys identical: every score ties
    lists2 = oracle.build_lists(K2, Qc, rho, SCALE)
    assert np.array_equal(lists2, np.broadcast_to(np.arange(rho, dtype=np.int32), (g, C, rho)))


def test_fixed_order_keys_lie_within_the_derived_bound_of_the_exact_ones():
    """The bound that the matrix-core parity test allows is derived, not chosen: here the one-route half of it is
    checked on the CPU, oracle keys (fp32, fixed order) against the definition in fp64, on inputs with the norms of
    the short workloads and, scaled up, of the long ones (query norms near 200)."""
    from tests.bands import key_error_bound, U_NEAREST
    for seed, s, gain in ((31, 700, 1.0), (32, 512, 16.0)):     # a power of two keeps the bf16 values exact
        h, g, C = 8, 2, 6
        sq = gen_sequence(seed, s, h, g, 128, C, 1, "bf16")
        Qc = oracle.centroids_last_c(sq.q_tail, C) * np.float32(gain)
        _, keys = oracle.build_lists(sq.K, Qc, 16, SCALE, return_keys=True)
        keys = keys.reshape(g, C, s)
        worst = 0.0
        for kv in range(g):
            for j in range(C):
                grp = Qc[kv * 4:(kv + 1) * 4, j]
                exact = np.log(brute.group_softmax_max(grp, sq.K[kv], SCALE))
                bound = key_error_bound(grp, sq.K[kv], SCALE, U_NEAREST)
                err = np.abs(keys[kv, j].astype(np.float64) - exact).max()
                assert err <= bound, (err, bound)
                worst = max(worst, err / bound)
        assert worst > 1e-4      # the bound is an error bound of this arithmetic, not a number of another scale


def test_index_bytes_closed_form_printed_in_paper():
    # the printed example, evaluated by the formula ...
    assert 1 * 4 * 512 * 2560 * 4 == int(GOLD["index_bytes_b1_g4_C512_rho2560"]) == 20 * 2 ** 20
    # ... and the array the oracle really returns for that (g, C, rho) has that many bytes
    g, C, rho, s = 4, 512, 2560, 2560
    sq = gen_sequence(5, s, 4, g, 128, C, 1, "bf16")
    lists = oracle.build_lists(sq.K, oracle.centroids_last_c(sq.q_tail, C), rho, SCALE)
    assert lists.nbytes == int(GOLD["index_bytes_b1_g4_C512_rho2560"])
    # rho = s: every list is every key
    assert np.array_equal(lists, np.broadcast_to(np.arange(s, dtype=np.int32), (g, C, rho)))


# --------------------------------------------------------------------------- #
# Algorithm 2 as a whole
# --------------------------------------------------------------------------- #
def _small_index(seed, s, h, g, C, rho, dtype="bf16", n_decode=2):
    sq = gen_sequence(seed, s, h, g, 128, C, n_decode, dtype)
    Qc = oracle.centroids_last_c(sq.q_tail, C)
    lists = oracle.build_lists(sq.K, Qc, rho, SCALE)
    return sq, Qc, lists


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_full_probe_full_budget_is_dense_attention(dtype):
    s, h, g, C = 200, 8, 2, 6
    sq, Qc, lists = _small_index(31, s, h, g, C, rho=s, dtype=dtype)
    for q in sq.q_decode:
        r = oracle.decode_step(q, sq.K, sq.V, Qc, lists, n_probe=C, top_k=s, scale=SCALE)
        assert np.array_equal(r.ncand, np.full(g, s))
        assert np.array_equal(r.sel, np.broadcast_to(np.arange(s), (g, s)))
        ref, lse = brute.dense_attention(q, sq.K, sq.V, SCALE)
        assert np.max(np.abs(r.out - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))
        assert np.max(np.abs(r.lse - lse)) <= 1e-12 * np.max(np.abs(lse))


def test_rerank_off_is_dense_attention_over_the_recalled_set():
    s, h, g, C, rho, n_probe = 300, 8, 2, 10, 40, 3
    sq, Qc, lists = _small_index(32, s, h, g, C, rho)
    G = h // g
    for q in sq.q_decode:
        r = oracle.decode_step(q, sq.K, sq.V, Qc, lists, n_probe, top_k=n_probe * rho, scale=SCALE)
        for kv in range(g):
            L = r.ncand[kv]
            assert rho <= L <= min(s, n_probe * rho)                     # L_recall = rho C' alpha, alpha <= 1
            assert np.array_equal(r.sel[kv, :L], r.cand[kv]) and np.all(r.sel[kv, L:] == -1)
            ref, lse = brute.dense_attention(q[kv * G:(kv + 1) * G], sq.K[kv:kv + 1, r.cand[kv]],
                                             sq.V[kv:kv + 1, r.cand[kv]], SCALE)
            assert np.max(np.abs(r.out[kv * G:(kv + 1) * G] - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))
            assert np.max(np.abs(r.lse[kv * G:(kv + 1) * G] - lse)) <= 1e-12 * np.max(np.abs(lse))


def test_decode_stages_against_bruteforce():
    s, h, g, C, rho, n_probe, top_k = 500, 8, 2, 16, 48, 4, 32
    sq, Qc, lists = _small_index(33, s, h, g, C, rho, n_decode=3)
    G = h // g
    for q in sq.q_decode:
        r = oracle.decode_step(q, sq.K, sq.V, Qc, lists, n_probe, top_k, SCALE)
        q64, Qc64 = q.astype(np.float64), Qc.astype(np.float64)
        for kv in range(g):
            # lines 1-2: cosine per query head, max over the group
            cos = np.stack([(Qc64[hh] @ q64[hh]) / (np.linalg.norm(Qc64[hh], axis=1) * np.linalg.norm(q64[hh]))
                            for hh in range(kv * G, (kv + 1) * G)]).max(axis=0)
            assert np.max(np.abs(r.cos_kv[kv] - cos)) <= 1e-6
            # line 3: top-C' == brute-force sort of the same scores, and of the exact ones up to a band
            assert np.array_equal(r.probe[kv], brute.top_ids(r.cos_kv[kv], np.arange(C), n_probe))
            brute.check_topn_within_band(r.probe[kv], cos, np.arange(C), n_probe, 1e-5)
            # line 4: sorted unique union of the probed lists
            union = sorted(set(int(t) for j in r.probe[kv] for t in lists[kv, j]))
            assert r.cand[kv].tolist() == union and r.ncand[kv] == len(union)
            # line 5: max over group of softmax over the recalled set
            A = brute.group_softmax_max(q[kv * G:(kv + 1) * G], sq.K[kv, r.cand[kv]], SCALE)
            assert np.allclose(np.exp(r.rerank_key[kv].astype(np.float64)), A, rtol=3e-6, atol=0)
            # line 6: top-rho'
            assert np.array_equal(r.sel[kv], brute.top_ids(r.rerank_key[kv], r.cand[kv], top_k))
            brute.check_topn_within_band(r.sel[kv], A, r.cand[kv], top_k, 1e-5)
            # lines 7-9: attention over exactly the selected keys
            ref, lse = brute.dense_attention(q[kv * G:(kv + 1) * G], sq.K[kv:kv + 1, r.sel[kv]],
                                             sq.V[kv:kv + 1, r.sel[kv]], SCALE)
            assert np.max(np.abs(r.out[kv * G:(kv + 1) * G] - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))
            assert np.max(np.abs(r.lse[kv * G:(kv + 1) * G] - lse)) <= 1e-12 * np.max(np.abs(lse))


def test_softmax_weights_sum_to_one_and_lse_merge():
    s, h, g, C, rho, n_probe, top_k = 400, 8, 2, 12, 40, 4, 30
    sq, Qc, lists = _small_index(34, s, h, g, C, rho)
    q = sq.q_decode[0]
    ones = np.ones_like(sq.V)
    r1 = oracle.decode_step(q, sq.K, ones, Qc, lists, n_probe, top_k, SCALE)
    assert np.max(np.abs(r1.out - 1.0)) < 1e-12            # sum of the softmax weights
    r = oracle.decode_step(q, sq.K, sq.V, Qc, lists, n_probe, top_k, SCALE)
    G = h // g
    for kv in range(g):
        a, b = r.sel[kv, :top_k // 2], r.sel[kv, top_k // 2:]
        qa = q[kv * G:(kv + 1) * G]
        oa, la = brute.dense_attention(qa, sq.K[kv:kv + 1, a], sq.V[kv:kv + 1, a], SCALE)
        ob, lb = brute.dense_attention(qa, sq.K[kv:kv + 1, b], sq.V[kv:kv + 1, b], SCALE)
        lse = np.logaddexp(la, lb)
        merged = oa * np.exp(la - lse)[:, None] + ob * np.exp(lb - lse)[:, None]
        assert np.max(np.abs(merged - r.out[kv * G:(kv + 1) * G])) < 1e-12
        assert np.max(np.abs(lse - r.lse[kv * G:(kv + 1) * G])) < 1e-12


def test_exact_ties_go_to_the_lowest_id():
    s, h, g, C, rho, n_probe, top_k = 256, 4, 2, 8, 64, 3, 20
    sq = gen_sequence(35, s, h, g, 128, C, 1, "bf16")
    K = sq.K.copy()
    K[:, 128:256] = K[:, 0:128]                      # every key exists twice
    tail = sq.q_tail.copy()
    tail[4:8] = tail[0:4]                            # every centroid exists twice
    Qc = oracle.centroids_last_c(tail, C)
    lists = oracle.build_lists(K, Qc, rho, SCALE)
    assert np.array_equal(lists[:, 4:8], lists[:, 0:4])
    r = oracle.decode_step(sq.q_decode[0], K, sq.V, Qc, lists, n_probe, top_k, SCALE)
    for kv in range(g):
        assert np.array_equal(r.cos_kv[kv, :4], r.cos_kv[kv, 4:])
        assert np.array_equal(r.probe[kv], brute.top_ids(r.cos_kv[kv], np.arange(C), n_probe))
        assert r.probe[kv].min() < 4                 # of a tied pair the lower id is taken first
        key_of = dict(zip(r.cand[kv].tolist(), r.rerank_key[kv].tolist()))
        both = [t for t in range(128) if t in key_of and t + 128 in key_of]
        assert both, "construction must recall some duplicated keys"
        for t in both:
            assert key_of[t] == key_of[t + 128]
            assert not (np.isin(t + 128, r.sel[kv]) and not np.isin(t, r.sel[kv]))
        assert np.array_equal(r.sel[kv], brute.top_ids(r.rerank_key[kv], r.cand[kv], top_k))


def test_query_equal_to_a_centroid_single_head_group_gives_exact_topk():
    # G = 1, q = c_j, C' = 1, rho' <= rho: centroid j wins with cosine 1 and the
    # selection is the exact global top-rho' of q over all keys (flat search).
    s, h, g, C, rho, top_k = 600, 2, 2, 9, 50, 20
    sq, Qc, lists = _small_index(36, s, h, g, C, rho)
    for j in (0, 4, 8):
        q = np.ascontiguousarray(Qc[:, j, :])
        r = oracle.decode_step(q, sq.K, sq.V, Qc, lists, 1, top_k, SCALE)
        assert np.all(r.probe == j)
        assert np.all(np.abs(r.cos_kv[:, j] - 1.0) <= 2e-7)
        for kv in range(g):
            flat = sq.K[kv].astype(np.float64) @ q[kv].astype(np.float64)
            brute.check_topn_within_band(r.sel[kv], flat, np.arange(s), top_k, 1e-6)
            assert np.array_equal(r.sel[kv], brute.top_ids(flat, np.arange(s), top_k))


def test_probe_invariant_to_rescaling_the_query():
    s, h, g, C, rho = 300, 8, 2, 20, 30
    sq, Qc, lists = _small_index(37, s, h, g, C, rho)
    q = sq.q_decode[0]
    c1, p1 = oracle.recall(q, Qc, g, 5)
    q2 = q.copy()
    q2[0::2] *= 4.0          # positive power-of-two factors, different per head
    q2[1::2] *= 0.125
    c2, p2 = oracle.recall(q2, Qc, g, 5)
    assert np.array_equal(p1, p2) and np.array_equal(c1, c2)


def test_lemma2_order_preservation_property():
    # unit vectors; delta = Q1.K1 - Q1.K2 > 4 sin(theta/2)  =>  Q2.K1 >= Q2.K2  (Appendix A, Lemma 2)
    r = _rng(8)
    unit = lambda v: (v / np.linalg.norm(v)).astype(np.float32)
    n_checked = 0
    for _ in range(3000):
        q1 = unit(r.standard_normal(128))
        q2 = unit(q1 + 0.02 * r.standard_normal(128))
        k1 = unit(q1 + 0.8 * r.standard_normal(128) / np.sqrt(128))
        k2 = unit(r.standard_normal(128))
        theta = math.acos(min(1.0, float(np.dot(q1.astype(np.float64), q2.astype(np.float64)))))
        delta = float(oracle.dot128(q1, k1)) - float(oracle.dot128(q1, k2))
        if delta > 4 * math.sin(theta / 2) + 1e-5:
            n_checked += 1
            assert float(oracle.dot128(q2, k1)) >= float(oracle.dot128(q2, k2))
    assert n_checked > 100


def test_cost_model_identities():
    f = lambda Lr, Lk: (Lr + 2 * Lk) / (2 * Lr)
    assert abs(f(10_000, 1_000) - float(GOLD["rerank_factor_Lrecall10K_Lrerank1K"])) < 1e-12
    s, h, g, C, rho, n_probe = 2000, 8, 2, 32, 100, 6
    sq, Qc, lists = _small_index(38, s, h, g, C, rho, n_decode=2)
    for q in sq.q_decode:
        r = oracle.decode_step(q, sq.K, sq.V, Qc, lists, n_probe, 50, SCALE)
        alpha = r.ncand / (rho * n_probe)
        assert np.all(alpha <= 1.0) and np.all(r.ncand >= rho)
