"""Pins of the oracle's resident window (Algorithm 1 lines 5-6, Algorithm 2 lines 10-11;
Section 3.2): the initial and local keys stay with the attention, the lists hold only the
keys in between, and the two attention outputs are merged."""
import numpy as np
import pytest

import oracle
from ctkvr_inputs import gen_sequence
from tests import brute

SCALE = oracle.default_scale(128)


def _seq(seed, s, h, g, C, n_decode=2, extra=0):
    sq = gen_sequence(seed, s + extra, h, g, 128, C, n_decode, "bf16")
    return sq


def test_lists_leave_out_the_window_and_match_the_definition():
    s, h, g, C, rho, n_init, n_local = 400, 8, 2, 6, 24, 7, 33
    G = h // g
    sq = _seq(81, s, h, g, C)
    Qc = oracle.centroids_last_c(sq.q_tail, C)
    lists = oracle.build_lists(sq.K, Qc, rho, SCALE, n_init=n_init, n_local=n_local)
    plain = oracle.build_lists(sq.K, Qc, rho, SCALE)
    assert lists.min() >= n_init and lists.max() < s - n_local
    assert np.all(np.diff(lists, axis=2) > 0)
    mid = np.arange(n_init, s - n_local)
    changed = 0
    for kv in range(g):
        for j in range(C):
            # line 2's score is the softmax over ALL s keys; only the choice is restricted
            A = brute.group_softmax_max(Qc[kv * G:(kv + 1) * G, j], sq.K[kv], SCALE)
            brute.check_topn_within_band(lists[kv, j], A[mid], mid, rho, 1e-5)
            # a list of the plain build that holds no window key must be unchanged
            inside = np.all((plain[kv, j] >= n_init) & (plain[kv, j] < s - n_local))
            assert np.array_equal(lists[kv, j], plain[kv, j]) == bool(inside)
            changed += not inside
    assert changed > 0, "the case should exercise the exclusion"


def test_no_window_is_the_plain_path():
    s, h, g, C, rho = 300, 4, 2, 5, 20
    sq = _seq(82, s, h, g, C)
    Qc = oracle.centroids_last_c(sq.q_tail, C)
    lists = oracle.build_lists(sq.K, Qc, rho, SCALE)
    assert np.array_equal(lists, oracle.build_lists(sq.K, Qc, rho, SCALE, n_init=0, n_local=0))
    q = sq.q_decode[0]
    a = oracle.decode_step(q, sq.K, sq.V, Qc, lists, 3, 16, SCALE)
    b = oracle.decode_step_window(q, sq.K, sq.V, Qc, lists, 3, 16, s, 0, 0, SCALE)
    assert np.array_equal(a.sel, b.sel) and np.array_equal(a.out, b.out) and np.array_equal(a.lse, b.lse)


@pytest.mark.parametrize("grown", [0, 5])
def test_window_plus_everything_in_between_is_dense_attention(grown):
    """C' = C and rho = rho' = all keys between the windows: the sparse part attends over every
    indexed key, so the merged output is textbook attention over the whole cache -- including
    the tokens decoded after the index was built, which join the local window."""
    s, h, g, C, n_init, n_local = 260, 8, 2, 4, 9, 21
    sq = _seq(83, s, h, g, C, extra=grown)     # K, V hold s + grown tokens
    K0 = sq.K[:, :s]
    # the centroids: any C queries will do for this identity; take the generator's tail
    Qc = oracle.centroids_last_c(sq.q_tail, C)
    mid = s - n_init - n_local
    lists = oracle.build_lists(K0, Qc, mid, SCALE, n_init=n_init, n_local=n_local)
    assert np.array_equal(lists, np.broadcast_to(np.arange(n_init, s - n_local), lists.shape))
    for q in sq.q_decode:
        r = oracle.decode_step_window(q, sq.K, sq.V, Qc, lists, C, mid, s, n_init, n_local, SCALE)
        ref, lse = brute.dense_attention(q, sq.K, sq.V, SCALE)
        assert np.max(np.abs(r.out - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))
        assert np.max(np.abs(r.lse - lse)) <= 1e-12 * np.max(np.abs(lse))


def test_merge_is_attention_over_the_union_and_handles_an_empty_side():
    rng = np.random.default_rng(5)
    h, g, d, n = 4, 2, 128, 50
    q = rng.standard_normal((h, d)).astype(np.float32)
    K = rng.standard_normal((g, n, d)).astype(np.float32)
    V = rng.standard_normal((g, n, d)).astype(np.float32)
    full, lse_full = brute.dense_attention(q, K, V, SCALE)
    a, la = brute.dense_attention(q, K[:, :17], V[:, :17], SCALE)
    b, lb = brute.dense_attention(q, K[:, 17:], V[:, 17:], SCALE)
    m, lm = oracle.merge_attention(a, la, b, lb)
    assert np.max(np.abs(m - full)) < 1e-12 and np.max(np.abs(lm - lse_full)) < 1e-12
    # window_attention over "everything" is dense attention; an empty window contributes nothing
    w, lw = oracle.window_attention(q, K, V, n_init=n, s_index=n, n_local=0, scale=SCALE)
    assert np.max(np.abs(w - full)) < 1e-12 and np.max(np.abs(lw - lse_full)) < 1e-12
    e, le = oracle.window_attention(q, K, V, n_init=0, s_index=n, n_local=0, scale=SCALE)
    m2, lm2 = oracle.merge_attention(full, lse_full, e, le)
    assert np.array_equal(m2, full) and np.allclose(lm2, lse_full, rtol=0, atol=1e-12)
