"""Pins of the oracle's dynamic centroid update (Algorithm 2 line 12; Section 3.1.2,
"Dynamic Centroid Update"): the current query joins the index as a centroid whose list is
the top-rho keys by the rerank score, replacing the oldest mapping first."""
import numpy as np
import pytest

import oracle
from ctkvr_inputs import gen_sequence
from tests import brute

SCALE = oracle.default_scale(128)


def _index(seed, s, h, g, C, rho, n_decode):
    sq = gen_sequence(seed, s, h, g, 128, C, n_decode, "bf16")
    Qc = oracle.centroids_last_c(sq.q_tail, C)
    lists = oracle.build_lists(sq.K, Qc, rho, SCALE)
    return sq, Qc, lists


@pytest.mark.parametrize("rho,top_k", [(48, 48), (48, 20), (30, 64)])
def test_new_list_is_the_top_rho_of_the_rerank_scores(rho, top_k):
    s, h, g, C, n_probe = 600, 8, 2, 12, 4
    G = h // g
    sq, Qc, lists = _index(71, s, h, g, C, rho, 1)
    q = sq.q_decode[0]
    r = oracle.decode_step(q, sq.K, sq.V, Qc, lists, n_probe, top_k, SCALE)
    # the same ranking with budget rho, from the C routine that serves line 6
    _, _, _, sel_rho, _, _ = oracle.rerank_attend(q, sq.K, sq.V, lists, r.probe, rho, SCALE)
    Qc2, lists2 = Qc.copy(), lists.copy()
    slot = oracle.centroid_update(q, Qc2, lists2, r, n_updates=5)
    assert slot == 5
    for kv in range(g):
        assert r.ncand[kv] >= rho                       # every probed list has rho distinct ids
        assert np.array_equal(lists2[kv, slot], sel_rho[kv])
        if rho == top_k:
            assert np.array_equal(lists2[kv, slot], r.sel[kv])
        # and against the definition in fp64: softmax over the recalled set, max over the group
        A = brute.group_softmax_max(q[kv * G:(kv + 1) * G], sq.K[kv, r.cand[kv]], SCALE)
        brute.check_topn_within_band(lists2[kv, slot], A, r.cand[kv], rho, 1e-5)
    # the query is the new centroid of every query head; nothing else moved
    assert np.array_equal(Qc2[:, slot], q)
    keep = np.arange(C) != slot
    assert np.array_equal(Qc2[:, keep], Qc[:, keep]) and np.array_equal(lists2[:, keep], lists[:, keep])


def test_reissuing_the_query_probes_the_new_slot_first():
    s, h, g, C, rho, n_probe, top_k = 500, 8, 2, 10, 40, 3, 40
    sq, Qc, lists = _index(72, s, h, g, C, rho, 2)
    q = sq.q_decode[0]
    r = oracle.decode_step(q, sq.K, sq.V, Qc, lists, n_probe, top_k, SCALE)
    slot = oracle.centroid_update(q, Qc, lists, r, n_updates=3)
    r2 = oracle.decode_step(q, sq.K, sq.V, Qc, lists, n_probe, top_k, SCALE)
    for kv in range(g):
        assert slot in r2.probe[kv]
        assert np.argmax(r2.cos_kv[kv]) == slot and abs(r2.cos_kv[kv, slot] - 1.0) < 1e-6
        # the slot's list is among the recalled keys, so the keys the query attended to are found again
        assert np.all(np.isin(lists[kv, slot], r2.cand[kv]))
        assert np.array_equal(r2.sel[kv], r.sel[kv]) or len(np.intersect1d(r2.sel[kv], r.sel[kv])) >= 0.9 * top_k


def test_fifo_replaces_the_oldest_mapping_first_and_wraps():
    s, h, g, C, rho, n_probe, top_k = 400, 4, 2, 5, 24, 2, 24
    sq, Qc, lists = _index(73, s, h, g, C, rho, 2 * C + 1)
    Qc0 = Qc.copy()
    slots = []
    for n, q in enumerate(sq.q_decode):
        r = oracle.decode_step(q, sq.K, sq.V, Qc, lists, n_probe, top_k, SCALE)
        slots.append(oracle.centroid_update(q, Qc, lists, r, n_updates=n))
        if n == C - 2:   # the newest prompt query (last slot) is still there, the older ones are gone
            assert np.array_equal(Qc[:, C - 1], Qc0[:, C - 1])
            assert not any(np.array_equal(Qc[:, j], Qc0[:, j]) for j in range(C - 1))
    assert slots == [n % C for n in range(2 * C + 1)]
    # after the wrap every slot holds one of the last C decode queries, the oldest of them in the next slot to go
    for j in range(C):
        n = max(m for m in range(2 * C + 1) if m % C == j)
        assert np.array_equal(Qc[:, j], sq.q_decode[n])
    # every list stays well-formed: rho ascending distinct ids inside the context
    assert np.all(np.diff(lists, axis=2) > 0) and lists.min() >= 0 and lists.max() < s


def test_fewer_recalled_keys_than_rho_repeat_the_last_id():
    """Reading D-4: a list always holds rho entries.  While every list holds rho distinct ids the
    recalled set has at least rho keys and the rule cannot fire from a decode step, so it is pinned
    on a hand-made step result: 5 recalled keys for a list of 8, scores planted so that the order by
    score differs from the order by id."""
    g, C, rho, h = 2, 4, 8, 4
    lists = np.full((g, C, rho), -7, np.int32)
    Qc = np.zeros((h, C, 128), np.float32)
    q = np.arange(h * 128, dtype=np.float32).reshape(h, 128)
    cand = [np.array([3, 10, 11, 40, 90], np.int32), np.array([], np.int32)]
    key = [np.array([-5.0, -1.0, -9.0, -2.0, -3.0], np.float32), np.array([], np.float32)]
    res = oracle.DecodeResult(cos_kv=None, probe=None, cand=cand, ncand=np.array([5, 0], np.int32), rerank_key=key,
                              sel=None, out=None, lse=None)
    slot = oracle.centroid_update(q, Qc, lists, res, n_updates=6)
    assert slot == 2
    assert lists[0, 2].tolist() == [3, 10, 11, 40, 90, 90, 90, 90]     # all five, ascending, the last one repeated
    assert np.all(lists[1, 2] == -7)                                   # nothing recalled: the list is left alone
    assert np.all(lists[:, [0, 1, 3]] == -7)
    assert np.array_equal(Qc[:, 2], q) and not Qc[:, [0, 1, 3]].any()
