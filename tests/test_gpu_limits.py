"""GPU parity at the documented maxima of the library: the longest context it accepts
(2^20 tokens, the length of the paper's longest needle-in-a-haystack runs), the most
centroids per sequence together with the most probed centroids, and the largest group
size.  Same bar as the other parity tests: integers bit-equal, outputs within 2e-3."""
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


def _say(msg):
    print(msg, flush=True)


def test_maximum_context_length(ck):
    # one sequence of 2^20 tokens, one KV head shared by two query heads
    wl = small_workload("max_ctx", "bf16", 2, 1, (1 << 20,), (270,), 32, 0, 8, 4096, 2048, 2)
    _say("[max_ctx] generating 2^20 tokens")
    bt = gen_batch(wl)
    _say("[max_ctx] oracle index")
    oi = H.oracle_index(bt)
    db = H.device_batch(bt)
    _say("[max_ctx] exact build")
    idx = ck.ctkvr_build_index(H.params_of(wl), db.q_prefill, db.cu_seqlens, True, db.k_pages, db.block_table,
                               db.ctx_lens)
    assert np.array_equal(ck.ctkvr_index_lists(idx)[0], oi.lists[0])
    _say("[max_ctx] decode parity")
    st = H.run_decode_parity(bt, oi, idx, db)
    _say(f"[max_ctx] ok {st}")
    ck.ctkvr_free(idx)
    # one token more is refused on the host
    with pytest.raises(ck.CtkvrError):
        ck.ctkvr_index_load(H.params_of(wl), np.array([(1 << 20) + 1], np.int32), *oi.padded(wl))


def test_maximum_centroids_and_probes(ck):
    # C = 8192 centroids (every prompt query but the first 40), C' = 1024 probed lists of 8 keys
    wl = small_workload("max_c", "bf16", 1, 1, (8232,), (271,), 8192, 0, 1024, 8, 64, 2)
    _say("[max_c] generating")
    bt = gen_batch(wl)
    oi = H.oracle_index(bt)
    db = H.device_batch(bt)
    _say("[max_c] exact build")
    idx = ck.ctkvr_build_index(H.params_of(wl), db.q_prefill, db.cu_seqlens, True, db.k_pages, db.block_table,
                               db.ctx_lens)
    assert np.array_equal(ck.ctkvr_index_lists(idx)[0], oi.lists[0])
    st = H.run_decode_parity(bt, oi, idx, db)
    _say(f"[max_c] ok {st}")
    ck.ctkvr_free(idx)
    with pytest.raises(ck.CtkvrError):
        ck.ctkvr_index_load(H.params_of(wl, n_probe=1025), db.ctx_lens, *oi.padded(wl))


def test_largest_group_ragged_batch_with_updates(ck):
    # 8 query heads per KV head, ragged batch, centroid updates after every step
    wl = small_workload("g8_all", "bf16", 16, 2, (3001, 1999, 4500), (272, 273, 274), 40, 0, 6, 150, 90, 4)
    bt = gen_batch(wl)
    oi = H.oracle_index(bt)
    db = H.device_batch(bt)
    cen, lst = oi.padded(wl)
    idx = ck.ctkvr_index_load(H.params_of(wl), db.ctx_lens, cen, lst)
    st = H.run_decode_parity(bt, oi, idx, db, update=True)
    _say(f"[g8_all] ok {st}")
    ck.ctkvr_free(idx)


def test_few_probes_among_thousands_of_centroids(ck):
    # C' = 4 of C = 3000 centroids (more than 2048): the one-maximum-per-probe selection with 32 keys per thread
    wl = small_workload("c3000_p4", "bf16", 2, 1, (3100,), (275,), 3000, 0, 4, 16, 32, 3)
    bt = gen_batch(wl)
    oi = H.oracle_index(bt)
    db = H.device_batch(bt)
    cen, lst = oi.padded(wl)
    idx = ck.ctkvr_index_load(H.params_of(wl), db.ctx_lens, cen, lst)
    st = H.run_decode_parity(bt, oi, idx, db)
    _say(f"[c3000_p4] ok {st}")
    ck.ctkvr_free(idx)


def test_fp32_keys_beyond_the_cache_size(ck):
    # 138 MB of fp32 keys for one KV head: the scoring kernel takes its non-temporal loads in the fp32 form
    wl = small_workload("f32_stream", "f32", 1, 1, (270000,), (276,), 8, 0, 2, 64, 32, 2)
    _say("[f32_stream] generating")
    bt = gen_batch(wl)
    oi = H.oracle_index(bt)
    db = H.device_batch(bt)
    cen, lst = oi.padded(wl)
    idx = ck.ctkvr_index_load(H.params_of(wl), db.ctx_lens, cen, lst)
    st = H.run_decode_parity(bt, oi, idx, db)
    _say(f"[f32_stream] ok {st}")
    ck.ctkvr_free(idx)
