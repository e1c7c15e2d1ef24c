"""Full-size, sampled GPU parity for the rows that follow the core path, in the launch shape of the
128K benchmark workload (4 sequences of 131072 tokens, 32 query / 8 KV heads, C = 2048, C' = 64,
rho = rho' = 2048): the resident window with its merge (Algorithm 1 lines 5-6, Algorithm 2 lines
10-11; L_init = 128, L_local = 512) and the dynamic centroid update after every step (Algorithm 2
line 12).  The oracle rebuilds exactly the lists each step probes."""
import pytest

from ctkvr_inputs import gen_batch, workload
from tests import harness as H

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module")
def ck():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2512_15550_amd as ck
    ck.load_library()
    return ck


@pytest.fixture(scope="module")
def cfg3(ck):
    wl = workload("cfg3")
    _say("[cfg3 next rows] generating inputs")
    bt = gen_batch(wl, n_decode=4)
    return wl, bt, H.device_batch(bt)


def test_resident_window_at_128k_sampled(ck, cfg3):
    wl, bt, db = cfg3
    n_init, n_local = 128, 512
    _say("[cfg3 window] GPU index build without the window's keys")
    idx = ck.ctkvr_build_index(H.params_of(wl, n_init=n_init, n_local=n_local), db.q_prefill, db.cu_seqlens, True,
                               db.k_pages, db.block_table, db.ctx_lens)
    st = H.run_sampled_parity_next(bt, idx, db, [0, 3], n_init=n_init, n_local=n_local, say=_say)
    _say(f"[cfg3 window] ok {st}")
    ck.ctkvr_free(idx)


def test_centroid_update_at_128k_sampled(ck, cfg3):
    wl, bt, db = cfg3
    _say("[cfg3 update] GPU index build")
    idx = ck.ctkvr_build_index(H.params_of(wl), db.q_prefill, db.cu_seqlens, True, db.k_pages, db.block_table, db.ctx_lens)
    st = H.run_sampled_parity_next(bt, idx, db, [0, 1, 2, 3], update=True, say=_say)
    assert st["updates"] == 4
    _say(f"[cfg3 update] ok {st}")
    ck.ctkvr_free(idx)
