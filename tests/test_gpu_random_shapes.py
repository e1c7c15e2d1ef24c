"""GPU parity on seeded random geometries: group sizes, ragged batches, centroid counts fixed or by divisor, probe
counts on both sides of the selection routes' switch points, list lengths that are and are not multiples of four,
budgets below and above the number of recalled keys, both storage types.  Every case is a valid input inside the
documented limits; the integers must equal the oracle's bit for bit and the outputs lie within the tolerance."""
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


def _cases(n, seed):
    rng = np.random.Generator(np.random.Philox(seed))
    out = []
    for i in range(n):
        g = int(rng.choice([1, 2, 4]))
        G = int(rng.choice([1, 2, 4, 8]))
        B = int(rng.choice([1, 1, 2, 3, 5]))
        lens = tuple(int(x) for x in rng.integers(600, 9000, B))
        s_min = min(lens)
        if rng.random() < 0.5:
            C, div = int(rng.integers(8, min(600, s_min // 2))), 0
        else:
            C, div = 0, int(rng.choice([16, 40, 64]))
        c_min = C if C else s_min // div
        n_probe = int(min(c_min, rng.choice([1, 3, 4, 8, 9, 17, 40])))
        rho = int(min(s_min, rng.choice([16, 50, 77, 128, 300])))
        top_k = int(rng.choice([1, 20, 64, 150, 500, 2000]))
        dtype = "f32" if rng.random() < 0.2 else "bf16"
        out.append((f"rnd{i}_b{B}_g{g}x{G}_C{C or ('s/%d' % div)}_p{n_probe}_r{rho}_k{top_k}_{dtype}", dtype, g * G, g, lens,
                    tuple(range(7000 + 10 * i, 7000 + 10 * i + B)), C, div, n_probe, rho, top_k, 2))
    return out


CASES = _cases(28, 20251128)


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_random_geometry_matches_the_oracle(ck, case):
    name, dtype, h, g, lens, seeds, C, div, n_probe, rho, top_k, steps = case
    print(f"[random {name}] lens {lens}", flush=True)
    wl = small_workload(name, dtype, h, g, lens, seeds, C, div, n_probe, rho, top_k, steps)
    bt = gen_batch(wl)
    db = H.device_batch(bt)
    oi = H.oracle_index(bt)
    idx = ck.ctkvr_build_index(H.params_of(wl), db.q_prefill, db.cu_seqlens, True, db.k_pages, db.block_table, db.ctx_lens)
    lists = ck.ctkvr_index_lists(idx)
    for b, l in enumerate(oi.lists):
        assert np.array_equal(lists[b, :, :l.shape[1]], l), f"sequence {b}: lists differ"
    st = H.run_decode_parity(bt, oi, idx, db, update=(top_k != rho and len(lens) < 3))
    print(f"[random {name}] ok {st}", flush=True)
    ck.ctkvr_index_check(idx)
    ck.ctkvr_free(idx)
