"""GPU test of ctkvr_decode_step_static, the decode step on the library's static scratch array
(for callers that cannot allocate): its results must equal ctkvr_decode_step's on the same index
and inputs -- integers bit for bit, outputs bit for bit too (the same kernels run on the same data) --
on two calls in a row that share the array, the second for a smaller index, and then again for the
first.  Geometries beyond the array are refused on the host."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

import paper_2512_15550_amd as ck
from ctkvr_inputs import gen_batch, small_workload
from ctkvr_inputs.device import device_batch, params_of, to_dev


def _setup(name, dtype, h, g, ctx, seeds, C, n_probe, rho, top_k, n_decode):
    wl = small_workload(name, dtype, h, g, ctx, seeds, C, 0, n_probe, rho, top_k, n_decode)
    bt = gen_batch(wl)
    db = device_batch(bt)
    idx = ck.ctkvr_build_index(params_of(wl), db.q_prefill, db.cu_seqlens, True, db.k_pages, db.block_table, db.ctx_lens)
    return wl, bt, db, idx


def _step(fn, wl, bt, db, idx, st):
    B, h, g, d = wl.batch, wl.h, wl.g, wl.d
    out = torch.full((B, h, d), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((B, h), float("nan"), dtype=torch.float32, device="cuda")
    sel = torch.full((B, g, wl.top_k), -5, dtype=torch.int32, device="cuda")
    ncand = torch.full((B, g), -5, dtype=torch.int32, device="cuda")
    probe = torch.full((B, g, wl.n_probe), -5, dtype=torch.int32, device="cuda")
    q = to_dev(np.stack([sq.q_decode[st] for sq in bt.seqs]), wl)
    fn(idx, q, db.k_pages, db.v_pages, db.block_table, out, lse, sel, ncand, probe)
    torch.cuda.synchronize()
    return [t.cpu().numpy() for t in (out, lse, sel, ncand, probe)]


def _same(a, b, tag):
    names = ("out", "lse", "sel", "ncand", "probe")
    for x, y, n in zip(a, b, names):
        assert np.array_equal(x, y), f"{tag}: {n} differs between the static-scratch step and ctkvr_decode_step"
    assert np.all(np.isfinite(a[0])) and np.all(a[3] > 0)


def test_static_scratch_step_equals_the_allocating_one_twice_in_a_row():
    big = _setup("static_big", "bf16", 8, 2, (6000, 4111), (11, 12), 96, 8, 200, 160, 2)
    small = _setup("static_small", "bf16", 4, 1, (1500,), (13,), 24, 4, 64, 48, 2)
    try:
        for rnd in range(2):
            for name, (wl, bt, db, idx) in (("big", big), ("small", small)):
                for st in range(2):
                    ref = _step(ck.ctkvr_decode_step, wl, bt, db, idx, st)
                    got = _step(ck.ctkvr_decode_step_static, wl, bt, db, idx, st)
                    _same(got, ref, f"round {rnd} {name} step {st}")
    finally:
        ck.ctkvr_free(big[3])
        ck.ctkvr_free(small[3])


def test_static_scratch_step_fp32_and_wide_group():
    a = _setup("static_f32", "f32", 8, 2, (3000,), (21,), 40, 6, 128, 100, 1)
    b = _setup("static_g8", "bf16", 8, 1, (2500, 900), (22, 23), 32, 5, 96, 64, 1)
    try:
        for name, (wl, bt, db, idx) in (("f32", a), ("g8", b), ("f32 again", a)):
            ref = _step(ck.ctkvr_decode_step, wl, bt, db, idx, 0)
            got = _step(ck.ctkvr_decode_step_static, wl, bt, db, idx, 0)
            _same(got, ref, name)
    finally:
        ck.ctkvr_free(a[3])
        ck.ctkvr_free(b[3])


def test_geometry_beyond_the_scratch_is_refused_before_any_launch():
    # 4 sequences of 100K tokens, 64 probes of 2048 ids: the step's buffers take far more than 16 MiB.
    # No data is needed to be refused: an all-zero index and cache (loaded, not built) do.
    B, h, g, s, C, n_probe, rho = 4, 8, 2, 100000, 64, 64, 2048
    p = ck.Params(batch=B, n_q_heads=h, n_kv_heads=g, n_centroids=C, list_len=rho, n_probe=n_probe, top_k=2048)
    lists = np.broadcast_to(np.arange(rho, dtype=np.int32), (B, g, C, rho))
    idx = ck.ctkvr_index_load(p, [s] * B, np.zeros((B, h, C, 128), np.uint16), lists)
    try:
        n_pages = (s + 15) // 16
        bt = torch.arange(B * n_pages, dtype=torch.int32, device="cuda").reshape(B, n_pages)
        kv = torch.zeros((B * n_pages, g, 16, 128), dtype=torch.bfloat16, device="cuda")
        out = torch.zeros((B, h, 128), dtype=torch.float32, device="cuda")
        q = torch.ones((B, h, 128), dtype=torch.bfloat16, device="cuda")
        with pytest.raises(ck.CtkvrError) as ei:
            ck.ctkvr_decode_step_static(idx, q, kv, kv, bt, out)
        assert ei.value.code == -4 and "static scratch" in str(ei.value)
        torch.cuda.synchronize()
        assert not out.any()
        ncand = torch.zeros((B, g), dtype=torch.int32, device="cuda")
        ck.ctkvr_decode_step(idx, q, kv, kv, bt, out, out_ncand=ncand)   # the allocating step still serves it
        torch.cuda.synchronize()
        assert int(ncand.min()) == rho and int(ncand.max()) == rho
    finally:
        ck.ctkvr_free(idx)
