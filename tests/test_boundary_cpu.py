"""The C-ABI library without a GPU: it loads, exports every symbol the header
declares, and rejects bad arguments on the host before touching the device."""
import ctypes
import os
import re

import pytest

import paper_2512_15550_amd as ck
from paper_2512_15550_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "ctkvr.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ctkvr_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ck.load_library()
    names = _declared()
    assert "ctkvr_build_index" in names and "ctkvr_decode_step" in names and "ctkvr_free" in names
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_params_struct_matches_header_layout():
    assert ctypes.sizeof(binding._CParams) == 17 * 4
    assert ctypes.sizeof(binding._CInfo) == 10 * 4 + 2 * 8


def _build_rc(p, ctx):
    lib = ck.load_library()
    cp = p.c()
    arr = (ctypes.c_int32 * len(ctx))(*ctx)
    out = ctypes.c_void_p()
    one = (ctypes.c_int32 * 4)(0, 8, 0, 0)
    dummy = ctypes.c_void_p(1)   # never dereferenced: every case below fails validation first
    return lib.ctkvr_build_index(ctypes.byref(cp), dummy, one, 1, dummy, dummy, 1 << 20, arr, None, None,
                                 ctypes.byref(out)), out


@pytest.mark.parametrize("change,code", [
    (dict(head_dim=64), -4), (dict(n_q_heads=6, n_kv_heads=2), -4), (dict(n_q_heads=7), -1),
    (dict(n_probe=9), -1), (dict(list_len=5000), -1), (dict(top_k=0), -1), (dict(page_size=12), -4),
    (dict(dtype=7), -1), (dict(n_centroids=0, centroid_div=0), -1), (dict(sm_scale=-1.0), -1),
    (dict(n_init=-1), -1), (dict(n_init=2000, n_local=2040), -1),   # the window leaves fewer than list_len keys
])
def test_bad_parameters_are_rejected_on_the_host(change, code):
    base = dict(batch=1, n_q_heads=8, n_kv_heads=2, n_centroids=8, list_len=64, n_probe=4, top_k=32)
    base.update(change)
    rc, out = _build_rc(ck.Params(**base), [4096])
    assert rc == code and not out.value
    assert ck.ctkvr_last_error()


def test_null_arguments():
    lib = ck.load_library()
    assert lib.ctkvr_decode_step(None, None, None, None, None, 0, None, None, None, None, None, None) == -1
    assert "NULL" in ck.ctkvr_last_error()
    lib.ctkvr_free(None)   # allowed
    assert lib.ctkvr_index_info(None, None) == -1


def test_new_entry_points_reject_null_arguments():
    lib = ck.load_library()
    assert lib.ctkvr_decode_step_window(None, None, None, None, None, 0, None, None, None, None, None, None, None) == -1
    assert lib.ctkvr_centroid_update(None, None, None) == -1
    assert lib.ctkvr_selftest_exp(None, None) == -1
    assert "NULL" in ck.ctkvr_last_error()


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr
