"""ctypes binding of ``libctkvr.so`` -- argument marshalling only.

Device arguments are torch tensors (used for their memory and for the current
HIP stream); host arguments are numpy arrays.  Function names are the C ABI's.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libctkvr.so")

F32, BF16 = 0, 1
LAST_C, KMEANS = 0, 1
BUILD_EXACT, BUILD_MFMA = 0, 1

_STATUS = {0: "OK", -1: "EINVAL", -2: "ENOMEM", -3: "EHIP", -4: "EUNSUPPORTED"}


class CtkvrError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"ctkvr: {_STATUS.get(code, code)}: {msg}")
        self.code = code


class _CParams(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("page_size", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("n_centroids", ctypes.c_int32), ("centroid_div", ctypes.c_int32), ("list_len", ctypes.c_int32),
                ("n_probe", ctypes.c_int32), ("top_k", ctypes.c_int32), ("sm_scale", ctypes.c_float),
                ("centroid_mode", ctypes.c_int32), ("kmeans_iters", ctypes.c_int32), ("build_algo", ctypes.c_int32),
                ("n_init", ctypes.c_int32), ("n_local", ctypes.c_int32)]


class _CInfo(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32), ("c_max", ctypes.c_int32),
                ("list_len", ctypes.c_int32), ("n_probe", ctypes.c_int32), ("top_k", ctypes.c_int32),
                ("l_stride", ctypes.c_int32), ("index_bytes", ctypes.c_int64), ("device_bytes", ctypes.c_int64)]


@dataclass
class Params:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int = 128
    page_size: int = 16
    dtype: int = BF16
    n_centroids: int = 0
    centroid_div: int = 0
    list_len: int = 0
    n_probe: int = 0
    top_k: int = 0
    sm_scale: float = 0.0
    centroid_mode: int = LAST_C
    kmeans_iters: int = 0
    build_algo: int = BUILD_EXACT
    n_init: int = 0
    n_local: int = 0

    def c(self) -> _CParams:
        return _CParams(self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim, self.page_size, self.dtype,
                        self.n_centroids, self.centroid_div, self.list_len, self.n_probe, self.top_k,
                        float(self.sm_scale), self.centroid_mode, self.kmeans_iters, self.build_algo, self.n_init,
                        self.n_local)


_lib = None

EXPORTS = ["ctkvr_build_index", "ctkvr_index_load", "ctkvr_decode_step", "ctkvr_free", "ctkvr_last_error",
           "ctkvr_index_info", "ctkvr_index_lists", "ctkvr_index_centroids", "ctkvr_index_last_candidates",
           "ctkvr_profile_enable", "ctkvr_profile_collect", "ctkvr_centroid_update", "ctkvr_decode_step_window",
           "ctkvr_selftest_exp", "ctkvr_decode_step_static", "ctkvr_index_set_decode_path", "ctkvr_index_decode_path",
           "ctkvr_index_check", "ctkvr_profile_phases", "ctkvr_measure_dispatch_floor", "ctkvr_index_build_route", "ctkvr_release_scratch"]
PATH_AUTO, PATH_STAGED, PATH_FUSED = 0, 1, 2
N_STAGES = 9
STAGE_NAMES = ["centroid_cos", "recall_gather", "score", "denom", "keyhist", "classify",
               "rerank_select", "sparse_attn", "null"]


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load ``libctkvr.so``; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2512_15550_amd.build` "
                          "(or __graft_entry__.build()); there is no fallback path")
    L = ctypes.CDLL(_LIB_PATH)
    vp, ip, fp = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
    L.ctkvr_last_error.restype = ctypes.c_char_p
    L.ctkvr_build_index.restype = ctypes.c_int
    L.ctkvr_build_index.argtypes = [ctypes.POINTER(_CParams), vp, ip, ctypes.c_int32, vp, ip, ctypes.c_int32, ip, ip,
                                    vp, ctypes.POINTER(ctypes.c_void_p)]
    L.ctkvr_index_load.restype = ctypes.c_int
    L.ctkvr_index_load.argtypes = [ctypes.POINTER(_CParams), ip, vp, ip, vp, ctypes.POINTER(ctypes.c_void_p)]
    L.ctkvr_decode_step.restype = ctypes.c_int
    L.ctkvr_decode_step.argtypes = [vp, vp, vp, vp, ip, ctypes.c_int32, fp, fp, ip, ip, ip, vp]
    L.ctkvr_decode_step_static.restype = ctypes.c_int
    L.ctkvr_decode_step_static.argtypes = L.ctkvr_decode_step.argtypes
    L.ctkvr_decode_step_window.restype = ctypes.c_int
    L.ctkvr_decode_step_window.argtypes = [vp, vp, vp, vp, ip, ctypes.c_int32, ip, fp, fp, ip, ip, ip, vp]
    L.ctkvr_centroid_update.restype = ctypes.c_int
    L.ctkvr_centroid_update.argtypes = [vp, vp, vp]
    L.ctkvr_free.restype = None
    L.ctkvr_free.argtypes = [vp]
    L.ctkvr_index_info.restype = ctypes.c_int
    L.ctkvr_index_info.argtypes = [vp, ctypes.POINTER(_CInfo)]
    for name in ("ctkvr_index_lists", "ctkvr_index_centroids", "ctkvr_index_last_candidates"):
        getattr(L, name).restype = ctypes.c_int
        getattr(L, name).argtypes = [vp, vp]
    L.ctkvr_profile_enable.restype = ctypes.c_int
    L.ctkvr_profile_enable.argtypes = [vp, ctypes.c_int32]
    L.ctkvr_profile_collect.restype = ctypes.c_int
    L.ctkvr_profile_collect.argtypes = [vp, vp, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)]
    L.ctkvr_index_set_decode_path.restype = ctypes.c_int
    L.ctkvr_index_set_decode_path.argtypes = [vp, ctypes.c_int32]
    L.ctkvr_index_decode_path.restype = ctypes.c_int
    L.ctkvr_index_decode_path.argtypes = [vp]
    L.ctkvr_index_check.restype = ctypes.c_int
    L.ctkvr_index_check.argtypes = [vp]
    L.ctkvr_release_scratch.restype = ctypes.c_int
    L.ctkvr_release_scratch.argtypes = []
    L.ctkvr_index_build_route.restype = ctypes.c_int
    L.ctkvr_index_build_route.argtypes = [vp, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
    L.ctkvr_profile_phases.restype = ctypes.c_int
    L.ctkvr_profile_phases.argtypes = [vp, ctypes.c_int32, vp]
    L.ctkvr_measure_dispatch_floor.restype = ctypes.c_int
    L.ctkvr_measure_dispatch_floor.argtypes = [ctypes.c_int32, ctypes.POINTER(ctypes.c_float), vp]
    L.ctkvr_selftest_exp.restype = ctypes.c_int
    L.ctkvr_selftest_exp.argtypes = [ctypes.POINTER(ctypes.c_uint64), vp]
    _lib = L
    return L


def ctkvr_last_error() -> str:
    return load_library().ctkvr_last_error().decode()


def _check(rc: int) -> None:
    if rc != 0:
        raise CtkvrError(rc, ctkvr_last_error())


def _dev(t, dtype=None) -> Optional[int]:
    """Device pointer of a contiguous CUDA/HIP torch tensor (None passes NULL)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    return t.data_ptr()


def _host_i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.int32)


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _torch_dtype(dtype: int):
    import torch
    return torch.bfloat16 if dtype == BF16 else torch.float32


class Index:
    """Owner of a ``ctkvr_index*``; freed on ``ctkvr_free`` or garbage collection."""

    def __init__(self, handle: int, params: Params):
        self.handle = handle
        self.params = params

    def __del__(self):
        try:
            ctkvr_free(self)
        except Exception:
            pass


def ctkvr_build_index(params: Params, q_prefill, cu_seqlens, q_is_tail: bool, k_pages, block_table, ctx_lens,
                      init_pos=None) -> Index:
    import torch
    L = load_library()
    cu = _host_i32(cu_seqlens)
    cl = _host_i32(ctx_lens)
    td = _torch_dtype(params.dtype)
    out = ctypes.c_void_p()
    cp = params.c()
    rc = L.ctkvr_build_index(ctypes.byref(cp), _dev(q_prefill, td), cu.ctypes.data, int(bool(q_is_tail)),
                             _dev(k_pages, td), _dev(block_table, torch.int32), int(block_table.shape[1]),
                             cl.ctypes.data, _dev(init_pos, torch.int32) if init_pos is not None else None, _stream(),
                             ctypes.byref(out))
    _check(rc)
    return Index(out.value, params)


def ctkvr_index_load(params: Params, ctx_lens, centroids: np.ndarray, lists: np.ndarray) -> Index:
    """centroids: host array [batch][h][C_max][d], uint16 bit patterns for bf16 or float32; lists int32."""
    L = load_library()
    cl = _host_i32(ctx_lens)
    want = np.uint16 if params.dtype == BF16 else np.float32
    cen = np.ascontiguousarray(centroids)
    if cen.dtype != want:
        raise ValueError(f"centroids must be {want}")
    li = _host_i32(lists)
    out = ctypes.c_void_p()
    cp = params.c()
    rc = L.ctkvr_index_load(ctypes.byref(cp), cl.ctypes.data, cen.ctypes.data, li.ctypes.data, _stream(),
                            ctypes.byref(out))
    _check(rc)
    return Index(out.value, params)


def ctkvr_decode_step(idx: Index, q, k_pages, v_pages, block_table, out, out_lse=None, out_sel=None, out_ncand=None,
                      out_probe=None) -> None:
    import torch
    L = load_library()
    td = _torch_dtype(idx.params.dtype)
    rc = L.ctkvr_decode_step(idx.handle, _dev(q, td), _dev(k_pages, td), _dev(v_pages, td),
                             _dev(block_table, torch.int32), int(block_table.shape[1]), _dev(out, torch.float32),
                             _dev(out_lse, torch.float32), _dev(out_sel, torch.int32), _dev(out_ncand, torch.int32),
                             _dev(out_probe, torch.int32), _stream())
    _check(rc)


def ctkvr_decode_step_static(idx: Index, q, k_pages, v_pages, block_table, out, out_lse=None, out_sel=None,
                             out_ncand=None, out_probe=None) -> None:
    """The decode step on the library's static scratch array (allocates nothing)."""
    import torch
    L = load_library()
    td = _torch_dtype(idx.params.dtype)
    rc = L.ctkvr_decode_step_static(idx.handle, _dev(q, td), _dev(k_pages, td), _dev(v_pages, td),
                                    _dev(block_table, torch.int32), int(block_table.shape[1]), _dev(out, torch.float32),
                                    _dev(out_lse, torch.float32), _dev(out_sel, torch.int32),
                                    _dev(out_ncand, torch.int32), _dev(out_probe, torch.int32), _stream())
    _check(rc)


def ctkvr_decode_step_window(idx: Index, q, k_pages, v_pages, block_table, cur_lens, out, out_lse=None, out_sel=None,
                             out_ncand=None, out_probe=None) -> None:
    """cur_lens: device int32 [batch] (tokens now in the cache) or None."""
    import torch
    L = load_library()
    td = _torch_dtype(idx.params.dtype)
    rc = L.ctkvr_decode_step_window(idx.handle, _dev(q, td), _dev(k_pages, td), _dev(v_pages, td),
                                    _dev(block_table, torch.int32), int(block_table.shape[1]),
                                    _dev(cur_lens, torch.int32), _dev(out, torch.float32), _dev(out_lse, torch.float32),
                                    _dev(out_sel, torch.int32), _dev(out_ncand, torch.int32),
                                    _dev(out_probe, torch.int32), _stream())
    _check(rc)


def ctkvr_centroid_update(idx: Index, q) -> None:
    td = _torch_dtype(idx.params.dtype)
    _check(load_library().ctkvr_centroid_update(idx.handle, _dev(q, td), _stream()))


def ctkvr_free(idx: Optional[Index]) -> None:
    if idx is not None and idx.handle:
        load_library().ctkvr_free(idx.handle)
        idx.handle = 0


def ctkvr_index_info(idx: Index) -> dict:
    info = _CInfo()
    _check(load_library().ctkvr_index_info(idx.handle, ctypes.byref(info)))
    return {name: getattr(info, name) for name, _ in _CInfo._fields_}


def ctkvr_index_lists(idx: Index) -> np.ndarray:
    i = ctkvr_index_info(idx)
    out = np.empty((i["batch"], i["n_kv_heads"], i["c_max"], i["list_len"]), np.int32)
    _check(load_library().ctkvr_index_lists(idx.handle, out.ctypes.data))
    return out


def ctkvr_index_centroids(idx: Index) -> np.ndarray:
    i = ctkvr_index_info(idx)
    out = np.empty((i["batch"], i["n_q_heads"], i["c_max"], i["head_dim"]),
                   np.uint16 if i["dtype"] == BF16 else np.float32)
    _check(load_library().ctkvr_index_centroids(idx.handle, out.ctypes.data))
    return out


def ctkvr_index_last_candidates(idx: Index) -> np.ndarray:
    i = ctkvr_index_info(idx)
    out = np.empty((i["batch"], i["n_kv_heads"], i["l_stride"]), np.int32)
    _check(load_library().ctkvr_index_last_candidates(idx.handle, out.ctypes.data))
    return out


def ctkvr_profile_enable(idx: Index, max_steps: int) -> None:
    _check(load_library().ctkvr_profile_enable(idx.handle, int(max_steps)))


def ctkvr_profile_collect(idx: Index, capacity_steps: int) -> np.ndarray:
    """ms per (step, stage) for the steps recorded since the last collect."""
    out = np.zeros((capacity_steps, N_STAGES), np.float32)
    n = ctypes.c_int32(0)
    _check(load_library().ctkvr_profile_collect(idx.handle, out.ctypes.data, int(capacity_steps), ctypes.byref(n)))
    return out[:n.value]


def ctkvr_selftest_exp() -> int:
    """Number of fp32 inputs in [-32, 0] on which the library's two forms of the fixed-point exponential differ."""
    n = ctypes.c_uint64(0)
    _check(load_library().ctkvr_selftest_exp(ctypes.byref(n), _stream()))
    return int(n.value)


def ctkvr_index_set_decode_path(idx: Index, path: int) -> None:
    """PATH_AUTO, PATH_STAGED (one launch per stage) or PATH_FUSED (the whole step in one launch)."""
    _check(load_library().ctkvr_index_set_decode_path(idx.handle, int(path)))


def ctkvr_index_decode_path(idx: Index) -> int:
    rc = load_library().ctkvr_index_decode_path(idx.handle)
    if rc < 0:
        _check(rc)
    return rc


def ctkvr_index_build_route(idx: Index):
    """(built by the candidate route?, chunks it handed back to the route that ranks every key)."""
    a, b = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(load_library().ctkvr_index_build_route(idx.handle, ctypes.byref(a), ctypes.byref(b)))
    return bool(a.value), int(b.value)


def ctkvr_release_scratch() -> None:
    """Frees the device scratch the matrix-core list build keeps between builds (current device)."""
    _check(load_library().ctkvr_release_scratch())


def ctkvr_index_check(idx: Index) -> None:
    """Synchronises; raises if a single-launch step on this index gave up a wait."""
    _check(load_library().ctkvr_index_check(idx.handle))


def ctkvr_profile_phases(idx: Index, enable: bool = True) -> np.ndarray:
    """The 16 wall-clock stamps (100 MHz ticks) of the last single-launch step's first block (0-7 leaving each
    phase, 8-13 arriving at each barrier); sets stamping on or off."""
    out = np.zeros(64, np.int64)
    _check(load_library().ctkvr_profile_phases(idx.handle, int(bool(enable)), out.ctypes.data))
    return out


def ctkvr_measure_dispatch_floor(n_launches: int = 200) -> float:
    """Microseconds per launch of a graph of empty kernels launched one behind the other."""
    us = ctypes.c_float(0.0)
    _check(load_library().ctkvr_measure_dispatch_floor(int(n_launches), ctypes.byref(us), _stream()))
    return float(us.value)
