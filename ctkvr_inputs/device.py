"""Device-side glue for the seeded inputs: uploads a generated batch to the GPU and
fills the library's parameter block from a workload.  No arithmetic of the method
lives here, and nothing here touches the CPU checker; torch and the binding are
imported when a function is called, so that importing the generators stays cheap."""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from . import Batch, Workload


def torch_dtype(wl: Workload):
    import torch
    return torch.bfloat16 if wl.dtype == "bf16" else torch.float32


def to_dev(x: np.ndarray, wl: Workload):
    """fp32 values (exactly representable in the workload dtype) -> device tensor of that dtype."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).to(device="cuda", dtype=torch_dtype(wl))


def params_of(wl: Workload, **over):
    import paper_2512_15550_amd as ck
    p = ck.Params(batch=wl.batch, n_q_heads=wl.h, n_kv_heads=wl.g, head_dim=wl.d, page_size=wl.page_size,
                  dtype=ck.BF16 if wl.dtype == "bf16" else ck.F32, n_centroids=wl.n_centroids,
                  centroid_div=wl.centroid_div, list_len=wl.list_len, n_probe=wl.n_probe, top_k=wl.top_k)
    for k, v in over.items():
        setattr(p, k, v)
    return p


@dataclass
class DeviceBatch:
    k_pages: object
    v_pages: object
    block_table: object
    q_prefill: object       # concatenated tails [sum C_i][h][d]
    cu_seqlens: np.ndarray
    ctx_lens: np.ndarray


def device_batch(bt: Batch) -> DeviceBatch:
    import torch
    wl = bt.wl
    tails = [sq.q_tail[sq.q_tail.shape[0] - wl.centroids_of(sq.s):] for sq in bt.seqs]
    cu = np.zeros(len(tails) + 1, np.int32)
    cu[1:] = np.cumsum([t.shape[0] for t in tails])
    return DeviceBatch(k_pages=to_dev(bt.paged.k_pages, wl), v_pages=to_dev(bt.paged.v_pages, wl),
                       block_table=torch.from_numpy(bt.paged.block_table).cuda(),
                       q_prefill=to_dev(np.concatenate(tails, axis=0), wl), cu_seqlens=cu,
                       ctx_lens=bt.paged.ctx_lens.copy())


def device_full_queries(bt: Batch):
    """All prompt queries of every sequence (needs gen_batch(..., full_walk=True)) as one
    device tensor [sum s_i][h][d] plus the HOST cu_seqlens the k-means centroid mode takes."""
    wl = bt.wl
    cu = np.zeros(len(bt.seqs) + 1, np.int32)
    cu[1:] = np.cumsum([sq.s for sq in bt.seqs])
    return to_dev(np.concatenate([sq.q_full for sq in bt.seqs], axis=0), wl), cu
