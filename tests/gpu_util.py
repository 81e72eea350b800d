"""Helpers for the GPU parity tests: move a seeded workload to the device, call the HIP
path through the C ABI binding, bring the result back as float64."""
from __future__ import annotations

import numpy as np
import torch

import kvc_workloads as W

BF16_TOL = 2e-2   # max-abs error allowed against the fp64 oracle, bf16 tensors
F32_TOL = 1e-5    # same, fp32 tensors


def dev_tensor(a: np.ndarray, dtype: str) -> torch.Tensor:
    if dtype == W.BF16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def to_device(w: W.PagedWorkload):
    return dict(q=dev_tensor(w.q, w.dtype), k=dev_tensor(w.k_cache, w.dtype),
                v=dev_tensor(w.v_cache, w.dtype),
                tables=torch.from_numpy(w.block_tables).cuda(),
                lens=torch.from_numpy(w.context_lens).cuda())


def out_to_f64(out: torch.Tensor) -> np.ndarray:
    return out.float().cpu().numpy().astype(np.float64)


def out_bits(out: torch.Tensor) -> np.ndarray:
    if out.dtype == torch.bfloat16:
        return out.view(torch.int16).cpu().numpy()
    return out.view(torch.int32).cpu().numpy()


def run_gpu(w: W.PagedWorkload, d=None, *, tight: bool = True, **opts) -> torch.Tensor:
    import paper_2503_13773_amd as K
    d = d or to_device(w)
    if tight and "max_context_len" not in opts:
        opts["max_context_len"] = max(1, w.max_context_len)
    out = K.paged_attention_decode(d["q"], d["k"], d["v"], d["tables"], d["lens"], w.scale, **opts)
    torch.cuda.synchronize()
    return out


def tol_of(w: W.PagedWorkload) -> float:
    return F32_TOL if w.dtype == W.F32 else BF16_TOL
