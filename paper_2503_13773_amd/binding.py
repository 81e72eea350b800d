"""ctypes binding of the C ABI in include/kvc.h (same names, argument marshalling only)."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch  # device memory and streams; also makes sure one HIP runtime is shared

KVC_F32, KVC_BF16 = 0, 1
KERNEL_AUTO, KERNEL_VALU, KERNEL_MFMA, KERNEL_MFMA_LDS, KERNEL_MFMA_BALANCED = 0, 1, 2, 3, 4

_PKG = os.path.dirname(os.path.abspath(__file__))
# KVC_HIP_LIBRARY points at another build of the same library (A/B comparisons of kernels)
_LIB_PATH = os.environ.get("KVC_HIP_LIBRARY") or os.path.join(_PKG, "libkvc_hip.so")
_lib = None


class KvcError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status}, hip error "
                         f"{lib().kvc_last_hip_error()})")


class AttnDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "num_seqs", "num_q_heads", "num_kv_heads", "head_dim", "block_size",
        "max_blocks_per_seq", "num_pool_blocks", "dtype", "max_context_len",
        "partition_tokens", "kernel", "reserved")]


class AttnPlan(ctypes.Structure):
    _fields_ = [("kernel", ctypes.c_int32), ("partition_tokens", ctypes.c_int32),
                ("max_partitions", ctypes.c_int32), ("partial_grid", ctypes.c_int32),
                ("merge_grid", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("workspace_bytes", ctypes.c_uint64)]


class Pool(ctypes.Structure):
    _fields_ = [("base", ctypes.c_void_p), ("num_blocks", ctypes.c_int64),
                ("block_bytes", ctypes.c_int64), ("plane_stride_bytes", ctypes.c_int64),
                ("num_planes", ctypes.c_int32), ("reserved", ctypes.c_int32)]


def library_path() -> str:
    return _LIB_PATH


def lib():
    """Load libkvc_hip.so (built in-tree by paper_2503_13773_amd.build).  No fallback."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: run `python -m paper_2503_13773_amd.build` "
                           "(there is no CPU fallback)")
    L = ctypes.CDLL(_LIB_PATH)
    vp, i32p, f, sz = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float, ctypes.c_size_t
    dp = ctypes.POINTER(AttnDesc)
    pp = ctypes.POINTER(Pool)
    L.kvc_version.restype = ctypes.c_int
    L.kvc_status_string.restype = ctypes.c_char_p
    L.kvc_status_string.argtypes = [ctypes.c_int]
    L.kvc_last_hip_error.restype = ctypes.c_int
    L.kvc_attn_plan.restype = ctypes.c_int
    L.kvc_attn_plan.argtypes = [dp, ctypes.POINTER(AttnPlan)]
    L.kvc_paged_attention_decode_workspace_bytes.restype = sz
    L.kvc_paged_attention_decode_workspace_bytes.argtypes = [dp]
    for name in ("kvc_paged_attention_decode", "kvc_paged_attention_decode_partial"):
        fn = getattr(L, name)
        fn.restype = ctypes.c_int
        fn.argtypes = [vp, vp, vp, i32p, i32p, f, vp, dp, vp, sz, vp]
    L.kvc_paged_attention_decode_workspace_init.restype = ctypes.c_int
    L.kvc_paged_attention_decode_workspace_init.argtypes = [vp, sz, vp]
    L.kvc_attn_schedule_bytes.restype = sz
    L.kvc_attn_schedule_bytes.argtypes = [dp]
    L.kvc_attn_schedule_build.restype = ctypes.c_int
    L.kvc_attn_schedule_build.argtypes = [i32p, i32p, dp, vp, sz, vp]
    L.kvc_paged_attention_decode_scheduled.restype = ctypes.c_int
    L.kvc_paged_attention_decode_scheduled.argtypes = [vp, vp, vp, vp, sz, f, vp, dp, vp, sz, vp]
    L.kvc_paged_attention_decode_noalloc.restype = ctypes.c_int
    L.kvc_paged_attention_decode_noalloc.argtypes = [vp, vp, vp, i32p, i32p, f, vp, dp, vp]
    L.kvc_paged_attention_decode_merge.restype = ctypes.c_int
    L.kvc_paged_attention_decode_merge.argtypes = [i32p, vp, dp, vp, sz, vp]
    L.kvc_validate_attention_inputs.restype = ctypes.c_int
    L.kvc_validate_attention_inputs.argtypes = [i32p, i32p, dp, vp]
    L.kvc_paged_attention_prefill.restype = ctypes.c_int
    L.kvc_paged_attention_prefill.argtypes = [vp, vp, vp, i32p, i32p, i32p, f, vp, dp, ctypes.c_int32,
                                              ctypes.c_int32, vp]
    L.kvc_kv_cache_append.restype = ctypes.c_int
    L.kvc_kv_cache_append.argtypes = [vp, vp, vp, vp, i32p, i32p, dp, vp]
    L.kvc_kv_block_copy.restype = ctypes.c_int
    L.kvc_kv_block_copy.argtypes = [pp, pp, vp, ctypes.c_int64, vp]
    L.kvc_validate_block_mapping.restype = ctypes.c_int
    L.kvc_validate_block_mapping.argtypes = [pp, pp, vp, ctypes.c_int64, vp]
    _lib = L
    return L


def version() -> int:
    return int(lib().kvc_version())


def status_string(status: int) -> str:
    return lib().kvc_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise KvcError(status, where)


def _stream_handle(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return KVC_F32
    if t.dtype == torch.bfloat16:
        return KVC_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def attn_desc(q, k_cache, block_tables, *, max_context_len: int = 0, partition_tokens: int = 0,
              kernel: int = KERNEL_AUTO) -> AttnDesc:
    """Describe the shapes of a decode call from its tensors."""
    nseq, hq, d = q.shape
    nb, hkv, bs, d2 = k_cache.shape
    if d2 != d:
        raise ValueError("head_dim of q and k_cache differ")
    return AttnDesc(num_seqs=nseq, num_q_heads=hq, num_kv_heads=hkv, head_dim=d, block_size=bs,
                    max_blocks_per_seq=block_tables.shape[1], num_pool_blocks=nb,
                    dtype=_dtype_code(q), max_context_len=int(max_context_len),
                    partition_tokens=int(partition_tokens), kernel=int(kernel), reserved=0)


def attn_plan(desc: AttnDesc) -> AttnPlan:
    plan = AttnPlan()
    _check(lib().kvc_attn_plan(ctypes.byref(desc), ctypes.byref(plan)), "kvc_attn_plan")
    return plan


def workspace_bytes(desc: AttnDesc) -> int:
    return int(lib().kvc_paged_attention_decode_workspace_bytes(ctypes.byref(desc)))


def workspace_init(workspace, stream=None) -> None:
    """Zero the counter header of a workspace tensor (needed once after allocation)."""
    _check(lib().kvc_paged_attention_decode_workspace_init(
        workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream_handle(stream)),
        "kvc_paged_attention_decode_workspace_init")


def new_workspace(desc: AttnDesc, device="cuda", stream=None):
    """Allocate a workspace for `desc` and prepare it (None when the descriptor needs none)."""
    need = workspace_bytes(desc)
    if not need:
        return None
    ws = torch.empty(need, dtype=torch.uint8, device=device)
    workspace_init(ws, stream)
    return ws


def _attn_args(q, k_cache, v_cache, block_tables, context_lens, out, desc, workspace):
    for t in (q, k_cache, v_cache, block_tables, context_lens):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("tensors must be contiguous device tensors")
    if v_cache.shape != k_cache.shape or v_cache.dtype != q.dtype or k_cache.dtype != q.dtype:
        raise ValueError("k_cache / v_cache must match each other and q's dtype")
    if block_tables.dtype != torch.int32 or context_lens.dtype != torch.int32:
        raise TypeError("block_tables and context_lens must be int32")
    if block_tables.shape[0] != q.shape[0] or context_lens.shape != (q.shape[0],):
        raise ValueError("block_tables / context_lens do not match the batch")
    if out is None:
        out = torch.empty_like(q)
    elif out.shape != q.shape or out.dtype != q.dtype or not out.is_cuda or not out.is_contiguous():
        raise ValueError("out must look like q")
    if workspace is False:          # the call brings its own workspace
        return out, None, None, 0
    need = workspace_bytes(desc)
    if workspace is None and need:
        workspace = new_workspace(desc, q.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    return out, workspace, ws_ptr, ws_len


def paged_attention_decode(q, k_cache, v_cache, block_tables, context_lens, scale: float,
                           out=None, *, desc: Optional[AttnDesc] = None, max_context_len: int = 0,
                           partition_tokens: int = 0, kernel: int = KERNEL_AUTO, workspace=None,
                           stream=None):
    """out[n,h] = softmax(scale * q[n,h] . K[n]) V[n] over each sequence's block list."""
    if desc is None:
        desc = attn_desc(q, k_cache, block_tables, max_context_len=max_context_len,
                         partition_tokens=partition_tokens, kernel=kernel)
    out, workspace, ws_ptr, ws_len = _attn_args(q, k_cache, v_cache, block_tables, context_lens,
                                                out, desc, workspace)
    _check(lib().kvc_paged_attention_decode(
        q.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(), block_tables.data_ptr(),
        context_lens.data_ptr(), float(scale), out.data_ptr(), ctypes.byref(desc), ws_ptr, ws_len,
        _stream_handle(stream)), "kvc_paged_attention_decode")
    return out


def schedule_bytes(desc: AttnDesc) -> int:
    return int(lib().kvc_attn_schedule_bytes(ctypes.byref(desc)))


def attn_schedule_build(block_tables, context_lens, desc: AttnDesc, schedule=None, stream=None):
    """Placement of the balanced kernel's workers for (block_tables, context_lens): built once per
    iteration, reused by every layer's paged_attention_decode_scheduled.  Returns the schedule tensor."""
    need = schedule_bytes(desc)
    if schedule is None:
        schedule = torch.empty(max(need, 256), dtype=torch.uint8, device=block_tables.device)
    _check(lib().kvc_attn_schedule_build(block_tables.data_ptr(), context_lens.data_ptr(), ctypes.byref(desc),
                                         schedule.data_ptr(), schedule.numel(), _stream_handle(stream)),
           "kvc_attn_schedule_build")
    return schedule


def paged_attention_decode_scheduled(q, k_cache, v_cache, schedule, scale: float, out, desc: AttnDesc,
                                     workspace, stream=None):
    if out is None:
        out = torch.empty_like(q)
    _check(lib().kvc_paged_attention_decode_scheduled(
        q.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(), schedule.data_ptr(), schedule.numel(), float(scale),
        out.data_ptr(), ctypes.byref(desc), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
        _stream_handle(stream)), "kvc_paged_attention_decode_scheduled")
    return out


NOALLOC_WORKSPACE_BYTES = 32 << 20


def paged_attention_decode_noalloc(q, k_cache, v_cache, block_tables, context_lens, scale: float,
                                   out, desc: AttnDesc, stream=None):
    """kvc_paged_attention_decode_noalloc: the caller passes `out`; nothing is allocated here or
    in the library (the workspace is the library's own fixed per-GPU region)."""
    if out is None:
        raise ValueError("out is required")
    _attn_args(q, k_cache, v_cache, block_tables, context_lens, out, desc, workspace=False)
    _check(lib().kvc_paged_attention_decode_noalloc(
        q.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(), block_tables.data_ptr(),
        context_lens.data_ptr(), float(scale), out.data_ptr(), ctypes.byref(desc),
        _stream_handle(stream)), "kvc_paged_attention_decode_noalloc")
    return out


def paged_attention_decode_partial(q, k_cache, v_cache, block_tables, context_lens, scale: float,
                                   out, desc: AttnDesc, workspace, stream=None):
    out, workspace, ws_ptr, ws_len = _attn_args(q, k_cache, v_cache, block_tables, context_lens,
                                                out, desc, workspace)
    _check(lib().kvc_paged_attention_decode_partial(
        q.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(), block_tables.data_ptr(),
        context_lens.data_ptr(), float(scale), out.data_ptr(), ctypes.byref(desc), ws_ptr, ws_len,
        _stream_handle(stream)), "kvc_paged_attention_decode_partial")
    return out


def paged_attention_decode_merge(context_lens, out, desc: AttnDesc, workspace, stream=None):
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().kvc_paged_attention_decode_merge(
        context_lens.data_ptr(), out.data_ptr(), ctypes.byref(desc), ws_ptr, ws_len,
        _stream_handle(stream)), "kvc_paged_attention_decode_merge")
    return out


def validate_attention_inputs(block_tables, context_lens, desc: AttnDesc, stream=None) -> int:
    """Blocking range check of the index arrays; returns the status (0 = fine)."""
    return int(lib().kvc_validate_attention_inputs(block_tables.data_ptr(), context_lens.data_ptr(),
                                                   ctypes.byref(desc), _stream_handle(stream)))


def paged_attention_prefill(q, k_cache, v_cache, block_tables, context_lens, q_start, scale: float,
                            max_query_len: int, out=None, stream=None, kernel: int = KERNEL_AUTO):
    """Causal attention of the last Qn = q_start[n+1]-q_start[n] positions of every sequence
    (q is [total_q][Hq][D], rows of all sequences back to back) over its block list.
    kernel=KERNEL_MFMA asks for the 16x16-tile matrix-core kernel where AUTO would take 32x32 tiles."""
    for t in (q, k_cache, v_cache, block_tables, context_lens, q_start):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("tensors must be contiguous device tensors")
    if q_start.dtype != torch.int32 or q_start.shape != (context_lens.shape[0] + 1,):
        raise TypeError("q_start must be int32 [num_seqs + 1]")
    if block_tables.dtype != torch.int32 or context_lens.dtype != torch.int32:
        raise TypeError("block_tables and context_lens must be int32")
    if v_cache.shape != k_cache.shape or k_cache.dtype != q.dtype or v_cache.dtype != q.dtype:
        raise ValueError("k_cache / v_cache must match each other and q's dtype")
    total_q, hq, d = q.shape
    nb, hkv, bs, d2 = k_cache.shape
    if d2 != d or block_tables.shape[0] != context_lens.shape[0]:
        raise ValueError("shapes do not match")
    if out is None:
        out = torch.empty_like(q)
    desc = AttnDesc(num_seqs=context_lens.shape[0], num_q_heads=hq, num_kv_heads=hkv, head_dim=d,
                    block_size=bs, max_blocks_per_seq=block_tables.shape[1], num_pool_blocks=nb,
                    dtype=_dtype_code(q), max_context_len=0, partition_tokens=0, kernel=int(kernel),
                    reserved=0)
    _check(lib().kvc_paged_attention_prefill(
        q.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(), block_tables.data_ptr(),
        context_lens.data_ptr(), q_start.data_ptr(), float(scale), out.data_ptr(), ctypes.byref(desc),
        int(total_q), int(max_query_len), _stream_handle(stream)), "kvc_paged_attention_prefill")
    return out


def kv_cache_append(k_new, v_new, k_cache, v_cache, block_tables, positions, stream=None) -> None:
    """Write token positions[n] of every sequence: cache[table[n][pos // Bs]][h][pos % Bs] = new[n][h]."""
    for t in (k_new, v_new, k_cache, v_cache, block_tables, positions):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("tensors must be contiguous device tensors")
    nseq, hkv, d = k_new.shape
    if v_new.shape != k_new.shape or k_cache.shape != v_cache.shape or k_cache.shape[1] != hkv \
            or k_cache.shape[3] != d or not (k_new.dtype == v_new.dtype == k_cache.dtype == v_cache.dtype):
        raise ValueError("k_new / v_new / caches do not match")
    if block_tables.dtype != torch.int32 or positions.dtype != torch.int32 or positions.shape != (nseq,) \
            or block_tables.shape[0] != nseq:
        raise TypeError("block_tables / positions must be int32 and match the batch")
    desc = AttnDesc(num_seqs=nseq, num_q_heads=hkv, num_kv_heads=hkv, head_dim=d,
                    block_size=k_cache.shape[2], max_blocks_per_seq=block_tables.shape[1],
                    num_pool_blocks=k_cache.shape[0], dtype=_dtype_code(k_new), max_context_len=0,
                    partition_tokens=0, kernel=KERNEL_VALU, reserved=0)
    _check(lib().kvc_kv_cache_append(k_new.data_ptr(), v_new.data_ptr(), k_cache.data_ptr(),
                                     v_cache.data_ptr(), block_tables.data_ptr(), positions.data_ptr(),
                                     ctypes.byref(desc), _stream_handle(stream)), "kvc_kv_cache_append")


_hip = None


def _device_pointer_of_pinned(t: torch.Tensor) -> int:
    """Device-side address of a pinned host tensor (asks the HIP runtime; raises if the
    allocation is not mapped into the device address space)."""
    global _hip
    if _hip is None:
        _hip = ctypes.CDLL("libamdhip64.so.7")   # the runtime torch already loaded (same SONAME)
        _hip.hipHostGetDevicePointer.restype = ctypes.c_int
        _hip.hipHostGetDevicePointer.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_void_p,
                                                 ctypes.c_uint]
    dptr = ctypes.c_void_p()
    rc = _hip.hipHostGetDevicePointer(ctypes.byref(dptr), t.data_ptr(), 0)
    if rc != 0 or not dptr.value:
        raise RuntimeError(f"pinned tensor is not device-accessible (hipHostGetDevicePointer -> {rc})")
    return int(dptr.value)


def pool_of(t: torch.Tensor) -> Pool:
    """View a tensor shaped [num_planes][num_blocks][...] as a kvc_pool.

    The tensor lives in device memory or in pinned host memory (which the GPU reads and
    writes over PCIe: the swap-to-CPU-memory path).
    """
    if not (t.is_cuda or t.is_pinned()) or not t.is_contiguous() or t.dim() < 3:
        raise ValueError("pool tensor must be a contiguous device or pinned-host tensor [planes][blocks][...]")
    block_bytes = t[0, 0].numel() * t.element_size()
    base = t.data_ptr() if t.is_cuda else _device_pointer_of_pinned(t)
    return Pool(base=base, num_blocks=t.shape[1], block_bytes=block_bytes,
                plane_stride_bytes=t.shape[1] * block_bytes, num_planes=t.shape[0], reserved=0)


def kv_block_copy(src_pool, dst_pool, block_mapping, stream=None) -> None:
    """dst[p][d] = src[p][s] for every (s, d) in block_mapping (device int64 [n][2]).

    Pools are Pool structs or tensors shaped [num_planes][num_blocks][...].
    """
    src = src_pool if isinstance(src_pool, Pool) else pool_of(src_pool)
    dst = dst_pool if isinstance(dst_pool, Pool) else pool_of(dst_pool)
    if block_mapping.dtype != torch.int64 or not block_mapping.is_cuda or not block_mapping.is_contiguous():
        raise TypeError("block_mapping must be a contiguous device int64 tensor [n][2]")
    n = block_mapping.numel() // 2
    _check(lib().kvc_kv_block_copy(ctypes.byref(src), ctypes.byref(dst), block_mapping.data_ptr(), n,
                                   _stream_handle(stream)), "kvc_kv_block_copy")


def validate_block_mapping(src_pool, dst_pool, block_mapping, stream=None) -> int:
    src = src_pool if isinstance(src_pool, Pool) else pool_of(src_pool)
    dst = dst_pool if isinstance(dst_pool, Pool) else pool_of(dst_pool)
    n = block_mapping.numel() // 2
    return int(lib().kvc_validate_block_mapping(ctypes.byref(src), ctypes.byref(dst),
                                                block_mapping.data_ptr(), n, _stream_handle(stream)))
