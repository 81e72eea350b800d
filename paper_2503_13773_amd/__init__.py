"""Paged-KV decode hot path for MI355X: thin Python binding over libkvc_hip.so.

The two operations (see include/kvc.h for the contract):
    paged_attention_decode  batched decode attention over a block-allocated KV cache
    kv_block_copy           bit-exact block gather/scatter between KV pools
    kv_cache_append         write one new token per sequence into the block-allocated cache
    paged_attention_prefill causal attention of many query positions (recompute / chunked prefill)
Every step runs in the HIP kernels of the library; this package only marshals
arguments.  PyTorch supplies device memory and streams.
"""
from .binding import (  # noqa: F401
    KVC_F32, KVC_BF16, KERNEL_AUTO, KERNEL_VALU, KERNEL_MFMA, KERNEL_MFMA_LDS, KERNEL_MFMA_BALANCED,
    KvcError, AttnDesc, AttnPlan, Pool, lib, library_path, attn_desc, attn_plan,
    workspace_bytes, workspace_init, new_workspace, paged_attention_decode, paged_attention_decode_partial,
    paged_attention_decode_noalloc, NOALLOC_WORKSPACE_BYTES, schedule_bytes, attn_schedule_build,
    paged_attention_decode_scheduled,
    paged_attention_decode_merge, paged_attention_prefill, validate_attention_inputs, kv_block_copy, kv_cache_append,
    validate_block_mapping, pool_of, status_string, version,
)
