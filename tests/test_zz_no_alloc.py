"""The entry point that allocates nothing (kvc_paged_attention_decode_noalloc) against the
ordinary one, through the C ABI: two calls in a row on one GPU, the second on a smaller input,
so the second call runs on whatever the first left in the library's fixed workspace."""
import numpy as np
import pytest
import torch

import kvc_workloads as W
from gpu_util import BF16_TOL, out_bits, out_to_f64, to_device

pytestmark = pytest.mark.gpu


def _both(w, oracle_mod, label):
    import paper_2503_13773_amd as K
    d = to_device(w)
    desc = K.attn_desc(d["q"], d["k"], d["tables"], max_context_len=w.max_context_len)
    assert 0 < K.workspace_bytes(desc) <= K.NOALLOC_WORKSPACE_BYTES
    print(f"[case] noalloc {label}: {w.num_seqs} seqs, workspace need {K.workspace_bytes(desc)} B", flush=True)
    want = K.paged_attention_decode(d["q"], d["k"], d["v"], d["tables"], d["lens"], w.scale, desc=desc)
    torch.cuda.synchronize()
    out = torch.full_like(d["q"], 7.0)
    before = torch.cuda.memory_allocated()
    K.paged_attention_decode_noalloc(d["q"], d["k"], d["v"], d["tables"], d["lens"], w.scale, out, desc)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert np.array_equal(out_bits(out), out_bits(want)), label        # same kernels: same bits
    ref = oracle_mod.attention_of_workload(w, num_threads=8)
    assert np.abs(out_to_f64(out) - ref).max() <= BF16_TOL


def test_noalloc_matches_the_ordinary_call_twice_in_a_row(oracle_mod):
    _both(W.make_config("cfg3b"), oracle_mod, "first, cfg3b at full size")
    _both(W.make_config("cfg3", num_seqs=9, ctx_scale=0.3), oracle_mod, "second, smaller")


def test_noalloc_refuses_what_does_not_fit_and_bad_arguments():
    import paper_2503_13773_amd as K
    w = W.make_config("cfg3", num_seqs=4, ctx_scale=0.2)
    d = to_device(w)
    out = torch.empty_like(d["q"])
    big = K.AttnDesc(num_seqs=4096, num_q_heads=32, num_kv_heads=8, head_dim=128, block_size=16,
                     max_blocks_per_seq=256, num_pool_blocks=1 << 20, dtype=K.KVC_BF16,
                     max_context_len=4096, partition_tokens=256, kernel=K.KERNEL_MFMA, reserved=0)
    assert K.workspace_bytes(big) > K.NOALLOC_WORKSPACE_BYTES
    rc = K.lib().kvc_paged_attention_decode_noalloc(d["q"].data_ptr(), d["k"].data_ptr(), d["v"].data_ptr(),
                                                    d["tables"].data_ptr(), d["lens"].data_ptr(), w.scale,
                                                    out.data_ptr(), __import__("ctypes").byref(big), None)
    assert rc == -5      # KVC_ERR_WORKSPACE, before anything is launched
    desc = K.attn_desc(d["q"], d["k"], d["tables"], max_context_len=w.max_context_len)
    rc = K.lib().kvc_paged_attention_decode_noalloc(None, d["k"].data_ptr(), d["v"].data_ptr(),
                                                    d["tables"].data_ptr(), d["lens"].data_ptr(), w.scale,
                                                    out.data_ptr(), __import__("ctypes").byref(desc), None)
    assert rc == -1      # KVC_ERR_NULL
