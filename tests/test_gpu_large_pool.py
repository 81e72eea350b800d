"""Pools larger than 4 GiB: every kernel must do its address arithmetic in 64 bits.  The big device
pools are left uninitialised except for the blocks the batch references, which are copied from a
small host pool; the oracle runs on the small pool with the block ids mapped back."""
import numpy as np
import pytest
import torch

import kvc_workloads as W
from gpu_util import BF16_TOL, dev_tensor, out_bits, out_to_f64

pytestmark = pytest.mark.gpu

NB_BIG = 150_000            # x 8 heads x 16 tokens x 128 dims x 2 bytes = 4.9 GB per pool


def big_pools(w, rng):
    """Device pools of NB_BIG blocks holding w's blocks at ids spread over the whole range."""
    nb = w.k_cache.shape[0]
    big_ids = np.sort(rng.choice(NB_BIG, nb, replace=False)).astype(np.int64)
    big_ids[-1] = NB_BIG - 1                                     # the very last block is used
    big_ids[0] = 0
    shape = (NB_BIG,) + w.k_cache.shape[1:]
    kb = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
    vb = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
    idx = torch.from_numpy(big_ids).cuda()
    kb[idx] = dev_tensor(w.k_cache, W.BF16)
    vb[idx] = dev_tensor(w.v_cache, W.BF16)
    tables = np.where(w.block_tables >= 0, big_ids[np.maximum(w.block_tables, 0)], -1).astype(np.int32)
    return kb, vb, tables, big_ids


def test_decode_prefill_append_and_copy_beyond_4_gib(oracle_mod):
    import paper_2503_13773_amd as K
    if torch.cuda.get_device_properties(0).total_memory < 24e9:
        pytest.skip("needs 24 GB of device memory")
    rng = np.random.default_rng(4100)
    w = W.make_config("cfg3", num_seqs=12, ctx_scale=0.5)
    kb, vb, tables, big_ids = big_pools(w, rng)
    assert kb.numel() * 2 > (1 << 32) and int(tables.max()) == NB_BIG - 1
    t_dev, lens = torch.from_numpy(tables).cuda(), torch.from_numpy(w.context_lens).cuda()

    print("[case] decode, pool of 4.9 GB", flush=True)
    for kernel in (0, 2, 1):                                     # balanced, fixed partitions, vector ALU
        out = K.paged_attention_decode(dev_tensor(w.q, W.BF16), kb, vb, t_dev, lens, w.scale,
                                       max_context_len=w.max_context_len, kernel=kernel)
        torch.cuda.synchronize()
        ref = oracle_mod.attention_of_workload(w, num_threads=8)
        assert np.abs(out_to_f64(out) - ref).max() <= BF16_TOL, kernel

    print("[case] prefill, pool of 4.9 GB", flush=True)
    qlens = np.minimum(w.context_lens, 40).astype(np.int32)
    q_start = np.concatenate([[0], np.cumsum(qlens)]).astype(np.int32)
    q = W.f32_to_bf16_bits(rng.standard_normal((int(q_start[-1]), w.num_q_heads, 128)).astype(np.float32))
    out = K.paged_attention_prefill(dev_tensor(q, W.BF16), kb, vb, t_dev, lens, torch.from_numpy(q_start).cuda(),
                                    w.scale, int(qlens.max()))
    torch.cuda.synchronize()
    ref = oracle_mod.paged_attention_prefill(q, w.k_cache, w.v_cache, w.block_tables, w.context_lens, q_start,
                                             w.scale, dtype="bf16", num_threads=8)
    assert np.abs(out_to_f64(out) - ref).max() <= BF16_TOL

    print("[case] append, pool of 4.9 GB", flush=True)
    pos = (w.context_lens - 1).astype(np.int32)
    kn = W.f32_to_bf16_bits(rng.standard_normal((w.num_seqs, w.num_kv_heads, 128)).astype(np.float32))
    vn = W.f32_to_bf16_bits(rng.standard_normal((w.num_seqs, w.num_kv_heads, 128)).astype(np.float32))
    K.kv_cache_append(dev_tensor(kn, W.BF16), dev_tensor(vn, W.BF16), kb, vb, t_dev, torch.from_numpy(pos).cuda())
    torch.cuda.synchronize()
    hk, hv = w.k_cache.copy(), w.v_cache.copy()
    oracle_mod.kv_cache_append(kn, vn, hk, hv, w.block_tables, pos)
    idx = torch.from_numpy(big_ids).cuda()
    assert np.array_equal(out_bits(kb[idx]).view(np.uint16), hk) and np.array_equal(out_bits(vb[idx]).view(np.uint16), hv)

    print("[case] block copy out of and into the far end of a 9.8 GB pool", flush=True)
    pool = torch.empty((2, NB_BIG) + tuple(kb.shape[1:]), dtype=torch.bfloat16, device="cuda")
    pool[0, idx] = kb[idx]
    pool[1, idx] = vb[idx]
    n = 64
    src = big_ids[-n:]
    dst_small = torch.zeros((2, n) + tuple(kb.shape[1:]), dtype=torch.bfloat16, device="cuda")
    K.kv_block_copy(pool, dst_small, torch.from_numpy(np.stack([src, np.arange(n)], axis=1).astype(np.int64)).cuda())
    torch.cuda.synchronize()
    assert torch.equal(dst_small[0], kb[idx[-n:]]) and torch.equal(dst_small[1], vb[idx[-n:]])
    far = np.arange(NB_BIG - 2 * n, NB_BIG - n).astype(np.int64)           # free blocks near the end
    far = far[~np.isin(far, big_ids)][: n // 2]
    K.kv_block_copy(dst_small, pool, torch.from_numpy(np.stack([np.arange(len(far)), far], axis=1).astype(np.int64)).cuda())
    torch.cuda.synchronize()
    assert torch.equal(pool[0, torch.from_numpy(far).cuda()], dst_small[0, :len(far)])
    assert torch.equal(pool[1, torch.from_numpy(far).cuda()], dst_small[1, :len(far)])
