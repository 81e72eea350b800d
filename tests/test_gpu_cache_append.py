"""kv_cache_append on the GPU against the oracle: bit-exact over both whole caches, and a
chained decode step (append, then attend over the longer context)."""
import numpy as np
import pytest
import torch

import kvc_workloads as W
from gpu_util import BF16_TOL, dev_tensor, out_to_f64

pytestmark = pytest.mark.gpu


def cache_bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32).cpu().numpy()


@pytest.mark.parametrize("dtype,d,bs,hkv,nseq", [(W.BF16, 128, 16, 8, 64), (W.BF16, 128, 8, 2, 7), (W.F32, 64, 16, 8, 4),
                                                 (W.F32, 128, 32, 1, 3), (W.BF16, 64, 1, 4, 9), (W.BF16, 128, 16, 8, 1000)])
def test_append_matches_oracle_bit_exactly(oracle_mod, dtype, d, bs, hkv, nseq):
    import paper_2503_13773_amd as K
    print(f"[case] append {dtype} d={d} bs={bs} hkv={hkv} nseq={nseq}", flush=True)
    rng = np.random.default_rng(nseq * 7 + bs)
    ctx = rng.integers(1, 6 * bs + 2, nseq).astype(np.int32)
    w = W.build_workload("append", rng, dtype=dtype, context_lens=ctx, num_q_heads=hkv, num_kv_heads=hkv,
                         head_dim=d, block_size=bs, max_blocks_per_seq=8, num_pool_blocks=None, occupancy=0.8)
    pos = (ctx - 1).astype(np.int32)                       # overwrite the last token of every sequence
    pos[rng.random(nseq) < 0.2] = -1                       # some sequences sit this step out
    npdt = np.float32 if dtype == W.F32 else np.uint16
    if dtype == W.F32:
        k_new = rng.standard_normal((nseq, hkv, d)).astype(np.float32)
        v_new = rng.standard_normal((nseq, hkv, d)).astype(np.float32)
    else:
        k_new = W.f32_to_bf16_bits(rng.standard_normal((nseq, hkv, d)).astype(np.float32))
        v_new = W.f32_to_bf16_bits(rng.standard_normal((nseq, hkv, d)).astype(np.float32))
    wk, wv = w.k_cache.copy(), w.v_cache.copy()
    oracle_mod.kv_cache_append(k_new, v_new, wk, wv, w.block_tables, pos)
    dk, dv = dev_tensor(w.k_cache, dtype), dev_tensor(w.v_cache, dtype)
    K.kv_cache_append(dev_tensor(k_new, dtype), dev_tensor(v_new, dtype), dk, dv,
                      torch.from_numpy(w.block_tables).cuda(), torch.from_numpy(pos).cuda())
    torch.cuda.synchronize()
    want_k = wk.view(np.int16) if dtype == W.BF16 else wk.view(np.int32)
    want_v = wv.view(np.int16) if dtype == W.BF16 else wv.view(np.int32)
    assert np.array_equal(cache_bits(dk), want_k) and np.array_equal(cache_bits(dv), want_v)
    assert not np.array_equal(want_k, w.k_cache.view(want_k.dtype))   # something was written


def test_chained_decode_steps_append_then_attend(oracle_mod):
    """Three decode steps of an 8B-shape batch: each appends one token per sequence (crossing
    block boundaries for some) and attends; every step equals the oracle on the oracle's cache."""
    import paper_2503_13773_amd as K
    w = W.make_config("cfg3", num_seqs=10, ctx_scale=0.2)
    rng = np.random.default_rng(77)
    room = w.max_blocks_per_seq * 16
    free = list(w.extra["free_blocks"])
    hk, hv, tables, lens = w.k_cache.copy(), w.v_cache.copy(), w.block_tables.copy(), w.context_lens.copy()
    lens[0] = 16 * ((lens[0] + 15) // 16)                  # sequence 0 starts a fresh block at once
    dk, dv = dev_tensor(hk, W.BF16), dev_tensor(hv, W.BF16)
    dq = dev_tensor(w.q, W.BF16)
    for step in range(3):
        pos = lens.copy().astype(np.int32)
        for n in range(w.num_seqs):                        # host-side block manager: new block when needed
            if pos[n] % 16 == 0:
                tables[n, pos[n] // 16] = free.pop()
        k_new = W.f32_to_bf16_bits(rng.standard_normal((w.num_seqs, 8, 128)).astype(np.float32))
        v_new = W.f32_to_bf16_bits(rng.standard_normal((w.num_seqs, 8, 128)).astype(np.float32))
        oracle_mod.kv_cache_append(k_new, v_new, hk, hv, tables, pos)
        dt, dp = torch.from_numpy(tables).cuda(), torch.from_numpy(pos).cuda()
        K.kv_cache_append(dev_tensor(k_new, W.BF16), dev_tensor(v_new, W.BF16), dk, dv, dt, dp)
        lens = lens + 1
        out = K.paged_attention_decode(dq, dk, dv, dt, torch.from_numpy(lens.astype(np.int32)).cuda(), w.scale,
                                       max_context_len=int(lens.max()))
        torch.cuda.synchronize()
        ref = oracle_mod.paged_attention_decode(w.q, hk, hv, tables, lens.astype(np.int32), w.scale,
                                                dtype="bf16", num_threads=8)
        assert np.abs(out_to_f64(out) - ref).max() <= BF16_TOL, step
    assert np.array_equal(cache_bits(dk), hk.view(np.int16))


def test_positions_past_the_block_table_are_skipped():
    """A position at or beyond max_blocks_per_seq * block_size has no table entry: the sequence is
    skipped like one with a negative position, nothing outside the table is read, nothing written."""
    import paper_2503_13773_amd as K
    rng = np.random.default_rng(77)
    nseq, hkv, d, bs, lmax = 5, 2, 128, 16, 4
    w = W.build_workload("append-oob", rng, dtype=W.BF16, context_lens=np.full(nseq, 20, dtype=np.int32),
                         num_q_heads=hkv, num_kv_heads=hkv, head_dim=d, block_size=bs, max_blocks_per_seq=lmax,
                         num_pool_blocks=None, occupancy=0.8)
    k_new = W.f32_to_bf16_bits(rng.standard_normal((nseq, hkv, d)).astype(np.float32))
    v_new = W.f32_to_bf16_bits(rng.standard_normal((nseq, hkv, d)).astype(np.float32))
    pos = np.array([19, lmax * bs, lmax * bs + 5, 2 ** 30, 3], dtype=np.int32)
    host_pos = np.where(pos >= lmax * bs, -1, pos).astype(np.int32)          # what the oracle is asked to do
    wk, wv = w.k_cache.copy(), w.v_cache.copy()
    oracle_mod_pos = host_pos
    import oracle
    oracle.kv_cache_append(k_new, v_new, wk, wv, w.block_tables, oracle_mod_pos)
    dk, dv = dev_tensor(w.k_cache, W.BF16), dev_tensor(w.v_cache, W.BF16)
    K.kv_cache_append(dev_tensor(k_new, W.BF16), dev_tensor(v_new, W.BF16), dk, dv,
                      torch.from_numpy(w.block_tables).cuda(), torch.from_numpy(pos).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(cache_bits(dk), wk.view(np.int16)) and np.array_equal(cache_bits(dv), wv.view(np.int16))
