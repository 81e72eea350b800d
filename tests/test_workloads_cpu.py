"""The seeded input generators: shapes, length statistics, block-table consistency."""
import numpy as np
import pytest

import kvc_workloads as W


def used_blocks(w):
    nblk = W.blocks_needed(w.context_lens, w.block_size)
    return [w.block_tables[n, :nblk[n]] for n in range(w.num_seqs)], nblk


def test_bf16_round_trip_and_rounding():
    x = np.array([1.0, -2.5, 3.140625, 1e-3, 65504.0, 0.0], dtype=np.float32)
    b = W.f32_to_bf16_bits(x)
    y = W.bf16_bits_to_f32(b)
    assert np.all(np.abs(y - x) <= np.abs(x) * 2.0 ** -8)
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert W.f32_to_bf16_bits(np.array([1.0 + 2.0 ** -8], dtype=np.float32))[0] == 0x3F80
    assert W.f32_to_bf16_bits(np.array([1.0 + 3 * 2.0 ** -8], dtype=np.float32))[0] == 0x3F82
    assert np.isnan(W.bf16_bits_to_f32(W.f32_to_bf16_bits(np.array([np.nan], dtype=np.float32))))[0]


def test_cfg1_matches_its_recipe():
    w = W.make_config("cfg1")
    assert (w.dtype, w.num_seqs, w.num_q_heads, w.num_kv_heads, w.head_dim, w.block_size) == ("f32", 4, 8, 8, 64, 16)
    assert w.num_pool_blocks == 128 and w.scale == 0.125
    assert w.context_lens.min() >= 16 and w.context_lens.max() <= 256
    assert w.k_cache.shape == (128, 8, 16, 64) and w.k_cache.dtype == np.float32
    w2 = W.make_config("cfg1")
    assert np.array_equal(w.k_cache, w2.k_cache) and np.array_equal(w.block_tables, w2.block_tables)


@pytest.mark.parametrize("name,nseq,hq,hkv,cap", [("cfg2", 64, 32, 32, 4096), ("cfg3", 128, 32, 8, 4096),
                                                  ("cfg3b", 64, 32, 8, 4096)])
def test_lognormal_configs(name, nseq, hq, hkv, cap):
    w = W.make_config(name, ctx_scale=1.0)
    assert (w.num_seqs, w.num_q_heads, w.num_kv_heads, w.head_dim, w.block_size) == (nseq, hq, hkv, 128, 16)
    assert w.context_lens.min() >= 9 and w.context_lens.max() <= cap
    assert 500 < w.context_lens.mean() < 1300          # the mix has mean ~860-880
    blocks, nblk = used_blocks(w)
    allb = np.concatenate(blocks)
    assert allb.min() >= 0 and allb.max() < w.num_pool_blocks
    assert len(np.unique(allb)) == len(allb)            # no block owned twice
    for n in range(w.num_seqs):
        assert (w.block_tables[n, nblk[n]:] == -1).all()
    if name != "cfg2":
        assert abs(len(allb) / w.num_pool_blocks - 0.9) < 0.01   # pool 90 % occupied
    else:
        assert len(allb) == w.num_pool_blocks
    # scattered, not allocated in order
    assert np.abs(np.diff(blocks[int(np.argmax(nblk))])).mean() > 10


def test_length_mix_statistics():
    rng = np.random.default_rng(0)
    ctx = W.lognormal_context_lens(rng, 200000, 4096, 4096)
    assert 840 < ctx.mean() < 920 and 600 < np.median(ctx) < 800
    assert ctx.max() == 4096 and ctx.min() >= 9
    ctx2 = W.lognormal_context_lens(rng, 200000, 2048)
    assert 820 < ctx2.mean() < 900 and ctx2.max() <= 4096


def test_cfg4_small_and_cfg5_sharing_and_swap_plan():
    w4 = W.make_config("cfg4", num_seqs=2, ctx_scale=0.01)
    assert (w4.num_q_heads, w4.num_kv_heads, w4.max_blocks_per_seq) == (64, 8, 2048)
    w = W.make_config("cfg5", num_seqs=40, ctx_scale=0.3)
    groups = w.extra["share_groups"]
    shared_seqs = sum(len(g[0]) for g in groups)
    assert shared_seqs == 10                              # 25 % of 40
    for seqs, k in groups:
        assert 2 <= len(seqs) <= 4 and k >= 1
        for s in seqs[1:]:
            assert np.array_equal(w.block_tables[s, :k], w.block_tables[seqs[0], :k])
            assert w.block_tables[s, k] != w.block_tables[seqs[0], k]
            assert k * w.block_size < min(w.context_lens[s], w.context_lens[seqs[0]])  # full blocks only
    sp = w.extra["swap"]
    assert len(sp["victims"]) == 8                        # ceil(20 % of 40)
    ingroup = {s for seqs, _ in groups for s in seqs}
    assert not ingroup & set(sp["victims"])
    out_m, in_m = sp["out_mapping"], sp["in_mapping"]
    assert np.array_equal(out_m[:, 1], in_m[:, 0])
    assert len(np.unique(out_m[:, 1])) == len(out_m) and out_m[:, 1].max() < sp["pool2_blocks"]
    blocks, nblk = used_blocks(w)
    used = set(np.concatenate(blocks).tolist())
    assert not used & set(in_m[:, 1].tolist())            # swap-in goes to slots nobody owns
    assert len(np.unique(in_m[:, 1])) == len(in_m)
    for v in sp["victims"]:
        assert not set(sp["tables_after"][v, :nblk[v]].tolist()) & set(w.block_tables[v, :nblk[v]].tolist())


def test_copy_mapping_is_a_partial_permutation():
    rng = np.random.default_rng(1)
    m = W.make_copy_mapping(rng, 8, 128, 128)
    assert m.shape == (8, 2) and m.dtype == np.int64
    assert len(np.unique(m[:, 0])) == 8 and len(np.unique(m[:, 1])) == 8 and m.max() < 128 and m.min() >= 0
