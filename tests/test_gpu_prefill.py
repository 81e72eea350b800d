"""Causal multi-query attention (recompute / chunked prefill) on the GPU against the fp64 oracle:
max-abs error <= 2e-2 for bf16, every element compared."""
import numpy as np
import pytest
import torch

import kvc_workloads as W
from gpu_util import BF16_TOL, dev_tensor, out_bits, out_to_f64, tol_of

pytestmark = pytest.mark.gpu


def make(seed, lens, qlens, hq, hkv, bs=16, dtype=W.BF16, d=128):
    rng = np.random.default_rng(seed)
    lens = np.asarray(lens, dtype=np.int32)
    nblk = W.blocks_needed(lens, bs)
    w = W.build_workload("prefill", rng, dtype=dtype, context_lens=lens, num_q_heads=hq, num_kv_heads=hkv,
                         head_dim=d, block_size=bs, max_blocks_per_seq=int(max(1, nblk.max())) + 1,
                         num_pool_blocks=int(nblk.sum()) + 5)
    q_start = np.concatenate([[0], np.cumsum(qlens)]).astype(np.int32)
    q = rng.standard_normal((int(q_start[-1]), hq, d)).astype(np.float32)
    if dtype == W.BF16:
        q = W.f32_to_bf16_bits(q)
    return w, q, q_start


def run(w, q, q_start, max_q, kernel=0):
    import paper_2503_13773_amd as K
    out = K.paged_attention_prefill(dev_tensor(q, w.dtype), dev_tensor(w.k_cache, w.dtype), dev_tensor(w.v_cache, w.dtype),
                                    torch.from_numpy(w.block_tables).cuda(), torch.from_numpy(w.context_lens).cuda(),
                                    torch.from_numpy(q_start).cuda(), w.scale, max_q, kernel=kernel)
    torch.cuda.synchronize()
    return out


def check(oracle_mod, w, q, q_start, label, kernel=0):
    print(f"[case] prefill {label} kernel={kernel} lens={w.context_lens.tolist()[:6]} q={np.diff(q_start).tolist()[:6]}", flush=True)
    max_q = int(np.diff(q_start).max())
    got = out_to_f64(run(w, q, q_start, max_q, kernel))
    ref = oracle_mod.paged_attention_prefill(q, w.k_cache, w.v_cache, w.block_tables, w.context_lens, q_start,
                                             w.scale, dtype=w.dtype, num_threads=8)
    rows = np.concatenate([np.arange(q_start[n], q_start[n + 1]) for n in range(len(w.context_lens))]) \
        if q_start[-1] else np.zeros(0, dtype=int)
    assert np.isfinite(got[rows]).all()
    err = np.abs(got[rows] - ref[rows]).max() if len(rows) else 0.0
    assert err <= tol_of(w), (label, err)
    return err


@pytest.mark.parametrize("hq,hkv", [(4, 1), (8, 2), (2, 2), (2, 1), (8, 1), (3, 1), (32, 8)])
def test_full_recompute_matches_oracle(oracle_mod, hq, hkv):
    lens = [1, 5, 16, 17, 63, 64, 65, 130, 300]
    w, q, qs = make(300 + hq, lens, lens, hq, hkv)
    check(oracle_mod, w, q, qs, f"recompute {hq}/{hkv}")


@pytest.mark.parametrize("hq,hkv,bs", [(4, 1, 16), (8, 2, 32), (32, 8, 16), (3, 1, 16), (4, 4, 16), (5, 1, 32)])
def test_both_tile_kernels(oracle_mod, hq, hkv, bs):
    """kernel = 2 (KVC_KERNEL_MFMA) asks for the 16x16-tile kernel where the default takes 32x32 tiles (two
    heads per wavefront for even group sizes, one head and 32 query rows for odd ones): both against the
    oracle on the same input."""
    lens = [1, 5, 16, 17, 63, 64, 65, 130, 300, 1000]
    w, q, qs = make(340 + hq + bs, lens, lens, hq, hkv, bs=bs)
    check(oracle_mod, w, q, qs, f"16x16 tiles {hq}/{hkv} bs={bs}", kernel=2)
    check(oracle_mod, w, q, qs, f"32x32 tiles {hq}/{hkv} bs={bs}", kernel=0)


@pytest.mark.parametrize("hq,hkv", [(32, 8), (4, 2)])
def test_ragged_query_counts(oracle_mod, hq, hkv):
    """Chunked: query rows are the last Qn positions; counts around the 16-row, 64-row and 128-row
    boundaries of the kernels' wavefronts and workgroups."""
    lens = [130, 40, 64, 65, 127, 129, 200, 256, 300, 513, 97, 1000]
    qlens = [130, 1, 64, 65, 127, 129, 200, 256, 300, 17, 96, 129]
    w, q, qs = make(360 + hq, lens, qlens, hq, hkv)
    check(oracle_mod, w, q, qs, f"ragged {hq}/{hkv}")


@pytest.mark.parametrize("bs", [64, 128, 256])
def test_blocks_of_several_tiles(oracle_mod, bs):
    """Blocks of 4, 8 and 16 tiles of 16 tokens: a wavefront's tile of a step is a sub-tile of a block."""
    lens = [1, 17, 63, 64, 65, 250, 256, 257, 700]
    w, q, qs = make(380 + bs, lens, lens, 8, 2, bs=bs)
    check(oracle_mod, w, q, qs, f"bs={bs}")


def test_long_ragged_recompute_in_128_row_workgroups(oracle_mod):
    """From 3072 query rows per sequence on (and 512 workgroups or more) a workgroup is two groups of
    four wavefronts and 128 query rows: 3100 and 3073 rows leave the last workgroup with 28 rows (two
    wavefronts of the first group) and with 1 row; sampled rows against the oracle's decode over the
    truncated context."""
    lens, qlens = [3100, 3300], [3100, 3073]
    w, q, qs = make(370, lens, qlens, 32, 8)
    got = out_to_f64(run(w, q, qs, 3100))
    rng = np.random.default_rng(2)
    for n in range(2):
        first = lens[n] - qlens[n]
        for i in [0, 15, 16, 63, 64, 127, 128, qlens[n] - 29, qlens[n] - 1] + rng.integers(0, qlens[n], 6).tolist():
            pos = first + i
            tbl = w.block_tables[n:n + 1]
            ref = oracle_mod.paged_attention_decode(q[qs[n] + i:qs[n] + i + 1], w.k_cache, w.v_cache, tbl,
                                                    np.array([pos + 1], dtype=np.int32), w.scale, dtype="bf16")
            assert np.abs(got[qs[n] + i] - ref[0]).max() <= BF16_TOL, (n, i)


def test_negative_scale_takes_the_small_tile_kernel(oracle_mod):
    """The 32x32-tile kernel takes its max over raw scores and needs a positive scale; any other
    scale is served by the 16x16-tile kernel."""
    import dataclasses
    lens = [40, 130]
    w, q, qs = make(350, lens, lens, 4, 1)
    w = dataclasses.replace(w, scale=-w.scale)
    check(oracle_mod, w, q, qs, "negative scale")


def test_chunked_prefill_unaligned_positions(oracle_mod):
    lens = [100, 77, 300, 16, 200, 45]
    qlens = [30, 77, 1, 16, 0, 44]          # chunk starts at positions 70, 0, 299, 0, -, 1
    w, q, qs = make(310, lens, qlens, 8, 2)
    check(oracle_mod, w, q, qs, "chunked")
    w, q, qs = make(311, [900, 513], [129, 500], 4, 1, bs=32)
    check(oracle_mod, w, q, qs, "chunked bs=32")


def test_single_query_row_equals_decode_attention():
    import paper_2503_13773_amd as K
    w = W.make_config("cfg3", num_seqs=6, ctx_scale=0.3)
    qs = np.arange(7, dtype=np.int32)
    pre = out_bits(run(w, w.q.reshape(6, 32, 128), qs, 1))
    dec = K.paged_attention_decode(dev_tensor(w.q, W.BF16), dev_tensor(w.k_cache, W.BF16), dev_tensor(w.v_cache, W.BF16),
                                   torch.from_numpy(w.block_tables).cuda(), torch.from_numpy(w.context_lens).cuda(),
                                   w.scale, max_context_len=w.max_context_len)
    torch.cuda.synchronize()
    # same per-tile arithmetic; decode may split the context, so compare within the bf16 tolerance
    assert np.abs(out_to_f64(dec) - dev_f64(pre)).max() <= BF16_TOL


def dev_f64(bits):
    return W.bf16_bits_to_f32(bits.view(np.uint16)).astype(np.float64)


def test_first_position_returns_v_exactly_and_poison_is_ignored(oracle_mod):
    w, q, qs = make(320, [37, 50], [37, 50], 4, 2)
    clean = out_bits(run(w, q, qs, 50))
    for n in range(2):
        blk = w.block_tables[n, 0]
        for h in range(4):
            assert np.array_equal(clean[qs[n], h], w.v_cache[blk, h // 2, 0].view(np.int16))
    nblk = W.blocks_needed(w.context_lens, 16)
    for n, L in enumerate(w.context_lens):
        b = w.block_tables[n, nblk[n] - 1]
        w.k_cache[b, :, L % 16:, :] = np.uint16(0x7FC0)
        w.v_cache[b, :, L % 16:, :] = np.uint16(0x7FC0)
        w.block_tables[n, nblk[n]:] = -1
    dirty = out_bits(run(w, q, qs, 50))
    assert np.array_equal(clean, dirty)
    check(oracle_mod, w, q, qs, "poisoned")


def test_long_recompute_sampled(oracle_mod):
    """A 4096-token recompute of an 8B-shape request; the oracle checks a sample of rows by
    treating each as a decode over the truncated context."""
    w, q, qs = make(330, [4096], [4096], 32, 8)
    got = out_to_f64(run(w, q, qs, 4096))
    rng = np.random.default_rng(1)
    for pos in [0, 15, 16, 1000, 2047, 4095] + rng.integers(0, 4096, 4).tolist():
        ref = oracle_mod.paged_attention_decode(q[pos:pos + 1], w.k_cache, w.v_cache, w.block_tables,
                                                np.array([pos + 1], dtype=np.int32), w.scale, dtype="bf16")
        assert np.abs(got[pos] - ref[0]).max() <= BF16_TOL, pos


@pytest.mark.parametrize("bs", [1, 2, 4, 8])
def test_block_sizes_below_a_tile(oracle_mod, bs):
    """A 16-token tile spans 2 to 16 blocks; table entries past the last needed block are -1."""
    lens = [1, 15, 16, 33, 100, 257]
    qlens = [1, 15, 7, 33, 100, 130]
    w, q, qs = make(340 + bs, lens, qlens, 4, 2, bs=bs)
    nblk = W.blocks_needed(w.context_lens, bs)
    for n in range(len(lens)):
        w.block_tables[n, nblk[n]:] = -1
    check(oracle_mod, w, q, qs, f"block_size {bs}")


@pytest.mark.parametrize("dtype,d,hq,hkv,bs", [(W.F32, 64, 8, 2, 16), (W.F32, 128, 4, 4, 8), (W.BF16, 64, 8, 2, 16),
                                                (W.BF16, 128, 32, 1, 16), (W.F32, 64, 6, 2, 1)])
def test_shapes_off_the_matrix_core_path(oracle_mod, dtype, d, hq, hkv, bs):
    """fp32, head_dim 64 and groups above 16 take the vector-ALU kernel (fp32: max-abs error <= 1e-5)."""
    lens = [1, 17, 64, 150, 333]
    qlens = [1, 17, 10, 0, 333]
    w, q, qs = make(370 + d + hq, lens, qlens, hq, hkv, bs=bs, dtype=dtype, d=d)
    check(oracle_mod, w, q, qs, f"valu {dtype} D={d} {hq}/{hkv} bs={bs}")


def test_prefill_argument_errors():
    import paper_2503_13773_amd as K
    w, q, qs = make(340, [20], [20], 4, 2)
    with pytest.raises(K.KvcError):                      # head_dim 32 is not a shape of this library
        K.paged_attention_prefill(dev_tensor(q, W.BF16)[:, :, :32].contiguous(),
                                  dev_tensor(w.k_cache, W.BF16)[..., :32].contiguous(),
                                  dev_tensor(w.v_cache, W.BF16)[..., :32].contiguous(),
                                  torch.from_numpy(w.block_tables).cuda(), torch.from_numpy(w.context_lens).cuda(),
                                  torch.from_numpy(qs).cuda(), w.scale, 20)
    bad_qs = torch.from_numpy(qs).cuda()[:1]              # q_start must have num_seqs + 1 entries
    with pytest.raises(TypeError):
        K.paged_attention_prefill(dev_tensor(q, W.BF16), dev_tensor(w.k_cache, W.BF16), dev_tensor(w.v_cache, W.BF16),
                                  torch.from_numpy(w.block_tables).cuda(), torch.from_numpy(w.context_lens).cuda(),
                                  bad_qs, w.scale, 20)


def test_context_beyond_32k_tokens_chunk(oracle_mod):
    """The last 150 positions of a 40000-token context (block ids come through the scalar cache,
    no per-workgroup table staging, so the context length is not bounded by LDS)."""
    w, q, qs = make(350, [40000, 33], [150, 33], 4, 2)
    check(oracle_mod, w, q, qs, "40000-token context")


def test_scores_that_keep_growing_along_the_context(oracle_mod):
    """Scores that rise steadily with the token index keep the running max moving by a few units
    (base 2) per 32-token step, and large queries give a wide dynamic range: both the rare
    full rebase of the softmax reference point and the steps in between are exercised."""
    rng = np.random.default_rng(360)
    lens = [700, 257]
    w, q, qs = make(360, lens, lens, 4, 2)
    kf = W.bf16_bits_to_f32(w.k_cache).copy()
    u = rng.standard_normal(128).astype(np.float32)
    u /= np.linalg.norm(u)
    nblk = W.blocks_needed(w.context_lens, 16)
    for n, L in enumerate(lens):
        for b in range(nblk[n]):
            t = (16 * b + np.arange(16)).astype(np.float32)
            kf[w.block_tables[n, b]] += (0.12 * t)[None, :, None] * u[None, None, :] * np.sqrt(128.0)
    w.k_cache[...] = W.f32_to_bf16_bits(kf)
    qf = W.bf16_bits_to_f32(q) * 0.3 + u[None, None, :] * 1.0
    q = W.f32_to_bf16_bits(qf.astype(np.float32))
    check(oracle_mod, w, q, qs, "rising scores")
    q = W.f32_to_bf16_bits((W.bf16_bits_to_f32(q) * 6.0).astype(np.float32))
    check(oracle_mod, w, q, qs, "rising scores, 6x queries")
