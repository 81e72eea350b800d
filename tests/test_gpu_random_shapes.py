"""Seeded sweep over legal shapes: the HIP decode and prefill attention against the fp64 oracle,
every element compared, on shapes the hand-picked cases do not name (odd batch sizes, every
group size up to 16, block sizes 1..64, both dtypes, head_dim 64 and 128, empty and one-token
sequences mixed in)."""
import numpy as np
import pytest
import torch

import kvc_workloads as W
from gpu_util import BF16_TOL, dev_tensor, out_to_f64, run_gpu, tol_of

pytestmark = pytest.mark.gpu


def random_lens(rng, nseq, cap):
    lens = np.exp(rng.normal(4.5, 1.2, nseq)).astype(np.int64).clip(1, cap)
    lens[rng.random(nseq) < 0.08] = 0
    lens[rng.random(nseq) < 0.08] = 1
    return lens.astype(np.int32)


@pytest.mark.parametrize("seed", range(24))
def test_decode_random_shape(oracle_mod, seed):
    rng = np.random.default_rng(9000 + seed)
    dtype = W.BF16 if rng.random() < 0.7 else W.F32
    d = 128 if (dtype == W.BF16 and rng.random() < 0.8) else int(rng.choice([64, 128]))
    hkv = int(rng.choice([1, 2, 3, 8]))
    group = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 16]))
    bs = int(rng.choice([1, 2, 4, 8, 16, 32, 64]))
    nseq = int(rng.integers(1, 41))
    lens = random_lens(rng, nseq, 1500)
    nblk = W.blocks_needed(lens, bs)
    w = W.build_workload(f"rand{seed}", rng, dtype=dtype, context_lens=lens, num_q_heads=hkv * group,
                         num_kv_heads=hkv, head_dim=d, block_size=bs,
                         max_blocks_per_seq=int(max(1, nblk.max())) + int(rng.integers(0, 4)),
                         num_pool_blocks=int(nblk.sum()) + int(rng.integers(1, 30)))
    pt = int(rng.choice([0, 0, 64, 256]))
    print(f"[case] decode seed={seed} dtype={dtype} D={d} Hkv={hkv} G={group} Bs={bs} nseq={nseq} "
          f"max_len={int(lens.max())} partition_tokens={pt}", flush=True)
    got = out_to_f64(run_gpu(w, partition_tokens=pt))
    ref = oracle_mod.attention_of_workload(w, num_threads=8)
    assert np.isfinite(got).all()
    assert np.abs(got - ref).max() <= tol_of(w)


@pytest.mark.parametrize("seed", range(12))
def test_prefill_random_shape(oracle_mod, seed):
    import paper_2503_13773_amd as K
    rng = np.random.default_rng(9500 + seed)
    hkv = int(rng.choice([1, 2, 4]))
    group = int(rng.choice([1, 2, 3, 4, 6, 8, 16]))
    hq = hkv * group
    bs = int(rng.choice([2, 8, 16, 32, 64]))
    nseq = int(rng.integers(1, 9))
    lens = np.exp(rng.normal(5.0, 1.0, nseq)).astype(np.int64).clip(1, 900).astype(np.int32)
    # a mix of full recomputes, chunk tails and skipped sequences
    kind = rng.integers(0, 3, nseq)
    qlens = np.where(kind == 0, lens, np.where(kind == 1, rng.integers(1, lens + 1), 0)).astype(np.int32)
    nblk = W.blocks_needed(lens, bs)
    w = W.build_workload(f"randp{seed}", rng, dtype=W.BF16, context_lens=lens, num_q_heads=hq, num_kv_heads=hkv,
                         head_dim=128, block_size=bs, max_blocks_per_seq=int(nblk.max()) + 1,
                         num_pool_blocks=int(nblk.sum()) + 3)
    q_start = np.concatenate([[0], np.cumsum(qlens)]).astype(np.int32)
    total = int(q_start[-1])
    print(f"[case] prefill seed={seed} Hkv={hkv} G={group} Bs={bs} lens={lens.tolist()} q={qlens.tolist()}", flush=True)
    if total == 0:
        qlens[0] = lens[0]
        q_start = np.concatenate([[0], np.cumsum(qlens)]).astype(np.int32)
        total = int(q_start[-1])
    q = W.f32_to_bf16_bits(rng.standard_normal((total, hq, 128)).astype(np.float32))
    out = K.paged_attention_prefill(dev_tensor(q, W.BF16), dev_tensor(w.k_cache, W.BF16), dev_tensor(w.v_cache, W.BF16),
                                    torch.from_numpy(w.block_tables).cuda(), torch.from_numpy(w.context_lens).cuda(),
                                    torch.from_numpy(q_start).cuda(), w.scale, int(qlens.max()))
    torch.cuda.synchronize()
    got = out_to_f64(out)
    ref = oracle_mod.paged_attention_prefill(q, w.k_cache, w.v_cache, w.block_tables, w.context_lens, q_start,
                                             w.scale, dtype="bf16", num_threads=8)
    assert np.isfinite(got).all()
    assert np.abs(got - ref).max() <= BF16_TOL
