"""kv_block_copy on the GPU against the memcpy oracle: bit-exact over the whole destination
pool (untouched blocks included), plus the swap-out / poison / swap-in round trip."""
import numpy as np
import pytest
import torch

import kvc_workloads as W
from gpu_util import dev_tensor, out_bits, run_gpu, to_device

pytestmark = pytest.mark.gpu


def gpu_copy(src_np, dst_np, mapping_np):
    import paper_2503_13773_amd as K
    src = torch.from_numpy(src_np).cuda()
    dst = torch.from_numpy(dst_np).cuda()
    mp = torch.from_numpy(np.ascontiguousarray(mapping_np, dtype=np.int64).reshape(-1, 2)).cuda()
    K.kv_block_copy(src, dst, mp)
    torch.cuda.synchronize()
    return dst.cpu().numpy()


@pytest.mark.parametrize("planes,sb,db,block_bytes,pairs", [
    (1, 128, 128, 32768, 8),          # cfg1-copy: 8 random blocks of 32 KiB
    (2, 64, 40, 32768, 17),
    (3, 50, 70, 16, 20),              # smallest legal block
    (2, 33, 33, 4112, 33),            # four 1 KiB slabs and one word
    (4, 20, 20, 16384 + 48, 9),       # sixteen slabs and three words
    (2, 12, 12, 1040, 7),             # just over one slab
    (1, 12, 12, 1008, 5),             # just under one slab
    (64, 24, 24, 32768, 5),           # many planes (K,V x 32 layers)
    (1, 16, 16, 131072, 16),          # 7B-MHA block
])
def test_block_copy_matches_oracle(oracle_mod, planes, sb, db, block_bytes, pairs):
    print(f"[case] copy planes={planes} sb={sb} db={db} bytes={block_bytes} pairs={pairs}", flush=True)
    rng = np.random.default_rng(planes * 1000 + pairs)
    src = rng.integers(0, 256, (planes, sb, block_bytes), dtype=np.uint8)
    dst = rng.integers(0, 256, (planes, db, block_bytes), dtype=np.uint8)
    mapping = W.make_copy_mapping(rng, pairs, sb, db)
    want = dst.copy()
    oracle_mod.kv_block_copy(src, want, mapping)
    got = gpu_copy(src, dst, mapping)
    assert np.array_equal(got, want)


def test_block_copy_fan_out_and_empty(oracle_mod):
    rng = np.random.default_rng(3)
    src = rng.integers(0, 256, (2, 10, 1024), dtype=np.uint8)
    dst = rng.integers(0, 256, (2, 12, 1024), dtype=np.uint8)
    mapping = np.array([[4, 0], [4, 7], [4, 11], [1, 3]], dtype=np.int64)
    want = dst.copy()
    oracle_mod.kv_block_copy(src, want, mapping)
    assert np.array_equal(gpu_copy(src, dst, mapping), want)
    assert np.array_equal(gpu_copy(src, dst, np.zeros((0, 2), dtype=np.int64)), dst)


def test_block_copy_within_one_pool_disjoint_sets(oracle_mod):
    import paper_2503_13773_amd as K
    rng = np.random.default_rng(4)
    pool = rng.integers(0, 256, (2, 32, 2048), dtype=np.uint8)
    ids = rng.permutation(32)
    mapping = np.stack([ids[:10], ids[10:20]], axis=1).astype(np.int64)
    want = pool.copy()
    snapshot = pool.copy()
    oracle_mod.kv_block_copy(snapshot, want, mapping)
    t = torch.from_numpy(pool).cuda()
    mp = torch.from_numpy(mapping).cuda()
    assert K.validate_block_mapping(t, t, mp) == 0
    K.kv_block_copy(t, t, mp)
    torch.cuda.synchronize()
    assert np.array_equal(t.cpu().numpy(), want)
    # validation catches what the fast path does not check
    dup = torch.tensor([[1, 5], [2, 5]], dtype=torch.int64, device="cuda")
    assert K.validate_block_mapping(t, t, dup) == -9
    ovl = torch.tensor([[1, 5], [5, 6]], dtype=torch.int64, device="cuda")
    assert K.validate_block_mapping(t, t, ovl) == -10
    oob = torch.tensor([[1, 32]], dtype=torch.int64, device="cuda")
    assert K.validate_block_mapping(t, t, oob) == -8


def test_block_copy_strided_planes(oracle_mod):
    """Planes that are slices of a larger allocation (plane stride > num_blocks * block_bytes)."""
    import paper_2503_13773_amd as K
    rng = np.random.default_rng(5)
    big = rng.integers(0, 256, (3, 20, 512), dtype=np.uint8)     # use blocks 0..11 of each plane
    dst = rng.integers(0, 256, (3, 9, 512), dtype=np.uint8)
    mapping = W.make_copy_mapping(rng, 6, 12, 9)
    want = dst.copy()
    oracle_mod.kv_block_copy(np.ascontiguousarray(big[:, :12]), want, mapping)
    tb = torch.from_numpy(big).cuda()
    td = torch.from_numpy(dst).cuda()
    src_pool = K.Pool(base=tb.data_ptr(), num_blocks=12, block_bytes=512, plane_stride_bytes=20 * 512,
                      num_planes=3, reserved=0)
    K.kv_block_copy(src_pool, td, torch.from_numpy(mapping).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(td.cpu().numpy(), want)


@pytest.mark.parametrize("full", [False, True])
def test_swap_out_poison_swap_in_round_trip(oracle_mod, full):
    """cfg5 protocol: 20 % of sequences swapped to a second device pool and back into other
    slots; copies bit-exact against the oracle, attention output bit-identical afterwards."""
    import paper_2503_13773_amd as K
    w = W.make_config("cfg5") if full else W.make_config("cfg5", num_seqs=20, ctx_scale=0.3)
    sp = w.extra["swap"]
    assert sp["victims"] and (not full or sp["out_mapping"].shape[0] > 200)
    print(f"[case] swap full={full} victims={len(sp['victims'])} blocks={sp['out_mapping'].shape[0]}",
          flush=True)
    d = to_device(w)
    before = out_bits(run_gpu(w, d))

    pool1 = torch.stack([d["k"], d["v"]])                      # [2 planes][NB][Hkv][Bs][D]
    shape2 = (2, sp["pool2_blocks"]) + tuple(pool1.shape[2:])
    pool2 = torch.zeros(shape2, dtype=pool1.dtype, device="cuda")
    out_map = torch.from_numpy(sp["out_mapping"]).cuda()
    in_map = torch.from_numpy(sp["in_mapping"]).cuda()
    assert K.validate_block_mapping(pool1, pool2, out_map) == 0
    assert K.validate_block_mapping(pool2, pool1, in_map) == 0

    # oracle on host copies of the same bytes
    h1 = np.stack([w.k_cache, w.v_cache])
    h2 = np.zeros(shape2, dtype=np.uint16)
    oracle_mod.kv_block_copy(h1, h2, sp["out_mapping"])
    K.kv_block_copy(pool1, pool2, out_map)
    torch.cuda.synchronize()
    assert np.array_equal(pool2.view(torch.int16).cpu().numpy().view(np.uint16), h2)

    victims_blocks = torch.from_numpy(sp["out_mapping"][:, 0]).cuda()
    pool1[:, victims_blocks] = float("nan")                    # poison the swapped-out originals
    h1[:, sp["out_mapping"][:, 0]] = np.uint16(0x7FC0)
    oracle_mod.kv_block_copy(h2, h1, sp["in_mapping"])
    K.kv_block_copy(pool2, pool1, in_map)
    torch.cuda.synchronize()
    got1 = pool1.view(torch.int16).cpu().numpy().view(np.uint16)
    keep = np.ones(h1.shape[1], dtype=bool)
    keep[sp["out_mapping"][:, 0]] = False                       # NaN payload bits may differ
    assert np.array_equal(got1[:, keep], h1[:, keep])

    d2 = dict(d, k=pool1[0].contiguous(), v=pool1[1].contiguous(),
              tables=torch.from_numpy(sp["tables_after"]).cuda())
    after = out_bits(run_gpu(w, d2))
    assert np.array_equal(before, after)
    # every element of the post-swap attention against the oracle on the post-swap host pools
    ref = oracle_mod.paged_attention_decode(w.q, h1[0], h1[1], sp["tables_after"], w.context_lens,
                                            w.scale, dtype="bf16", num_threads=8)
    got = run_gpu(w, d2).float().cpu().numpy().astype(np.float64)
    assert np.isfinite(ref).all() and np.isfinite(got).all()
    assert np.abs(got - ref).max() <= 2e-2


def test_swap_to_pinned_host_memory_and_back(oracle_mod):
    """The swap of the paper moves KV to CPU memory: one pool is pinned host memory that the
    kernel writes / reads over PCIe.  Both directions bit-exact against the oracle."""
    import paper_2503_13773_amd as K
    rng = np.random.default_rng(21)
    planes, nb, nb_host, bb = 4, 40, 12, 32768
    dev = rng.integers(0, 256, (planes, nb, bb), dtype=np.uint8)
    out_map = W.make_copy_mapping(rng, 9, nb, nb_host)
    host_want = np.zeros((planes, nb_host, bb), dtype=np.uint8)
    oracle_mod.kv_block_copy(dev, host_want, out_map)
    tdev = torch.from_numpy(dev).cuda()
    thost = torch.zeros((planes, nb_host, bb), dtype=torch.uint8, pin_memory=True)
    K.kv_block_copy(tdev, thost, torch.from_numpy(out_map).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(thost.numpy(), host_want)
    # back into other device slots
    free = np.setdiff1d(np.arange(nb), out_map[:, 0])
    in_map = np.stack([out_map[:, 1], rng.permutation(free)[:9]], axis=1).astype(np.int64)
    dev_want = dev.copy()
    oracle_mod.kv_block_copy(host_want, dev_want, in_map)
    K.kv_block_copy(thost, tdev, torch.from_numpy(in_map).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(tdev.cpu().numpy(), dev_want)
    with pytest.raises(ValueError):
        K.pool_of(torch.zeros((planes, nb_host, bb), dtype=torch.uint8))   # pageable host memory is refused
