"""Parity of the HIP paged decode attention with the fp64 oracle (needs an MI355X).

Every case calls the kernels through the C ABI (ctypes binding) on seeded inputs and
compares with oracle.paged_attention_decode element by element: max-abs error <= 2e-2
for bf16 tensors and <= 1e-5 for fp32 tensors.
"""
import numpy as np
import pytest
import torch

import kvc_workloads as W
from gpu_util import BF16_TOL, F32_TOL, dev_tensor, out_bits, out_to_f64, run_gpu, to_device, tol_of

pytestmark = pytest.mark.gpu

VALU, MFMA, MFMA_LDS, BALANCED = 1, 2, 3, 4


def check(w, oracle_mod, label, **opts):
    print(f"[case] {label} {w.name} nseq={w.num_seqs} opts={opts}", flush=True)
    got = out_to_f64(run_gpu(w, **opts))
    ref = oracle_mod.attention_of_workload(w, num_threads=8)
    err = np.abs(got - ref).max()
    assert np.isfinite(got).all()
    assert err <= tol_of(w), (label, err)
    return err


def custom(seed, *, dtype, lens, hq, hkv, d, bs, nb_extra=7, lmax=None, name="custom"):
    rng = np.random.default_rng(seed)
    lens = np.asarray(lens, dtype=np.int32)
    nblk = W.blocks_needed(lens, bs)
    lmax = lmax or int(max(1, nblk.max())) + 2
    return W.build_workload(name, rng, dtype=dtype, context_lens=lens, num_q_heads=hq,
                            num_kv_heads=hkv, head_dim=d, block_size=bs, max_blocks_per_seq=lmax,
                            num_pool_blocks=int(nblk.sum()) + nb_extra)


# ---------------------------------------------------------------------------
# the named configurations at oracle-sized scale, every element compared
# ---------------------------------------------------------------------------
def test_cfg1_tiny_fp32(oracle_mod):
    w = W.make_config("cfg1")
    check(w, oracle_mod, "cfg1")
    check(w, oracle_mod, "cfg1 split", partition_tokens=64)
    check(w, oracle_mod, "cfg1 loose bound", tight=False)


@pytest.mark.parametrize("kernel", [VALU, MFMA, MFMA_LDS, BALANCED])
@pytest.mark.parametrize("name,nseq,scale", [("cfg2", 6, 0.5), ("cfg3", 12, 0.5), ("cfg4", 2, 0.04),
                                             ("cfg5", 16, 0.5)])
def test_configs_small_every_element(oracle_mod, name, nseq, scale, kernel):
    w = W.make_config(name, num_seqs=nseq, ctx_scale=scale)
    check(w, oracle_mod, f"{name} small", kernel=kernel)
    check(w, oracle_mod, f"{name} small pt=64", kernel=kernel, partition_tokens=64)


# ---------------------------------------------------------------------------
# the named configurations at full size, in the launch configuration the bench times:
# every (sequence, head, dim) element against the oracle
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["cfg2", "cfg3", "cfg3b", "cfg4", "cfg5"])
def test_configs_full_size_every_element(oracle_mod, name):
    import paper_2503_13773_amd as K
    w = W.make_config(name)
    print(f"[case] full {name} mean ctx {w.context_lens.mean():.0f}", flush=True)
    d = to_device(w)
    desc = K.attn_desc(d["q"], d["k"], d["tables"], max_context_len=w.max_context_len)
    plan = K.attn_plan(desc)
    assert plan.kernel == BALANCED           # what bench.py times
    # how the kernel cuts this batch: rows split over workers are merged by the last to arrive
    min_chunk = plan.partition_tokens // 16
    tiles = -(-w.context_lens.astype(np.int64) // 16)
    units = np.where(tiles > 0, tiles + 1, 0)           # one flat unit charged per non-empty row
    total = int(units.sum()) * w.num_kv_heads
    chunk = max(min_chunk, -(-total // (plan.partial_grid * 4)))
    pref = np.concatenate([[0], np.cumsum(units)[:-1]]) * w.num_kv_heads
    cut, worst = 0, 0
    for n in np.nonzero(tiles)[0]:
        for g in range(w.num_kv_heads):
            f = int(pref[n] + g * units[n])
            c = (f + int(tiles[n]) - 1) // chunk - f // chunk + 1
            cut += c > 1
            worst = max(worst, c)
    print(f"[case] full {name} chunk {chunk} tiles, {cut} cut rows, at most {worst} partials per row",
          flush=True)
    assert cut > 0 and plan.merge_grid == 0
    got = out_to_f64(run_gpu(w, d))
    assert np.isfinite(got).all()
    ref = oracle_mod.attention_of_workload(w, num_threads=8)
    assert np.isfinite(ref).all()
    err = np.abs(got - ref).max()
    print(f"[case] full {name} max abs err {err:.3e}", flush=True)
    assert err <= BF16_TOL, (name, err)


# ---------------------------------------------------------------------------
# shapes, tails and degenerate cases
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("kernel", [VALU, MFMA, MFMA_LDS, BALANCED])
def test_ragged_tails_and_partition_edges(oracle_mod, kernel):
    lens = [1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 300, 511, 512, 513]
    w = custom(101, dtype=W.BF16, lens=lens, hq=8, hkv=2, d=128, bs=16)
    for pt in (0, 16, 64, 128, 256):
        check(w, oracle_mod, f"tails pt={pt}", kernel=kernel, partition_tokens=pt)


@pytest.mark.parametrize("hkv", [1, 2, 8])
def test_balanced_ranges_cross_rows_and_skip_empty_sequences(oracle_mod, hkv):
    """Worker ranges of the balanced kernel start and end inside rows, span several short rows
    and step over empty sequences (also at both ends of the batch)."""
    lens = [0, 0, 5, 16, 17, 0, 33, 1, 250, 0, 0, 47, 48, 49, 700, 3, 0, 90, 16, 0]
    w = custom(120 + hkv, dtype=W.BF16, lens=lens, hq=2 * hkv, hkv=hkv, d=128, bs=16)
    w.block_tables[np.asarray(lens) == 0, :] = -1
    for chunk_tokens in (16, 48, 80, 112, 176, 1024):
        check(w, oracle_mod, f"balanced chunk={chunk_tokens}", kernel=BALANCED,
              partition_tokens=chunk_tokens)
    w2 = custom(130 + hkv, dtype=W.BF16, lens=[0, 0, 0], hq=2 * hkv, hkv=hkv, d=128, bs=16)
    check(w2, oracle_mod, "balanced all empty", kernel=BALANCED)


@pytest.mark.parametrize("hq,hkv", [(1, 1), (2, 1), (3, 1), (4, 1), (8, 1), (16, 1), (12, 4), (5, 5), (40, 8)])
def test_group_sizes(oracle_mod, hq, hkv):
    w = custom(102, dtype=W.BF16, lens=[40, 200, 77], hq=hq, hkv=hkv, d=128, bs=16)
    for kernel in (VALU, MFMA, MFMA_LDS, BALANCED):
        check(w, oracle_mod, f"group {hq}/{hkv}", kernel=kernel, partition_tokens=64)


def test_group_larger_than_16_takes_valu(oracle_mod):
    import paper_2503_13773_amd as K
    w = custom(103, dtype=W.BF16, lens=[50, 90], hq=32, hkv=1, d=128, bs=16)
    d = to_device(w)
    desc = K.attn_desc(d["q"], d["k"], d["tables"])
    assert K.attn_plan(desc).kernel == VALU
    check(w, oracle_mod, "group 32")
    for kernel in (MFMA, BALANCED):
        with pytest.raises(K.KvcError):
            run_gpu(w, kernel=kernel)


@pytest.mark.parametrize("bs", [1, 2, 4, 8, 16, 32, 64])
def test_block_sizes(oracle_mod, bs):
    w = custom(104, dtype=W.BF16, lens=[5, 70, 131], hq=8, hkv=2, d=128, bs=bs)
    check(w, oracle_mod, f"bs={bs} valu", kernel=VALU, partition_tokens=64)
    if bs >= 16:
        check(w, oracle_mod, f"bs={bs} mfma", kernel=MFMA, partition_tokens=64)
        check(w, oracle_mod, f"bs={bs} mfma lds", kernel=MFMA_LDS, partition_tokens=64)
    if bs >= 4:
        check(w, oracle_mod, f"bs={bs} balanced", kernel=BALANCED, partition_tokens=16)
        check(w, oracle_mod, f"bs={bs} balanced auto chunk", kernel=BALANCED)
    wf = custom(105, dtype=W.F32, lens=[5, 70, 131], hq=4, hkv=2, d=64, bs=bs)
    check(wf, oracle_mod, f"bs={bs} f32", partition_tokens=32)


@pytest.mark.parametrize("dtype,d", [(W.F32, 64), (W.F32, 128), (W.BF16, 64), (W.BF16, 128)])
def test_dtype_head_dim_grid(oracle_mod, dtype, d):
    w = custom(106, dtype=dtype, lens=[33, 260, 9, 100], hq=8, hkv=4, d=d, bs=16)
    check(w, oracle_mod, f"{dtype} d={d}")
    check(w, oracle_mod, f"{dtype} d={d} pt=48", partition_tokens=48)


def test_fp32_long_context_stays_within_1e5(oracle_mod):
    w = custom(107, dtype=W.F32, lens=[4096, 3000], hq=2, hkv=2, d=64, bs=16)
    assert check(w, oracle_mod, "f32 long") <= F32_TOL


@pytest.mark.parametrize("kernel", [VALU, MFMA, MFMA_LDS, BALANCED])
def test_maximum_partition_length(oracle_mod, kernel):
    w = custom(108, dtype=W.BF16, lens=[4096, 4095, 8200], hq=4, hkv=1, d=128, bs=16)
    check(w, oracle_mod, "pt=4096", kernel=kernel, partition_tokens=4096)


@pytest.mark.parametrize("bs", [4, 8])
def test_small_blocks_on_the_matrix_core_path(oracle_mod, bs):
    """block_size 8 (the paper's default) and 4: a 16-token tile spans 2 or 4 blocks, the last
    tile may touch blocks that were never allocated (table entries poisoned)."""
    import paper_2503_13773_amd as K
    lens = [1, 3, 4, 5, 7, 8, 9, 12, 13, 15, 16, 17, 20, 31, 33, 100, 257, 1000]
    w = custom(150 + bs, dtype=W.BF16, lens=lens, hq=8, hkv=2, d=128, bs=bs)
    d = to_device(w)
    assert K.attn_plan(K.attn_desc(d["q"], d["k"], d["tables"])).kernel == BALANCED
    nblk = W.blocks_needed(w.context_lens, bs)
    for n in range(w.num_seqs):
        w.block_tables[n, nblk[n]:] = 2 ** 30 if n % 2 else -1
        L = int(w.context_lens[n])
        if L % bs:
            w.k_cache[w.block_tables[n, nblk[n] - 1], :, L % bs:, :] = np.uint16(0x7FC0)
            w.v_cache[w.block_tables[n, nblk[n] - 1], :, L % bs:, :] = np.uint16(0x7FC0)
    for chunk in (0, 16, 48, 160):
        check(w, oracle_mod, f"bs={bs} chunk={chunk}", kernel=BALANCED, partition_tokens=chunk)
    check(w, oracle_mod, f"bs={bs} auto")


def test_balanced_ranges_longer_than_the_staging_window(oracle_mod):
    """A worker range of 512 tiles makes the balanced kernel refill its LDS window of tile
    addresses (256 entries) mid-range, also across a row change."""
    w = custom(140, dtype=W.BF16, lens=[20000, 37, 9000], hq=2, hkv=1, d=128, bs=16)
    check(w, oracle_mod, "balanced chunk=8192", kernel=BALANCED, partition_tokens=8192)
    w2 = custom(141, dtype=W.BF16, lens=[6000, 6000], hq=8, hkv=2, d=128, bs=32)
    check(w2, oracle_mod, "balanced chunk=4800", kernel=BALANCED, partition_tokens=4800)


@pytest.mark.parametrize("dtype,kernels", [(W.F32, [VALU]), (W.BF16, [VALU, MFMA, MFMA_LDS, BALANCED])])
def test_context_one_returns_v_bit_exactly(dtype, kernels):
    d_ = 64 if dtype == W.F32 else 128
    w = custom(109, dtype=dtype, lens=[1, 1, 1, 1], hq=8, hkv=2, d=d_, bs=16)
    for kernel in kernels:
        for pt in (0, 16):   # pt=16 with the loose bound goes through empty partitions
            out = run_gpu(w, kernel=kernel, partition_tokens=pt, tight=(pt == 0))
            bits = out_bits(out)
            for n in range(4):
                blk = w.block_tables[n, 0]
                for h in range(8):
                    want = w.v_cache[blk, h // 4, 0, :]
                    want = want.view(np.int16) if dtype == W.BF16 else want.view(np.int32)
                    assert np.array_equal(bits[n, h], want), (kernel, pt, n, h)


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_context_zero_gives_zeros_and_leaves_neighbours_alone(oracle_mod, dtype):
    d_ = 64 if dtype == W.F32 else 128
    w = custom(110, dtype=dtype, lens=[0, 37, 0, 300, 0], hq=4, hkv=2, d=d_, bs=16)
    w.block_tables[[0, 2, 4], :] = -1
    kernels = [VALU] if dtype == W.F32 else [VALU, MFMA, MFMA_LDS, BALANCED]
    ref = oracle_mod.attention_of_workload(w)
    for kernel in kernels:
        for pt in (0, 64):
            dv = to_device(w)
            import paper_2503_13773_amd as K
            out = torch.full_like(dv["q"], 7.0)
            K.paged_attention_decode(dv["q"], dv["k"], dv["v"], dv["tables"], dv["lens"], w.scale,
                                     out, kernel=kernel, partition_tokens=pt, max_context_len=300)
            got = out_to_f64(out)
            assert np.array_equal(got[[0, 2, 4]], np.zeros_like(got[[0, 2, 4]]))
            assert np.abs(got - ref).max() <= tol_of(w)


@pytest.mark.parametrize("kernel", [VALU, MFMA, MFMA_LDS, BALANCED])
def test_poison_beyond_context_and_in_unused_entries(oracle_mod, kernel):
    """NaN in slots past the context, in unused blocks; -1 / huge ids in unused table entries."""
    w = custom(111, dtype=W.BF16, lens=[5, 16, 17, 100, 250, 1], hq=8, hkv=2, d=128, bs=16, nb_extra=9)
    clean = out_bits(run_gpu(w, kernel=kernel, partition_tokens=64))
    nan = np.uint16(0x7FC0)
    used = np.zeros(w.num_pool_blocks, dtype=bool)
    nblk = W.blocks_needed(w.context_lens, 16)
    for n, L in enumerate(w.context_lens):
        used[w.block_tables[n, :nblk[n]]] = True
        if L % 16:
            b = w.block_tables[n, nblk[n] - 1]
            w.k_cache[b, :, L % 16:, :] = nan
            w.v_cache[b, :, L % 16:, :] = nan
        w.block_tables[n, nblk[n]:] = 2 ** 30 if n % 2 else -1
    w.k_cache[~used] = nan
    w.v_cache[~used] = nan
    dirty = out_bits(run_gpu(w, kernel=kernel, partition_tokens=64))
    assert np.array_equal(clean, dirty)
    check(w, oracle_mod, "poisoned", kernel=kernel, partition_tokens=64)


@pytest.mark.parametrize("kernel", [VALU, MFMA, MFMA_LDS, BALANCED])
def test_placement_invariance_is_bitwise_on_gpu(kernel):
    """Same logical KV at another physical placement / pool size: identical output bits."""
    w = custom(112, dtype=W.BF16, lens=[70, 300, 33], hq=8, hkv=2, d=128, bs=16)
    a = out_bits(run_gpu(w, kernel=kernel, partition_tokens=128))
    rng = np.random.default_rng(5)
    nb2 = w.num_pool_blocks + 11
    perm = rng.permutation(nb2)[:w.num_pool_blocks]
    k2 = np.zeros((nb2,) + w.k_cache.shape[1:], dtype=np.uint16)
    v2 = np.zeros_like(k2)
    k2[perm] = w.k_cache
    v2[perm] = w.v_cache
    t2 = w.block_tables.copy()
    t2[t2 >= 0] = perm[t2[t2 >= 0]]
    w.k_cache, w.v_cache, w.block_tables, w.num_pool_blocks = k2, v2, t2, nb2
    b = out_bits(run_gpu(w, kernel=kernel, partition_tokens=128))
    assert np.array_equal(a, b)


def test_shared_prefix_equals_private_copies(oracle_mod):
    """Block ids referenced by several tables give what private copies of the same data give."""
    w = W.make_config("cfg5", num_seqs=24, ctx_scale=0.4)
    assert w.extra["share_groups"]
    shared = out_bits(run_gpu(w))
    nblk = W.blocks_needed(w.context_lens, 16)
    total = int(nblk.sum())
    k2 = np.zeros((total,) + w.k_cache.shape[1:], dtype=np.uint16)
    v2 = np.zeros_like(k2)
    t2 = np.full_like(w.block_tables, -1)
    pos = 0
    for n in range(w.num_seqs):
        ids = w.block_tables[n, :nblk[n]]
        k2[pos:pos + nblk[n]] = w.k_cache[ids]
        v2[pos:pos + nblk[n]] = w.v_cache[ids]
        t2[n, :nblk[n]] = np.arange(pos, pos + nblk[n])
        pos += nblk[n]
    w.k_cache, w.v_cache, w.block_tables, w.num_pool_blocks = k2, v2, t2, total
    private = out_bits(run_gpu(w))
    assert np.array_equal(shared, private)


@pytest.mark.parametrize("kernel", [VALU, MFMA, BALANCED])
def test_partial_then_merge_equals_the_fused_call(kernel):
    import paper_2503_13773_amd as K
    w = W.make_config("cfg3", num_seqs=8, ctx_scale=0.5)
    d = to_device(w)
    desc = K.attn_desc(d["q"], d["k"], d["tables"], max_context_len=w.max_context_len, kernel=kernel,
                       partition_tokens=64)
    assert (K.attn_plan(desc).merge_grid == 0) == (kernel == BALANCED)   # balanced: one launch
    ws = K.new_workspace(desc)
    a = K.paged_attention_decode(d["q"], d["k"], d["v"], d["tables"], d["lens"], w.scale, desc=desc,
                                 workspace=ws)
    b = torch.zeros_like(d["q"])
    K.paged_attention_decode_partial(d["q"], d["k"], d["v"], d["tables"], d["lens"], w.scale, b, desc, ws)
    K.paged_attention_decode_merge(d["lens"], b, desc, ws)
    torch.cuda.synchronize()
    assert np.array_equal(out_bits(a), out_bits(b))


def test_one_workspace_serves_call_after_call_without_another_init(oracle_mod):
    """The arrival counters in the workspace header start at 0 (one init after allocation) and
    every call leaves them at 0: different batches, chunk lengths and kernels then share the
    workspace back to back, results do not depend on which wavefront arrived last (repeats are
    bit-identical), and the header reads 0 after each call."""
    import paper_2503_13773_amd as K
    cases = [(W.make_config("cfg3b"), dict()),
             (W.make_config("cfg3", num_seqs=12, ctx_scale=0.5), dict(partition_tokens=16)),
             (W.make_config("cfg3", num_seqs=12, ctx_scale=0.5), dict(kernel=MFMA, partition_tokens=64)),
             (W.make_config("cfg4", num_seqs=2, ctx_scale=0.1), dict(partition_tokens=32)),
             (W.make_config("cfg3b"), dict())]
    descs, devs = [], []
    for w, o in cases:
        d = to_device(w)
        devs.append(d)
        descs.append(K.attn_desc(d["q"], d["k"], d["tables"], max_context_len=w.max_context_len, **o))
    ws = torch.full((max(K.workspace_bytes(x) for x in descs),), 0xAB, dtype=torch.uint8, device="cuda")
    K.workspace_init(ws)
    first = {}
    for rep in range(40):  # slots keep another batch's partials between calls: a piece read too early shows
        for i, ((w, o), d, desc) in enumerate(zip(cases, devs, descs)):
            if rep < 2:
                print(f"[case] shared workspace rep {rep} case {i} {w.name} {o}", flush=True)
            out = K.paged_attention_decode(d["q"], d["k"], d["v"], d["tables"], d["lens"], w.scale,
                                           desc=desc, workspace=ws)
            torch.cuda.synchronize()
            assert int(ws[:4096].max()) == 0, "counter header not left at zero"
            bits = out_bits(out)
            if rep == 0:
                first[i] = bits
                ref = oracle_mod.attention_of_workload(w, num_threads=8)
                assert np.abs(out_to_f64(out) - ref).max() <= BF16_TOL
            else:
                assert np.array_equal(bits, first[i]), (rep, i)


def test_cut_rows_merge_the_same_bits_launch_after_launch():
    """Partials travel between wavefronts on different XCDs inside one launch.  300 launches over
    rotating replicas of the batch (cold caches, varying arrival order) must all give the bits
    of the first, which is checked against the oracle elsewhere."""
    import paper_2503_13773_amd as K
    w = W.make_config("cfg3b")
    devs = [to_device(w) for _ in range(4)]
    desc = K.attn_desc(devs[0]["q"], devs[0]["k"], devs[0]["tables"], max_context_len=w.max_context_len)
    ws = K.new_workspace(desc)
    outs = [torch.empty_like(devs[0]["q"]) for _ in range(300)]
    for i, o in enumerate(outs):
        d = devs[i % 4]
        K.paged_attention_decode(d["q"], d["k"], d["v"], d["tables"], d["lens"], w.scale, o, desc=desc,
                                 workspace=ws)
    torch.cuda.synchronize()
    first = out_bits(outs[0])
    bad = [i for i, o in enumerate(outs) if not np.array_equal(out_bits(o), first)]
    assert not bad, bad[:10]
    assert int(ws[:4096].max()) == 0


def test_runs_on_a_side_stream_and_validates_inputs():
    import paper_2503_13773_amd as K
    w = W.make_config("cfg3", num_seqs=4, ctx_scale=0.3)
    d = to_device(w)
    ref = out_bits(run_gpu(w, d))
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        out = K.paged_attention_decode(d["q"], d["k"], d["v"], d["tables"], d["lens"], w.scale,
                                       max_context_len=w.max_context_len)
    s.synchronize()
    assert np.array_equal(out_bits(out), ref)
    desc = K.attn_desc(d["q"], d["k"], d["tables"], max_context_len=w.max_context_len)
    assert K.validate_attention_inputs(d["tables"], d["lens"], desc) == 0
    bad = d["tables"].clone()
    bad[1, 0] = w.num_pool_blocks
    assert K.validate_attention_inputs(bad, d["lens"], desc) == -8
    long = d["lens"].clone()
    long[0] = w.max_context_len + 1
    assert K.validate_attention_inputs(d["tables"], long, desc) == -8


@pytest.mark.parametrize("nseq", [63, 64, 65, 255, 256, 257, 1100, 4096, 4200])
def test_large_batches_of_short_sequences(oracle_mod, nseq):
    """4096 sequences is the limit of the balanced kernel (its prefix sum lives in LDS), 4200 takes
    the fixed-partition kernel; contexts of 0 to 80 tokens make every worker cross many rows.  Up
    to 256 sequences a worker is placed by a count over the prefix table, one entry per lane and
    64 per pass (empty sequences are ties in that table), beyond that by a binary search."""
    import paper_2503_13773_amd as K
    rng = np.random.default_rng(500 + nseq)
    lens = rng.integers(0, 81, nseq).astype(np.int32)
    w = custom(500 + nseq, dtype=W.BF16, lens=lens, hq=8, hkv=2, d=128, bs=16, name=f"short{nseq}")
    d = to_device(w)
    plan = K.attn_plan(K.attn_desc(d["q"], d["k"], d["tables"], max_context_len=80))
    assert plan.kernel == (BALANCED if nseq <= 4096 else MFMA)
    check(w, oracle_mod, f"{nseq} short sequences")


# ---------------------------------------------------------------------------
# schedule built once per iteration, reused by the layers
# ---------------------------------------------------------------------------
def _scheduled_equals_direct(w, oracle_mod, label, **opts):
    import paper_2503_13773_amd as K
    d = to_device(w)
    desc = K.attn_desc(d["q"], d["k"], d["tables"], max_context_len=max(1, w.max_context_len), kernel=BALANCED, **opts)
    assert K.schedule_bytes(desc) > 0
    print(f"[case] scheduled {label} {w.name} nseq={w.num_seqs} opts={opts} schedule {K.schedule_bytes(desc)} B", flush=True)
    ws = K.new_workspace(desc)
    direct = K.paged_attention_decode(d["q"], d["k"], d["v"], d["tables"], d["lens"], w.scale, desc=desc, workspace=ws)
    sched = K.attn_schedule_build(d["tables"], d["lens"], desc)
    # the block table and the lengths are not read by the scheduled call: poison them
    d["tables"].fill_(-7)
    d["lens"].fill_(-7)
    outs = []
    for layer in range(3):                      # "layers": the same schedule, other q each time would do as well
        outs.append(K.paged_attention_decode_scheduled(d["q"], d["k"], d["v"], sched, w.scale, None, desc, ws))
    torch.cuda.synchronize()
    for o in outs:
        assert np.array_equal(out_bits(o), out_bits(direct)), label
    ref = oracle_mod.attention_of_workload(w, num_threads=8)
    assert np.abs(out_to_f64(outs[-1]) - ref).max() <= tol_of(w)
    assert int(ws[:4096].max()) == 0


@pytest.mark.parametrize("name", ["cfg2", "cfg3b", "cfg4", "cfg5"])
def test_scheduled_call_equals_the_direct_call_full_size(oracle_mod, name):
    _scheduled_equals_direct(W.make_config(name), oracle_mod, "full")


def test_scheduled_call_on_ragged_empty_and_small_block_batches(oracle_mod):
    lens = [0, 0, 5, 16, 17, 0, 33, 1, 250, 0, 0, 47, 48, 49, 700, 3, 0, 90, 16, 0]
    for hkv in (1, 2):
        w = custom(620 + hkv, dtype=W.BF16, lens=lens, hq=2 * hkv, hkv=hkv, d=128, bs=16)
        w.block_tables[np.asarray(lens) == 0, :] = -1
        for chunk in (16, 48, 1024):
            _scheduled_equals_direct(w, oracle_mod, f"ragged chunk={chunk}", partition_tokens=chunk)
    for bs in (4, 8, 32):
        w = custom(630 + bs, dtype=W.BF16, lens=[1, 3, 9, 17, 100, 257, 1000], hq=8, hkv=2, d=128, bs=bs)
        _scheduled_equals_direct(w, oracle_mod, f"bs={bs}")
    w = custom(640, dtype=W.BF16, lens=[20000, 37, 9000], hq=2, hkv=1, d=128, bs=16)   # windows refilled from the schedule
    _scheduled_equals_direct(w, oracle_mod, "long ranges", partition_tokens=8192)
    w = custom(641, dtype=W.BF16, lens=[0, 0, 0], hq=4, hkv=2, d=128, bs=16)
    _scheduled_equals_direct(w, oracle_mod, "all empty")


def test_schedule_calls_refuse_what_they_cannot_serve():
    import ctypes
    import paper_2503_13773_amd as K
    w = W.make_config("cfg3", num_seqs=4, ctx_scale=0.3)
    d = to_device(w)
    valu = K.attn_desc(d["q"], d["k"], d["tables"], max_context_len=w.max_context_len, kernel=VALU)
    assert K.schedule_bytes(valu) == 0
    buf = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    L = K.lib()
    assert L.kvc_attn_schedule_build(d["tables"].data_ptr(), d["lens"].data_ptr(), ctypes.byref(valu),
                                     buf.data_ptr(), buf.numel(), None) == -4
    ok = K.attn_desc(d["q"], d["k"], d["tables"], max_context_len=w.max_context_len)
    assert L.kvc_attn_schedule_build(d["tables"].data_ptr(), d["lens"].data_ptr(), ctypes.byref(ok),
                                     buf.data_ptr(), 16, None) == -5
    assert L.kvc_attn_schedule_build(None, d["lens"].data_ptr(), ctypes.byref(ok), buf.data_ptr(), buf.numel(), None) == -1
