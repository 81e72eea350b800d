"""The C oracle against what the definition and the mathematics fix (no GPU)."""
import numpy as np
import pytest

import pins


def oracle_impl(oracle_mod):
    def impl(q, k, v, tables, lens, scale):
        return oracle_mod.paged_attention_decode(q, k, v, tables, lens, scale, dtype="f64")
    return impl


@pytest.mark.parametrize("pin", pins.ALL_PINS, ids=lambda f: f.__name__)
def test_oracle_attention_pin(oracle_mod, pin):
    pin(oracle_impl(oracle_mod))


def test_oracle_storage_dtypes_widen_exactly(oracle_mod):
    """bf16 / f32 storage gives the same result as the same values handed over as f64."""
    import kvc_workloads as W
    p = pins.random_problem(5, nseq=3, hq=4, hkv=2, d=8, bs=4, max_ctx=19)
    ref_f32 = oracle_mod.paged_attention_decode(
        p["q"].astype(np.float32).astype(np.float64), p["k"].astype(np.float32).astype(np.float64),
        p["v"].astype(np.float32).astype(np.float64), p["tables"], p["lens"], p["scale"], dtype="f64")
    got_f32 = oracle_mod.paged_attention_decode(
        p["q"].astype(np.float32), p["k"].astype(np.float32), p["v"].astype(np.float32),
        p["tables"], p["lens"], p["scale"], dtype="f32")
    assert np.array_equal(ref_f32, got_f32)
    qb, kb, vb = (W.f32_to_bf16_bits(x.astype(np.float32)) for x in (p["q"], p["k"], p["v"]))
    ref_bf = oracle_mod.paged_attention_decode(
        W.to_float64(qb, "bf16"), W.to_float64(kb, "bf16"), W.to_float64(vb, "bf16"),
        p["tables"], p["lens"], p["scale"], dtype="f64")
    got_bf = oracle_mod.paged_attention_decode(qb, kb, vb, p["tables"], p["lens"], p["scale"],
                                               dtype="bf16")
    assert np.array_equal(ref_bf, got_bf)
    # bf16 bit pattern 0x3FC0 is 1.5, 0xC000 is -2.0 (format definition)
    assert W.bf16_bits_to_f32(np.array([0x3FC0, 0xC000], dtype=np.uint16)).tolist() == [1.5, -2.0]


def test_oracle_row_subset_and_threads(oracle_mod):
    p = pins.random_problem(6, nseq=4, hq=4, hkv=2, d=8, bs=4, max_ctx=25)
    full = oracle_mod.paged_attention_decode(p["q"], p["k"], p["v"], p["tables"], p["lens"],
                                             p["scale"], dtype="f64")
    rows = [(0, 1), (3, 2), (2, 0)]
    sub = oracle_mod.paged_attention_decode(p["q"], p["k"], p["v"], p["tables"], p["lens"],
                                            p["scale"], dtype="f64", rows=rows)
    for n, h in rows:
        assert np.array_equal(sub[n, h], full[n, h])
    assert np.isnan(sub[1]).all()
    par = oracle_mod.paged_attention_decode(p["q"], p["k"], p["v"], p["tables"], p["lens"],
                                            p["scale"], dtype="f64", num_threads=4)
    assert np.array_equal(par, full)


def test_oracle_rejects_block_ids_outside_pool(oracle_mod):
    p = pins.random_problem(7, nseq=2, hq=2, hkv=1, d=4, bs=4, max_ctx=9)
    p["tables"][0, 0] = p["k"].shape[0]
    with pytest.raises(ValueError):
        oracle_mod.paged_attention_decode(p["q"], p["k"], p["v"], p["tables"], p["lens"],
                                          p["scale"], dtype="f64")


# ----------------------------------------------------------------------------
# block copy
# ----------------------------------------------------------------------------
def test_oracle_block_copy_matches_numpy_indexing(oracle_mod):
    rng = np.random.default_rng(8)
    src = rng.integers(0, 256, (3, 10, 48), dtype=np.uint8)
    dst = rng.integers(0, 256, (3, 7, 48), dtype=np.uint8)
    mapping = np.array([[9, 0], [2, 6], [2, 3], [5, 1]], dtype=np.int64)   # src 2 fans out
    want = dst.copy()
    want[:, mapping[:, 1]] = src[:, mapping[:, 0]]                         # numpy's own gather/scatter
    oracle_mod.kv_block_copy(src, dst, mapping)
    assert np.array_equal(dst, want)
    untouched = [b for b in range(7) if b not in mapping[:, 1]]
    assert len(untouched) == 3


def test_oracle_block_copy_hand_case(oracle_mod):
    """2 planes, 3 blocks of 2 bytes, hand-written expectation."""
    src = np.array([[[1, 2], [3, 4], [5, 6]], [[11, 12], [13, 14], [15, 16]]], dtype=np.uint8)
    dst = np.full((2, 2, 2), 99, dtype=np.uint8)
    oracle_mod.kv_block_copy(src, dst, np.array([[2, 0]], dtype=np.int64))
    assert dst.tolist() == [[[5, 6], [99, 99]], [[15, 16], [99, 99]]]


def test_oracle_block_copy_empty_and_bad_ids(oracle_mod):
    src = np.arange(24, dtype=np.uint8).reshape(1, 3, 8)
    dst = np.zeros((1, 3, 8), dtype=np.uint8)
    oracle_mod.kv_block_copy(src, dst, np.zeros((0, 2), dtype=np.int64))
    assert not dst.any()
    with pytest.raises(ValueError):
        oracle_mod.kv_block_copy(src, dst, np.array([[3, 0]], dtype=np.int64))
    with pytest.raises(ValueError):
        oracle_mod.kv_block_copy(src, dst, np.array([[0, -1]], dtype=np.int64))
    assert not dst.any()


def test_oracle_swap_round_trip_restores_attention(oracle_mod):
    """Swap a sequence's blocks out, poison them, swap back into other slots: same output bits."""
    p = pins.random_problem(9, nseq=3, hq=4, hkv=2, d=8, bs=4, max_ctx=22, nb=40)
    before = oracle_mod.paged_attention_decode(p["q"], p["k"], p["v"], p["tables"], p["lens"],
                                               p["scale"], dtype="f64")
    pool1 = np.stack([p["k"], p["v"]])                  # [2 planes][NB][Hkv][Bs][D]
    pool2 = np.zeros((2, 12) + p["k"].shape[1:])
    n = 1
    nblk = (p["lens"][n] + 3) // 4
    mine = p["tables"][n, :nblk].astype(np.int64)
    used = set(int(b) for row, L in zip(p["tables"], p["lens"]) for b in row[:(L + 3) // 4])
    free = np.array([b for b in range(40) if b not in used], dtype=np.int64)[:nblk]
    slot2 = np.arange(nblk, dtype=np.int64)[::-1].copy()
    oracle_mod.kv_block_copy(pool1, pool2, np.stack([mine, slot2], axis=1))
    pool1[:, mine] = np.nan
    oracle_mod.kv_block_copy(pool2, pool1, np.stack([slot2, free], axis=1))
    tables = p["tables"].copy()
    tables[n, :nblk] = free
    after = oracle_mod.paged_attention_decode(p["q"], pool1[0], pool1[1], tables, p["lens"],
                                              p["scale"], dtype="f64")
    assert np.array_equal(before, after)


# ----------------------------------------------------------------------------
# cache append
# ----------------------------------------------------------------------------
def test_oracle_cache_append_hand_case(oracle_mod):
    """2 sequences, 1 kv head, D=2, Bs=2, pool of 3 blocks; expectation written by hand."""
    k_cache = np.zeros((3, 1, 2, 2), dtype=np.float32)
    v_cache = np.zeros_like(k_cache)
    tables = np.array([[2, 0], [1, -1]], dtype=np.int32)
    k_new = np.array([[[1, 2]], [[3, 4]]], dtype=np.float32)
    v_new = np.array([[[5, 6]], [[7, 8]]], dtype=np.float32)
    # seq 0 writes position 3 = (table[0][1] = block 0, slot 1); seq 1 writes position 0 = (block 1, slot 0)
    oracle_mod.kv_cache_append(k_new, v_new, k_cache, v_cache, tables, np.array([3, 0], dtype=np.int32))
    assert k_cache.tolist() == [[[[0, 0], [1, 2]]], [[[3, 4], [0, 0]]], [[[0, 0], [0, 0]]]]
    assert v_cache.tolist() == [[[[0, 0], [5, 6]]], [[[7, 8], [0, 0]]], [[[0, 0], [0, 0]]]]


def test_oracle_cache_append_matches_numpy_indexing_and_skips_negative(oracle_mod):
    rng = np.random.default_rng(12)
    nseq, hkv, d, bs, nb, lmax = 5, 3, 8, 4, 30, 6
    k_cache = rng.standard_normal((nb, hkv, bs, d)).astype(np.float32)
    v_cache = rng.standard_normal((nb, hkv, bs, d)).astype(np.float32)
    tables = rng.permutation(nb)[:nseq * lmax].reshape(nseq, lmax).astype(np.int32)
    pos = np.array([0, 7, -1, 23, 10], dtype=np.int32)
    k_new = rng.standard_normal((nseq, hkv, d)).astype(np.float32)
    v_new = rng.standard_normal((nseq, hkv, d)).astype(np.float32)
    wk, wv = k_cache.copy(), v_cache.copy()
    for n in range(nseq):
        if pos[n] >= 0:
            wk[tables[n, pos[n] // bs], :, pos[n] % bs, :] = k_new[n]
            wv[tables[n, pos[n] // bs], :, pos[n] % bs, :] = v_new[n]
    oracle_mod.kv_cache_append(k_new, v_new, k_cache, v_cache, tables, pos)
    assert np.array_equal(k_cache, wk) and np.array_equal(v_cache, wv)
    with pytest.raises(ValueError):
        oracle_mod.kv_cache_append(k_new, v_new, k_cache, v_cache, tables, np.array([0, 0, 0, 24, 0], dtype=np.int32))


def test_oracle_append_then_attend_equals_attention_over_the_longer_sequence(oracle_mod):
    """Appending token L and attending over L+1 tokens equals attention on a cache built whole."""
    p = pins.random_problem(13, nseq=3, hq=4, hkv=2, d=8, bs=4, max_ctx=17, nb=40)
    lens = p["lens"].copy()
    full = oracle_mod.paged_attention_decode(p["q"], p["k"], p["v"], p["tables"], lens, p["scale"], dtype="f64")
    k2, v2 = p["k"].copy(), p["v"].copy()
    last = lens - 1
    k_new = np.stack([p["k"][p["tables"][n, last[n] // 4], :, last[n] % 4, :] for n in range(3)])
    v_new = np.stack([p["v"][p["tables"][n, last[n] // 4], :, last[n] % 4, :] for n in range(3)])
    for n in range(3):                                    # wipe the last token, then append it back
        k2[p["tables"][n, last[n] // 4], :, last[n] % 4, :] = 99.0
        v2[p["tables"][n, last[n] // 4], :, last[n] % 4, :] = 99.0
    oracle_mod.kv_cache_append(np.ascontiguousarray(k_new), np.ascontiguousarray(v_new), k2, v2,
                               p["tables"], last.astype(np.int32))
    again = oracle_mod.paged_attention_decode(p["q"], k2, v2, p["tables"], lens, p["scale"], dtype="f64")
    assert np.array_equal(full, again)


# ----------------------------------------------------------------------------
# causal (prefill / recompute) attention
# ----------------------------------------------------------------------------
def prefill_problem(seed, lens, qlens, hq=4, hkv=2, d=8, bs=4):
    p = pins.random_problem(seed, lens=lens, hq=hq, hkv=hkv, d=d, bs=bs)
    q_start = np.concatenate([[0], np.cumsum(qlens)]).astype(np.int32)
    p["q"] = np.random.default_rng(seed + 1).standard_normal((int(q_start[-1]), hq, d))
    p["q_start"] = q_start
    return p


def test_oracle_prefill_matches_dense_causal_bruteforce(oracle_mod):
    """Masked softmax with matrix ops + scipy on the un-paged sequence."""
    import scipy.special
    p = prefill_problem(201, lens=[13, 7, 20], qlens=[13, 3, 1])
    out = oracle_mod.paged_attention_prefill(p["q"], p["k"], p["v"], p["tables"], p["lens"], p["q_start"],
                                             p["scale"], dtype="f64")
    for n in range(3):
        Kd, Vd = pins.gather_dense(p, n)                                   # [S][Hkv][D]
        S, Qn = int(p["lens"][n]), int(p["q_start"][n + 1] - p["q_start"][n])
        qn = p["q"][p["q_start"][n]:p["q_start"][n + 1]]                   # [Qn][Hq][D]
        Kh, Vh = np.repeat(Kd, 2, axis=1), np.repeat(Vd, 2, axis=1)        # [S][Hq][D]
        sc = np.einsum("qhd,shd->hqs", qn, Kh) * p["scale"]
        pos = S - Qn + np.arange(Qn)
        sc = np.where(np.arange(S)[None, None, :] <= pos[None, :, None], sc, -np.inf)
        ref = np.einsum("hqs,shd->qhd", scipy.special.softmax(sc, axis=2), Vh)
        assert np.abs(out[p["q_start"][n]:p["q_start"][n + 1]] - ref).max() < 1e-12


def test_oracle_prefill_matches_library_causal_attention(oracle_mod):
    """torch scaled_dot_product_attention(is_causal=True), fp64, full recompute (Qn == S)."""
    import torch
    import torch.nn.functional as F
    p = prefill_problem(202, lens=[11], qlens=[11], hq=2, hkv=2, d=16)
    out = oracle_mod.paged_attention_prefill(p["q"], p["k"], p["v"], p["tables"], p["lens"], p["q_start"],
                                             p["scale"], dtype="f64")
    Kd, Vd = pins.gather_dense(p, 0)
    qh = torch.from_numpy(p["q"]).permute(1, 0, 2)[None]                   # [1][H][S][D]
    kh = torch.from_numpy(Kd).permute(1, 0, 2)[None]
    vh = torch.from_numpy(Vd).permute(1, 0, 2)[None]
    ref = F.scaled_dot_product_attention(qh, kh, vh, is_causal=True, scale=p["scale"])[0].permute(1, 0, 2).numpy()
    assert np.abs(out - ref).max() < 1e-12


def test_oracle_prefill_special_cases(oracle_mod):
    p = prefill_problem(203, lens=[9, 14], qlens=[9, 5])
    out = oracle_mod.paged_attention_prefill(p["q"], p["k"], p["v"], p["tables"], p["lens"], p["q_start"],
                                             p["scale"], dtype="f64")
    # position 0 sees one token: its v, bit-exactly
    for h in range(4):
        assert np.array_equal(out[0, h], p["v"][p["tables"][0, 0], h // 2, 0])
    # the last query row of every sequence equals decode attention with that row as the query
    last = p["q"][[8, 13]]
    dec = oracle_mod.paged_attention_decode(last, p["k"], p["v"], p["tables"], p["lens"], p["scale"], dtype="f64")
    assert np.abs(out[[8, 13]] - dec).max() < 1e-15
    # an earlier row equals decode attention over the truncated context
    dec5 = oracle_mod.paged_attention_decode(p["q"][[5]], p["k"], p["v"], p["tables"][:1],
                                             np.array([6], dtype=np.int32), p["scale"], dtype="f64")
    assert np.abs(out[5] - dec5[0]).max() < 1e-15
    # causality: changing tokens after position 4 of sequence 0 leaves rows 0..4 unchanged
    k2, v2 = p["k"].copy(), p["v"].copy()
    for t in range(5, 9):
        k2[p["tables"][0, t // 4], :, t % 4] += 3.0
        v2[p["tables"][0, t // 4], :, t % 4] -= 5.0
    out2 = oracle_mod.paged_attention_prefill(p["q"], k2, v2, p["tables"], p["lens"], p["q_start"],
                                              p["scale"], dtype="f64")
    assert np.array_equal(out[:5], out2[:5]) and np.abs(out[5:9] - out2[5:9]).max() > 1e-3
    with pytest.raises(ValueError):
        oracle_mod.paged_attention_prefill(p["q"], p["k"], p["v"], p["tables"], np.array([4, 14], dtype=np.int32),
                                           p["q_start"], p["scale"], dtype="f64")   # more queries than context
