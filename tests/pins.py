"""Pins for a paged decode-attention implementation.

Every check takes ``impl(q, k_cache, v_cache, block_tables, context_lens, scale)
-> float64 [num_seqs][Hq][D]`` on float64 inputs and raises AssertionError when
the implementation disagrees with what the definition and the mathematics fix.
None of the checks re-types the oracle's loop: they compare against hand-derived
values, closed forms, library routines (scipy softmax + matmul on the un-paged
sequence, torch's attention in fp64) and invariants.

``tests/test_oracle_pins.py`` runs them on the C oracle;
``tests/test_pins_have_teeth.py`` runs them on deliberately wrong
implementations and requires each one to be caught.
"""
from __future__ import annotations

import json
import math
import os

import numpy as np
import scipy.special

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


# ---------------------------------------------------------------------------
# helpers: random float64 problems (not the method: only inputs)
# ---------------------------------------------------------------------------
def random_problem(seed, nseq=3, hq=4, hkv=2, d=8, bs=4, max_ctx=23, nb=None, lens=None):
    rng = np.random.default_rng(seed)
    if lens is None:
        lens = rng.integers(1, max_ctx + 1, nseq)
    lens = np.asarray(lens, dtype=np.int32)
    nseq = len(lens)
    nblk = (lens + bs - 1) // bs
    lmax = int(max(1, nblk.max())) + 1
    need = int(nblk.sum())
    nb = nb or need + 5
    perm = rng.permutation(nb)[:need]
    tables = np.full((nseq, lmax), -1, dtype=np.int32)
    pos = 0
    for n in range(nseq):
        tables[n, :nblk[n]] = perm[pos:pos + nblk[n]]
        pos += nblk[n]
    q = rng.standard_normal((nseq, hq, d))
    k = rng.standard_normal((nb, hkv, bs, d))
    v = rng.standard_normal((nb, hkv, bs, d))
    return dict(q=q, k=k, v=v, tables=tables, lens=lens, scale=1.0 / math.sqrt(d))


def gather_dense(p, n):
    """Un-page sequence n: dense K, V of shape [L][Hkv][D] (numpy fancy indexing)."""
    L = int(p["lens"][n])
    bs = p["k"].shape[2]
    tok = np.arange(L)
    blk = p["tables"][n, tok // bs]
    return p["k"][blk, :, tok % bs, :], p["v"][blk, :, tok % bs, :]


def call(impl, p):
    return impl(p["q"], p["k"], p["v"], p["tables"], p["lens"], p["scale"])


# ---------------------------------------------------------------------------
# pins
# ---------------------------------------------------------------------------
def pin_golden_closed_forms(impl):
    """Hand-derived cases under tests/golden/ (weights are exact small fractions)."""
    with open(os.path.join(GOLDEN, "closed_form_cases.json")) as f:
        cases = json.load(f)["cases"]
    assert len(cases) >= 4
    for c in cases:
        out = impl(np.array(c["q"], dtype=np.float64), np.array(c["k_cache"], dtype=np.float64),
                   np.array(c["v_cache"], dtype=np.float64),
                   np.array(c["block_tables"], dtype=np.int32),
                   np.array(c["context_lens"], dtype=np.int32), float(c["scale"]))
        exp = np.array(c["expected"], dtype=np.float64)
        assert out.shape == exp.shape, c["name"]
        assert np.abs(out - exp).max() <= c["tol"], (c["name"], out, exp)


def pin_dense_bruteforce(impl):
    """softmax(q K^T scale) V with matrix ops + scipy softmax on the un-paged sequence."""
    for seed, kw in [(1, {}), (2, dict(hq=8, hkv=8, d=64, bs=16, max_ctx=100, nseq=4)),
                     (3, dict(hq=6, hkv=2, d=16, bs=8, max_ctx=70)),
                     (4, dict(hq=8, hkv=1, d=4, bs=1, max_ctx=9))]:
        p = random_problem(seed, **kw)
        out = call(impl, p)
        hq, hkv = p["q"].shape[1], p["k"].shape[1]
        G = hq // hkv
        for n in range(len(p["lens"])):
            Kd, Vd = gather_dense(p, n)                       # [L][Hkv][D]
            Kh = np.repeat(Kd, G, axis=1).transpose(1, 0, 2)  # [Hq][L][D]
            Vh = np.repeat(Vd, G, axis=1).transpose(1, 0, 2)
            S = np.einsum("hd,hld->hl", p["q"][n], Kh) * p["scale"]
            W = scipy.special.softmax(S, axis=1)
            ref = np.einsum("hl,hld->hd", W, Vh)
            assert np.abs(out[n] - ref).max() < 1e-12, (seed, n)


def pin_library_attention_fp64(impl):
    """torch.nn.functional.scaled_dot_product_attention, CPU, float64, one query row."""
    import torch
    import torch.nn.functional as F
    p = random_problem(11, nseq=3, hq=4, hkv=2, d=16, bs=4, max_ctx=37)
    out = call(impl, p)
    G = 2
    for n in range(3):
        Kd, Vd = gather_dense(p, n)
        Kh = torch.from_numpy(np.repeat(Kd, G, axis=1)).permute(1, 0, 2)[None]  # [1][Hq][L][D]
        Vh = torch.from_numpy(np.repeat(Vd, G, axis=1)).permute(1, 0, 2)[None]
        qh = torch.from_numpy(p["q"][n])[None, :, None, :]                       # [1][Hq][1][D]
        ref = F.scaled_dot_product_attention(qh, Kh, Vh, scale=p["scale"])[0, :, 0, :].numpy()
        assert np.abs(out[n] - ref).max() < 1e-12, n


def pin_context_one_is_v(impl):
    """A context of length 1 returns that token's v bit-exactly."""
    p = random_problem(21, lens=[1, 1, 1], hq=4, hkv=2, d=8, bs=4)
    out = call(impl, p)
    for n in range(3):
        blk = p["tables"][n, 0]
        for h in range(4):
            assert np.array_equal(out[n, h], p["v"][blk, h // 2, 0, :])


def pin_context_zero_is_zero(impl):
    p = random_problem(22, lens=[0, 5, 0], hq=2, hkv=1, d=4, bs=4)
    p["tables"][0, :] = -1
    p["tables"][2, :] = -1
    out = call(impl, p)
    assert np.array_equal(out[0], np.zeros_like(out[0]))
    assert np.array_equal(out[2], np.zeros_like(out[2]))
    assert np.isfinite(out[1]).all() and np.abs(out[1]).max() > 0


def pin_placement_invariance(impl):
    """Same logical K/V at two different physical placements / pool sizes: same output."""
    p = random_problem(31, nseq=4, hq=4, hkv=2, d=8, bs=4, max_ctx=30)
    out = call(impl, p)
    rng = np.random.default_rng(32)
    nb = p["k"].shape[0]
    nb2 = nb + 7
    perm = rng.permutation(nb2)[:nb]           # old block b -> new block perm[b]
    k2 = rng.standard_normal((nb2,) + p["k"].shape[1:])
    v2 = rng.standard_normal((nb2,) + p["v"].shape[1:])
    k2[perm] = p["k"]
    v2[perm] = p["v"]
    t2 = p["tables"].copy()
    t2[t2 >= 0] = perm[t2[t2 >= 0]]
    out2 = impl(p["q"], k2, v2, t2, p["lens"], p["scale"])
    assert np.array_equal(out, out2)           # same token order of summation => bitwise


def pin_token_order_permutation(impl):
    """Reordering whole blocks of a sequence (K and V together) only reorders the sums."""
    p = random_problem(33, lens=[16, 32], hq=2, hkv=2, d=8, bs=4)   # full blocks only
    out = call(impl, p)
    t2 = p["tables"].copy()
    t2[0, :4] = t2[0, :4][::-1]
    t2[1, :8] = np.roll(t2[1, :8], 3)
    out2 = impl(p["q"], p["k"], p["v"], t2, p["lens"], p["scale"])
    assert np.abs(out - out2).max() < 1e-13


def pin_equal_keys_give_mean_of_v(impl):
    p = random_problem(41, lens=[7, 13], hq=4, hkv=2, d=8, bs=4)
    for n in range(2):
        Kd, _ = gather_dense(p, n)
        for t in range(p["lens"][n]):
            p["k"][p["tables"][n, t // 4], :, t % 4, :] = Kd[0]     # every key = key of token 0
    out = call(impl, p)
    for n in range(2):
        _, Vd = gather_dense(p, n)
        mean = Vd.mean(axis=0)                                        # [Hkv][D]
        for h in range(4):
            assert np.abs(out[n, h] - mean[h // 2]).max() < 1e-13


def pin_zero_query_gives_mean_of_v(impl):
    p = random_problem(42, lens=[9, 4], hq=2, hkv=1, d=8, bs=4)
    p["q"][:] = 0.0
    out = call(impl, p)
    for n in range(2):
        _, Vd = gather_dense(p, n)
        assert np.abs(out[n] - Vd.mean(axis=0)[0][None]).max() < 1e-13


def pin_dominant_key_selects_its_v(impl):
    """One key scoring ~+200 above the rest: output is that token's v to ~e^-200."""
    p = random_problem(43, lens=[11], hq=1, hkv=1, d=8, bs=4)
    p["scale"] = 1.0
    p["q"][0, 0] = 0.0
    p["q"][0, 0, 3] = 1.0
    p["k"][:, :, :, 3] = 0.0
    t = 6
    p["k"][p["tables"][0, t // 4], 0, t % 4, 3] = 200.0
    out = call(impl, p)
    v = p["v"][p["tables"][0, t // 4], 0, t % 4]
    assert np.abs(out[0, 0] - v).max() < 1e-60 + 1e-15 * np.abs(v).max()


def pin_large_scores_are_stable(impl):
    """Scores in the thousands (exp would overflow without the max shift) stay finite and right."""
    p = random_problem(48, lens=[13], hq=2, hkv=1, d=8, bs=4)
    p["scale"] = 400.0
    out = call(impl, p)
    Kd, Vd = gather_dense(p, 0)
    S = np.einsum("hd,ld->hl", p["q"][0], Kd[:, 0]) * p["scale"]
    assert np.abs(S).max() > 800.0
    ref = scipy.special.softmax(S, axis=1) @ Vd[:, 0]
    assert np.isfinite(out).all() and np.abs(out[0] - ref).max() < 1e-12


def pin_constant_v_is_returned(impl):
    p = random_problem(44, lens=[19, 3], hq=4, hkv=2, d=8, bs=4)
    c = np.linspace(-2.0, 3.0, 8)
    p["v"][:] = c
    out = call(impl, p)
    assert np.abs(out - c).max() < 1e-14


def pin_softmax_shift_invariance(impl):
    """Adding one vector to every key shifts all scores by a constant: output unchanged."""
    p = random_problem(45, lens=[17, 6], hq=4, hkv=2, d=8, bs=4)
    out = call(impl, p)
    shift = np.random.default_rng(46).standard_normal(8)
    k2 = p["k"] + shift
    out2 = impl(p["q"], k2, p["v"], p["tables"], p["lens"], p["scale"])
    assert np.abs(out - out2).max() < 1e-12


def pin_scale_is_applied(impl):
    """Doubling scale equals doubling q; scale 0 gives the mean of v."""
    p = random_problem(47, lens=[10, 5], hq=2, hkv=1, d=8, bs=4)
    a = impl(p["q"], p["k"], p["v"], p["tables"], p["lens"], 2.0 * p["scale"])
    b = impl(2.0 * p["q"], p["k"], p["v"], p["tables"], p["lens"], p["scale"])
    assert np.abs(a - b).max() < 1e-12
    z = impl(p["q"], p["k"], p["v"], p["tables"], p["lens"], 0.0)
    for n in range(2):
        _, Vd = gather_dense(p, n)
        assert np.abs(z[n] - Vd.mean(axis=0)[0][None]).max() < 1e-13
    assert np.abs(a - call(impl, p)).max() > 1e-3


def pin_split_merge_algebra(impl):
    """Attention over [A;B] equals the log-sum-exp merge of attention over A and over B."""
    p = random_problem(51, lens=[24], hq=2, hkv=1, d=8, bs=4)
    full = call(impl, p)[0]
    Kd, Vd = gather_dense(p, 0)
    for cut_blocks in (0, 1, 4):
        cut = cut_blocks * 4
        parts = []
        for lo, hi in ((0, cut), (cut, 24)):
            if hi == lo:
                continue
            sub = dict(p)
            sub["tables"] = p["tables"][:, lo // 4:].copy()
            sub["lens"] = np.array([hi - lo], dtype=np.int32)
            o = call(impl, sub)[0]                                   # [Hq][D]
            s = np.einsum("hd,ld->hl", p["q"][0], Kd[lo:hi, 0]) * p["scale"]
            lse = scipy.special.logsumexp(s, axis=1)                 # [Hq]
            parts.append((o, lse))
        lses = np.stack([x[1] for x in parts])                       # [P][Hq]
        wts = scipy.special.softmax(lses, axis=0)
        merged = sum(w[:, None] * x[0] for w, x in zip(wts, parts))
        assert np.abs(merged - full).max() < 1e-12


def pin_gqa_equals_replicated_mha(impl):
    """Heads of a group with equal q give equal rows; GQA == MHA with G-fold replicated KV heads."""
    p = random_problem(61, nseq=2, hq=6, hkv=2, d=8, bs=4, max_ctx=21)
    p["q"][:, 1] = p["q"][:, 0]
    out = call(impl, p)
    assert np.array_equal(out[:, 0], out[:, 1])
    assert np.abs(out[:, 0] - out[:, 3]).max() > 1e-6
    k3 = np.repeat(p["k"], 3, axis=1)
    v3 = np.repeat(p["v"], 3, axis=1)
    mha = impl(p["q"], k3, v3, p["tables"], p["lens"], p["scale"])
    assert np.array_equal(out, mha)


def pin_garbage_isolation(impl):
    """NaN beyond the context in the last block, in unused blocks and -1 in unused table slots."""
    p = random_problem(71, lens=[5, 9, 4], hq=4, hkv=2, d=8, bs=4)
    out = call(impl, p)
    k2, v2 = p["k"].copy(), p["v"].copy()
    used = np.zeros(k2.shape[0], dtype=bool)
    for n, L in enumerate(p["lens"]):
        nb = (L + 3) // 4
        used[p["tables"][n, :nb]] = True
        if L % 4:
            b = p["tables"][n, nb - 1]
            k2[b, :, L % 4:, :] = np.nan
            v2[b, :, L % 4:, :] = np.nan
    k2[~used] = np.nan
    v2[~used] = np.nan
    out2 = impl(p["q"], k2, v2, p["tables"], p["lens"], p["scale"])
    assert np.array_equal(out, out2)


def pin_rows_are_independent(impl):
    """A sequence's output does not depend on what else is in the batch."""
    p = random_problem(81, nseq=3, hq=2, hkv=1, d=8, bs=4, max_ctx=15)
    out = call(impl, p)
    for n in range(3):
        one = impl(p["q"][n:n + 1], p["k"], p["v"], p["tables"][n:n + 1], p["lens"][n:n + 1],
                   p["scale"])
        assert np.array_equal(one[0], out[n])


ALL_PINS = [pin_golden_closed_forms, pin_dense_bruteforce, pin_library_attention_fp64,
            pin_context_one_is_v, pin_context_zero_is_zero, pin_placement_invariance,
            pin_token_order_permutation, pin_equal_keys_give_mean_of_v,
            pin_zero_query_gives_mean_of_v, pin_dominant_key_selects_its_v, pin_large_scores_are_stable,
            pin_constant_v_is_returned, pin_softmax_shift_invariance, pin_scale_is_applied,
            pin_split_merge_algebra, pin_gqa_equals_replicated_mha, pin_garbage_isolation,
            pin_rows_are_independent]
