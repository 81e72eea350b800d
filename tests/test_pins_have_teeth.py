"""The pins must catch plausible mistakes.

A small numpy implementation with switchable, deliberately planted bugs is run
through the same pins the oracle has to pass.  With no bug it passes all of
them (so a failure is due to the bug, not to the harness); with any one bug at
least one pin must fail.  All of this is on the CPU.
"""
import numpy as np
import pytest

import pins

BUGS = ["no_scale", "head_mod_instead_of_div", "slot_and_head_swapped", "drop_last_token",
        "read_whole_last_block", "v_read_from_k", "table_indexed_by_token", "not_normalised",
        "no_max_subtraction_overflow", "sum_of_abs_weights", "context_zero_nan",
        "wrong_block_for_v", "kv_head_zero_only", "scale_inside_exp_only_half", "mean_ignores_q"]


def make_impl(bug=None):
    def impl(q, k, v, tables, lens, scale):
        nseq, hq, d = q.shape
        nb, hkv, bs, _ = k.shape
        G = hq // hkv
        out = np.zeros((nseq, hq, d))
        for n in range(nseq):
            L = int(lens[n])
            if L == 0:
                if bug == "context_zero_nan":
                    out[n] = np.nan
                continue
            Lk = L - 1 if (bug == "drop_last_token" and L > 1) else L
            if bug == "read_whole_last_block":
                Lk = ((L + bs - 1) // bs) * bs
            for h in range(hq):
                g = h // G
                if bug == "head_mod_instead_of_div":
                    g = h % hkv
                if bug == "kv_head_zero_only":
                    g = 0
                s = np.empty(Lk)
                vs = np.empty((Lk, d))
                for t in range(Lk):
                    blk = tables[n, t // bs]
                    if bug == "table_indexed_by_token":
                        blk = tables[n, min(t, tables.shape[1] - 1)]
                    slot = t % bs
                    if bug == "slot_and_head_swapped":
                        flat_k = k.reshape(nb, -1, d)
                        flat_v = v.reshape(nb, -1, d)
                        kv = flat_k[blk, slot * hkv + g] if slot * hkv + g < flat_k.shape[1] else flat_k[blk, 0]
                        vv = flat_v[blk, slot * hkv + g] if slot * hkv + g < flat_v.shape[1] else flat_v[blk, 0]
                    else:
                        kv = k[blk, g, slot]
                        vv = v[blk, g, slot]
                    if bug == "v_read_from_k":
                        vv = kv
                    if bug == "wrong_block_for_v":
                        vv = v[tables[n, 0], g, slot]
                    s[t] = np.dot(q[n, h], kv) * (1.0 if bug == "no_scale" else scale)
                    if bug == "scale_inside_exp_only_half":
                        s[t] *= 0.5
                    if bug == "mean_ignores_q":
                        s[t] = 0.0
                    vs[t] = vv
                if bug == "no_max_subtraction_overflow":
                    with np.errstate(over="ignore", invalid="ignore"):
                        p = np.exp(s)
                else:
                    p = np.exp(s - s.max())
                if bug == "sum_of_abs_weights":
                    Z = np.abs(p).sum() + 1e-3
                else:
                    Z = p.sum()
                acc = (p[:, None] * vs).sum(axis=0)
                with np.errstate(invalid="ignore"):
                    out[n, h] = acc if bug == "not_normalised" else acc / Z
        return out
    return impl


def failing_pins(impl):
    bad = []
    for pin in pins.ALL_PINS:
        try:
            pin(impl)
        except AssertionError:
            bad.append(pin.__name__)
        except Exception as e:  # an out-of-range index is also a detection
            bad.append(pin.__name__ + ":" + type(e).__name__)
    return bad


def test_clean_implementation_passes_every_pin():
    assert failing_pins(make_impl(None)) == []


@pytest.mark.parametrize("bug", BUGS)
def test_planted_bug_is_caught(bug):
    bad = failing_pins(make_impl(bug))
    assert bad, f"no pin notices the planted bug {bug!r}"
