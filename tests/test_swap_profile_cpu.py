"""The two regressors of the preemption-strategy selection (paper Section 3.5), fitted by the
policy library: the least-squares line L_s = gamma * S + delta, the power law L_r = alpha * S^beta,
and the sweet spot where they meet.  Pins: data that lies exactly on a line / power law (closed
form), numpy.polyfit on noisy data (library routine), roots of the quadratic worked by hand."""
import math

import numpy as np
import pytest

from paper_2503_13773_amd import policy as P


def test_fit_recovers_an_exact_line():
    S = [100, 400, 1600, 6400]
    g, d, r2 = P.fit_linear(S, [0.02 * s + 3.0 for s in S])
    assert abs(g - 0.02) < 1e-12 and abs(d - 3.0) < 1e-9
    assert abs(r2 - 1.0) < 1e-12
    # two points: the line through them (slope 3/2, intercept -2)
    g, d, r2 = P.fit_linear([2.0, 4.0], [1.0, 4.0])
    assert (g, d) == (1.5, -2.0)


def test_fit_matches_numpy_polyfit_on_noisy_data():
    rng = np.random.default_rng(0)
    S = np.array([128, 256, 512, 1024, 2048, 4096, 8192], dtype=float)
    L = 0.0123 * S + 0.4 + rng.normal(0, 0.05, S.size)
    g, d, r2 = P.fit_linear(S.tolist(), L.tolist())
    pg, pd = np.polyfit(S, L, 1)
    assert abs(g - pg) < 1e-10 and abs(d - pd) < 1e-8
    want_r2 = 1.0 - ((L - (pg * S + pd)) ** 2).sum() / ((L - L.mean()) ** 2).sum()
    assert 0.99 < r2 <= 1.0 and abs(r2 - want_r2) < 1e-10


def test_fit_rejects_degenerate_input():
    for x, y in [([5], [1.0]), ([5, 5, 5], [1.0, 2.0, 3.0]), ([1.0, float("nan")], [1.0, 2.0]), ([1, 2], [1.0])]:
        with pytest.raises(ValueError):
            P.fit_linear(x, y)


def test_sweet_spot_closed_forms():
    # quadratic recompute a*S^2 against the line g*S + d: positive root of a S^2 - g S - d = 0
    a, g, d = 1e-6, 0.002, 1.0
    want = (g + math.sqrt(g * g + 4 * a * d)) / (2 * a)
    assert abs(P.sweet_spot(g, d, a, 2.0) - want) / want < 1e-9
    # linear recompute k*S against g*S + d with k > g: S = d / (k - g)
    assert abs(P.sweet_spot(0.01, 5.0, 0.0, 1.0, kappa_r=0.03) - 250.0) < 1e-6
    # all four recompute terms: 2e-6 S^2 + 0.001 S + 0.5 = 0.005 S + 8.5  ->  S^2 - 2000 S - 4e6 = 0
    # -> S = 1000 + sqrt(1e6 + 4e6) = 1000 (1 + sqrt 5)
    assert P.sweet_spot(0.005, 8.5, 2e-6, 2.0, kappa_r=0.001, eps_r=0.5) == pytest.approx(1000 * (1 + math.sqrt(5)), rel=1e-9)
    assert P.sweet_spot(0.01, 0.0, 1.0, 2.0, eps_r=1.0) == 0.0            # swapping always cheaper
    assert P.sweet_spot(1.0, 10.0, 1e-12, 1.0) == math.inf                 # recomputation always cheaper


def test_power_law_fit_and_flop_count():
    from paper_2503_13773_amd.recompute_profile import causal_attention_flops
    S = [256, 512, 1024, 2048, 4096]
    a, b, r2 = P.fit_power_law(S, [3e-6 * s ** 1.8 for s in S])
    assert abs(b - 1.8) < 1e-12 and abs(a - 3e-6) / 3e-6 < 1e-9 and abs(r2 - 1.0) < 1e-12
    pb, pa = np.polyfit(np.log(S), np.log([2.0 * s ** 2 + 5 * s for s in S]), 1)
    a, b, _ = P.fit_power_law(S, [2.0 * s ** 2 + 5 * s for s in S])
    assert abs(b - pb) < 1e-10 and abs(math.log(a) - pa) < 1e-9
    # one head, D = 1, S = 3: rows see 1, 2, 3 tokens -> 6 (q.k) + 6 (p.v) multiply-adds = 24 flops
    assert causal_attention_flops(3, 1, 1) == 24.0
    for x, y in [([4, 4], [1.0, 2.0]), ([1, 2], [0.0, 1.0]), ([-1, 2], [1.0, 1.0])]:
        with pytest.raises(ValueError):
            P.fit_power_law(x, y)
