"""The host-side policy core against the paper's closed forms (Sections 3.2-3.5).

Expected values are worked out by hand from the printed equations, not produced by the code.
"""
import math
import os
import re
import subprocess

import pytest

from paper_2503_13773_amd import policy as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def built():
    if not os.path.exists(P.library_path()):
        from paper_2503_13773_amd.build import build_policy_library
        build_policy_library()


def test_policy_library_exports_every_declared_symbol():
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "kvc_policy.h")).read(), flags=re.S)
    declared = set(re.findall(r"KVCP_API\s+[\w\s\*]+?\b(kvcp_\w+)\s*\(", text))
    assert len(declared) == 18
    out = subprocess.run(["nm", "-D", "--defined-only", P.library_path()], capture_output=True, text=True).stdout
    assert declared <= set(re.findall(r"\bT\s+(kvcp_\w+)", out))
    subprocess.check_call(["gcc", "-std=c99", "-fsyntax-only", "-x", "c", os.path.join(ROOT, "include", "kvc_policy.h")])


def test_confidence_follows_equation_4():
    # c = alpha / (1 + beta * lambda)
    assert P.confidence(0.9, 0.05, 20.0) == pytest.approx(0.45, abs=1e-15)      # 0.9 / 2
    assert P.confidence(0.9, 0.05, 0.0) == 0.9                                  # lambda -> 0 gives alpha
    assert P.confidence(1.0, 1.0, 3.0) == 0.25
    assert P.confidence(0.9, 0.05, 40.0) < P.confidence(0.9, 0.05, 20.0)        # decreases with arrival rate
    for bad in [(0.0, 1.0, 1.0), (1.5, 1.0, 1.0), (0.5, 0.0, 1.0), (0.5, 1.0, -1.0)]:
        assert math.isnan(P.confidence(*bad))


def test_padding_follows_equation_3():
    # t = sqrt(-(range^2 / 2) ln(1 - c)); range 100, c = 1 - e^-2  =>  t = sqrt(5000 * 2) = 100
    assert P.padding(100.0, 1.0 - math.exp(-2.0)) == pytest.approx(100.0, rel=1e-12)
    # range 64, c = 1 - e^-8  =>  t = sqrt(2048 * 8) = 128
    assert P.padding(64.0, 1.0 - math.exp(-8.0)) == pytest.approx(128.0, rel=1e-9)
    # c = 0.9, range 100: t = sqrt(5000 ln 10) = 107.2983...
    assert P.padding(100.0, 0.9) == pytest.approx(math.sqrt(5000.0 * math.log(10.0)), rel=1e-14)
    assert 107.29 < P.padding(100.0, 0.9) < 107.31
    assert P.padding(100.0, 0.0) == 0.0                                         # no confidence asked, no padding
    assert P.padding(100.0, 0.99) > P.padding(100.0, 0.9)                       # higher confidence, more padding
    assert P.padding(200.0, 0.9) == pytest.approx(2 * P.padding(100.0, 0.9))    # linear in the range
    # the bound it comes from: exp(-2 t^2 / range^2) = 1 - c
    t = P.padding(300.0, 0.8)
    assert math.exp(-2 * t * t / 300.0 ** 2) == pytest.approx(0.2, rel=1e-12)
    assert math.isnan(P.padding(100.0, 1.0)) and math.isnan(P.padding(-1.0, 0.5))


def test_padding_is_added_or_subtracted_by_deviation_direction():
    t = P.padding(100.0, 0.9)
    assert P.estimated_output_len(300.0, 100.0, 0.9, True) == pytest.approx(300.0 + t)
    assert P.estimated_output_len(300.0, 100.0, 0.9, False) == pytest.approx(300.0 - t)
    assert P.estimated_output_len(50.0, 100.0, 0.9, False) == 1.0               # never below one token


def test_embedding_condition_and_start_offset():
    # a_j - (u_j + so_i) - (sp_i + so_i) >= b ; s0 = a_j - (u_j + so_i) - b
    # a=1000, u=200, sp=100, so=150, b=8: 1000 - 350 - 250 = 400 >= 8 -> s0 = 1000 - 350 - 8 = 642
    assert P.embedding_fits(1000, 200, 100, 150, 8) == 642
    # the request occupies [s0, s0 + sp + so) = [642, 892) which ends b+... inside the allocation
    assert 642 + 100 + 150 <= 1000
    # exactly at the boundary: 1000 - (200+150) - (sp+150) = 8  <=> sp = 492
    assert P.embedding_fits(1000, 200, 492, 150, 8) is not None
    assert P.embedding_fits(1000, 200, 493, 150, 8) is None
    assert P.embedding_fits(100, 200, 1, 1, 8) is None                          # used > allocated is rejected


def test_embedding_chooses_the_host_with_minimum_remaining_allocation():
    a = [2000, 900, 1500, 700]
    u = [100, 100, 900, 650]
    # remaining: 1900, 800, 600, 50; request sp=100, so=100, b=8 needs a-u >= 308 -> hosts 0, 1, 2 fit
    j, s0 = P.embedding_choose(a, u, 100, 100, 8)
    assert j == 2 and s0 == 1500 - (900 + 100) - 8
    assert P.embedding_choose(a, u, 5000, 100, 8) is None
    assert P.embedding_choose([], [], 1, 1, 8) is None


def test_critical_requests_and_basic_demand():
    assert P.is_critical(0.30, 0.25, 0.1) and not P.is_critical(0.50, 0.25, 0.1)
    # D = sum (sp_i + B) + |N_r| B : prompts 100, 250, 3 returned, B = 8 -> 108 + 258 + 24 = 390
    assert P.basic_demand([100, 250], 3, 8) == 390
    assert P.basic_demand([], 0, 8) == 0


def test_allocation_three_cases():
    M, RT, sp = [300, 500, 200], [1.0, 2.0, 1.0], [100, 100, 200]
    assert P.allocate(M, RT, sp, 1000) == ([300, 500, 200], 0)                  # demand == supply
    assert P.allocate(M, RT, sp, 1300) == ([300, 500, 200], 300)                # room for more requests
    # excess: A' = 400. w_i = RT_i/sum RT * sp_i/sum sp = (1/4*1/4, 2/4*1/4, 1/4*2/4) = (1, 2, 2)/16
    # A_i = 400 * w_i / sum w = 400 * (1, 2, 2) / 5 = (80, 160, 160)
    alloc, slack = P.allocate(M, RT, sp, 400)
    assert alloc == [80, 160, 160] and slack == -600
    assert sum(alloc) <= 400
    # embedded requests (M_i = 0) take no share and do not dilute the weights
    alloc, _ = P.allocate([300, 0, 200], [1.0, 9.0, 1.0], [100, 999, 100], 100)
    assert alloc == [50, 0, 50]
    # a share is capped at the demand
    alloc, _ = P.allocate([10, 1000], [1.0, 1.0], [500, 500], 500)
    assert alloc == [10, 250]
    with pytest.raises(ValueError):
        P.allocate([300, 500], [1.0, 0.0], [100, 100], 100)


def test_preemption_order_buckets():
    #            0      1      2      3      4      5
    slo = [0.10, 1.00, 0.60, 0.30, 1.50, 0.55]      # buckets (edges 0.2, 0.5): 0, 2, 2, 1, 2, 2
    rem = [900, 100, 300, 50, 120, 260]             # 128-token buckets:        7, 0, 2, 0, 0, 2
    occ = [10, 500, 400, 20, 300, 100]
    # loosest SLO bucket first (1, 2, 4, 5); among them remaining bucket 2 (requests 2, 5) before bucket 0
    # (1, 4); inside a remaining bucket the smaller KVC occupancy first: 5 (100) before 2 (400); 4 (300) before 1 (500)
    assert P.preemption_order(slo, rem, occ) == [5, 2, 4, 1, 3, 0]
    assert P.preemption_order([], [], []) == []
    with pytest.raises(ValueError):
        P.preemption_order(slo, rem, occ, slo_edges=(0.5, 0.2))


def test_strategy_selection_and_sweet_spot():
    # quadratic recompute a S^2 against the swap line g S + d: positive root of a S^2 - g S - d
    a, g, d = 1e-6, 0.002, 1.0
    want = (g + math.sqrt(g * g + 4 * a * d)) / (2 * a)
    ss = P.sweet_spot(g, d, a, 2.0)
    assert ss == pytest.approx(want, rel=1e-9)
    assert P.choose_swap(want * 1.01, ss) and not P.choose_swap(want * 0.99, ss)
    assert P.sweet_spot(0.01, 0.0, 1.0, 2.0, eps_r=1.0) == 0.0
    assert P.sweet_spot(1.0, 10.0, 1e-12, 1.0) == math.inf
    # agrees with the Python solver used by the swap profiler
    from paper_2503_13773_amd.swap_profile import sweet_spot as py_ss
    assert P.sweet_spot(0.0047, 0.145, 3e-7, 2.0, 0.002, 0.5) == pytest.approx(py_ss(0.0047, 0.145, 3e-7, 2.0, 0.002, 0.5), rel=1e-9)


def test_block_manager_with_reserved_pool():
    bm = P.BlockManager(16, reserved_blocks=4)
    assert (bm.free_general, bm.free_reserved) == (12, 4)
    a = bm.allocate(5)
    assert a == [0, 1, 2, 3, 4]
    assert bm.allocate(8) is None and bm.free_general == 7                     # all-or-nothing
    b = bm.allocate(7)
    assert b == [5, 6, 7, 8, 9, 10, 11] and bm.free_general == 0
    assert bm.allocate(1) is None                                              # allocation failure ...
    r = bm.allocate_reserved(2)                                                # ... served by the reserved pool
    assert r == [12, 13] and bm.free_reserved == 2
    bm.release([3, 12, 0])
    assert (bm.free_general, bm.free_reserved) == (2, 3)
    assert bm.allocate(2) == [0, 3]                                            # lowest ids first; reserved ids never leak
    with pytest.raises(ValueError):
        bm.release([1, 1])
    with pytest.raises(ValueError):
        bm.release([12])                                                       # already free
    with pytest.raises(ValueError):
        bm.release([99])
    with pytest.raises(ValueError):
        P.BlockManager(4, 5)


# ---------------------------------------------------------------------------
# seeded random sweeps against properties and small Python models of the same definitions
# ---------------------------------------------------------------------------
def test_allocation_properties_on_random_inputs():
    import random
    rnd = random.Random(11)
    for _ in range(300):
        n = rnd.randint(1, 12)
        M = [rnd.choice([0, rnd.randint(1, 4000)]) for _ in range(n)]
        RT = [rnd.uniform(0.01, 5.0) for _ in range(n)]
        sp = [rnd.randint(1, 3000) for _ in range(n)]
        A = rnd.randint(0, 12000)
        alloc, slack = P.allocate(M, RT, sp, A)
        assert all(0 <= a <= m for a, m in zip(alloc, M))            # never above the demand, nothing for M = 0
        assert sum(alloc) <= A
        if sum(M) <= A:
            assert alloc == M and slack == A - sum(M)
        else:
            assert slack == -(sum(M) - A)
            # the printed weights: share before the cap = floor(A w_i / sum w) over requests with a demand
            live = [i for i in range(n) if M[i] > 0]
            srt, ssp = sum(RT[i] for i in live), sum(sp[i] for i in live)
            w = {i: RT[i] / srt * sp[i] / ssp for i in live}
            sw = sum(w.values())
            for i in live:
                share = A * w[i] / sw
                assert alloc[i] in (min(M[i], math.floor(share)), min(M[i], math.floor(share + 1e-9)),
                                    min(M[i], math.floor(share - 1e-9)))


def test_preemption_order_matches_a_sort_by_the_three_keys():
    import bisect
    import random
    rnd = random.Random(12)
    edges, width = (0.2, 0.5, 1.0), 64
    for _ in range(200):
        n = rnd.randint(0, 40)
        slo = [rnd.choice([0.05, 0.2, 0.3, 0.5, 0.7, 1.0, 2.0]) for _ in range(n)]
        rem = [rnd.randint(0, 600) for _ in range(n)]
        occ = [rnd.randint(0, 50) for _ in range(n)]
        want = sorted(range(n), key=lambda i: (-bisect.bisect_right(edges, slo[i]), -(rem[i] // width), occ[i], i))
        assert P.preemption_order(slo, rem, occ, slo_edges=edges, token_bucket=width) == want


def test_embedding_choice_matches_brute_force():
    import random
    rnd = random.Random(13)
    for _ in range(300):
        n = rnd.randint(0, 10)
        a = [rnd.randint(0, 4000) for _ in range(n)]
        u = [rnd.randint(0, x) for x in a]
        sp_i, so_i, b = rnd.randint(1, 800), rnd.randint(1, 800), rnd.randint(0, 64)
        fits = [j for j in range(n) if a[j] - (u[j] + so_i) - (sp_i + so_i) >= b]
        got = P.embedding_choose(a, u, sp_i, so_i, b)
        if not fits:
            assert got is None
        else:
            best = min(fits, key=lambda j: (a[j] - u[j], j))
            assert got == (best, a[best] - (u[best] + so_i) - b)


def test_block_manager_against_a_set_model():
    import random
    rnd = random.Random(14)
    for trial in range(20):
        nb, res = rnd.randint(1, 60), 0
        res = rnd.randint(0, nb)
        bm = P.BlockManager(nb, res)
        free_g, free_r, held = set(range(nb - res)), set(range(nb - res, nb)), []
        for _ in range(200):
            op = rnd.random()
            if op < 0.45:
                n = rnd.randint(0, 8)
                got = bm.allocate(n)
                if n <= len(free_g):
                    want = sorted(free_g)[:n]
                    assert got == want
                    free_g -= set(want)
                    held += want
                else:
                    assert got is None
            elif op < 0.6:
                n = rnd.randint(0, 4)
                got = bm.allocate_reserved(n)
                if n <= len(free_r):
                    want = sorted(free_r)[:n]
                    assert got == want
                    free_r -= set(want)
                    held += want
                else:
                    assert got is None
            elif held:
                k = rnd.randint(1, min(5, len(held)))
                ids = rnd.sample(held, k)
                bm.release(ids)
                for i in ids:
                    held.remove(i)
                    (free_r if i >= nb - res else free_g).add(i)
            assert (bm.free_general, bm.free_reserved) == (len(free_g), len(free_r))


def test_padding_and_sweet_spot_properties():
    import random
    rnd = random.Random(15)
    for _ in range(200):
        rng_, c1, c2 = rnd.uniform(1, 500), rnd.uniform(0.0, 0.98), rnd.uniform(0.0, 0.98)
        lo, hi = min(c1, c2), max(c1, c2)
        assert P.padding(rng_, lo) <= P.padding(rng_, hi) + 1e-12          # more confidence, more padding
        assert P.padding(2 * rng_, hi) == pytest.approx(2 * P.padding(rng_, hi), rel=1e-12)   # linear in the range
        # the padding inverts the tail bound it comes from: exp(-2 t^2 / range^2) = 1 - c
        t = P.padding(rng_, hi)
        assert math.exp(-2 * t * t / (rng_ * rng_)) == pytest.approx(1 - hi, rel=1e-9)
    for _ in range(100):
        g, d = rnd.uniform(1e-4, 1e-2), rnd.uniform(0.0, 2.0)
        a, b = rnd.uniform(1e-8, 1e-5), rnd.uniform(1.2, 2.2)
        ss = P.sweet_spot(g, d, a, b, s_max=1e7)
        if 0 < ss < math.inf:
            assert a * ss ** b == pytest.approx(g * ss + d, rel=1e-6)      # the two regressors meet there
            assert a * (2 * ss) ** b > g * (2 * ss) + d                     # recompute loses beyond it
