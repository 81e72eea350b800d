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
    assert len(declared) >= 22 and {'kvcp_schedule_step', 'kvcp_fit_linear', 'kvcp_fit_power_law'} <= declared
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
    # all four recompute terms, worked by hand: 2e-6 S^2 + 0.001 S + 0.5 = 0.005 S + 8.5 has the
    # positive root S = 1000 (1 + sqrt 5)
    assert P.sweet_spot(0.005, 8.5, 2e-6, 2.0, 0.001, 0.5) == pytest.approx(1000 * (1 + math.sqrt(5)), rel=1e-9)


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


# ---------------------------------------------------------------------------
# one scheduler step (Sections 3.3.2, 3.3.3, 3.4, 3.5): every expectation below is worked by hand
# ---------------------------------------------------------------------------
def R(state, sp, so, gen=0, alloc=0, used=0, rt=1.0, slo=0.1):
    return P.Request(state=state, reserved=0, prompt_len=sp, est_output_len=so, generated=gen,
                     allocated=alloc, used=used, remaining_time=rt, tbt_slo=slo)


STEP = dict(block_tokens=8, buffer_tokens=8, m=2, max_iteration_latency=0.05, eps=0.01)


def row(d):
    return (d.in_batch, d.critical, d.preempt, d.proactive, d.grant, d.host, d.s0, d.lender, d.shortfall)


def test_step_critical_sets_basic_demand_embedding_and_the_case_with_room_left():
    reqs = [R(P.RUNNING, 100, 50, gen=20, alloc=160, used=120, rt=0.5),    # 0 has 40 tokens of unused allocation
            R(P.RUNNING, 40, 30, gen=24, alloc=64, used=64, rt=0.055),     # 1 used up its KVC, RT - T < eps: N_r
            R(P.WAITING, 24, 16, rt=0.05),                                 # 2 critical waiting: N_w
            R(P.WAITING, 16, 8, rt=2.0),                                   # 3 fits inside request 0
            R(P.WAITING, 200, 100, rt=3.0)]                                # 4 too long for the token budget
    dec, s = P.schedule_step(reqs, unallocated=200, token_budget=50, **STEP)
    # request 2 cannot be embedded in 0: 160 - (120+16) - (24+16) = -16 < 8.  D = (24+8) + 8 = 40 <= 200: no
    # preemption; basic grants 32 and 8.  Batch so far: two running (1 token each) + 24 prompt tokens = 26.
    # Request 3 (prompt 16 -> 42 <= 50) is embedded in 0: 160 - (120+8) - (16+8) = 8 >= 8, s0 = 160-128-8 = 24
    # (its space begins 160 - 24 = 136 tokens into request 0's allocation).
    # Request 4 (42 + 200 > 50) stays out.  Demands: request 2: 40 - 32 = 8; request 1: 70 - 64 - 8 < 0 -> 0;
    # request 3: 0.  Sum 8 < 160: the case with room left; request 4's 300 does not fit either, so nothing is
    # added and everybody gets its demand.
    assert row(dec[0]) == (1, 0, P.KEEP, 0, 0, -1, 0, -1, 0)
    assert row(dec[1]) == (1, 1, P.KEEP, 0, 8, -1, 0, -1, 0)
    assert row(dec[2]) == (1, 1, P.KEEP, 0, 40, -1, 0, -1, 0)
    assert row(dec[3]) == (1, 0, P.KEEP, 0, 0, 0, 24, -1, 0)
    assert row(dec[4]) == (0, 0, P.KEEP, 0, 0, -1, 0, -1, 0)
    assert (s.unallocated_after, s.basic_demand, s.excess, s.batch_tokens, s.n_preempted, s.alloc_case) == \
        (152, 40, 0, 42, 0, P.CASE_LESS)


@pytest.mark.parametrize("sweet,strategy", [(100.0, P.PREEMPT_RECOMPUTE), (40.0, P.PREEMPT_SWAP)])
def test_step_preempts_in_policy_order_until_the_basic_demand_fits(sweet, strategy):
    reqs = [R(P.RUNNING, 50, 400, gen=10, alloc=100, used=60, slo=0.1),    # 0 tight TBT SLO: last to be preempted
            R(P.RUNNING, 300, 300, gen=50, alloc=400, used=350, slo=1.0),  # 1 loose SLO, 250 tokens left (bucket 1)
            R(P.RUNNING, 30, 300, gen=20, alloc=64, used=50, slo=1.0),     # 2 loose SLO, 280 tokens left (bucket 2)
            R(P.WAITING, 60, 20, rt=0.05)]                                 # 3 critical: needs 60 + 8 = 68
    dec, s = P.schedule_step(reqs, unallocated=10, token_budget=1000, sweet_spot=sweet, **STEP)
    # No host has room for request 3.  D = 68 > 10: victims in the order loosest SLO, then longest remaining
    # time: request 2 first.  Its 64 tokens make 74 >= 68, so request 1 is spared.  Request 2 occupies 50
    # tokens: recomputed when the sweet spot is 100, swapped when it is 40.
    # Request 3 gets 68 (6 left), still misses 80 - 68 = 12 > 6: amortised alone it takes the 6, shortfall 6.
    # It would run 74 - 60 = 14 iterations on what it holds; requests 0 and 1 finish far later: no lender.
    assert row(dec[2]) == (0, 0, strategy, 0, 0, -1, 0, -1, 0)
    assert row(dec[1]) == (1, 0, P.KEEP, 0, 0, -1, 0, -1, 0) and row(dec[0]) == (1, 0, P.KEEP, 0, 0, -1, 0, -1, 0)
    assert row(dec[3]) == (1, 1, P.KEEP, 0, 74, -1, 0, -1, 6)
    assert (s.unallocated_after, s.basic_demand, s.excess, s.batch_tokens, s.n_preempted, s.alloc_case) == \
        (0, 68, 6, 62, 1, P.CASE_MORE)


def test_step_amortises_adds_the_proactive_request_and_finds_a_lender():
    reqs = [R(P.RUNNING, 20, 10, gen=8, alloc=29, used=28, rt=2.0),    # 0 unfulfilled (29 < 30), 2 iterations left: proactive
            R(P.RUNNING, 50, 30, gen=27, alloc=80, used=77, rt=2.0),   # 1 fulfilled, finishes in 3 iterations
            R(P.WAITING, 40, 60, rt=2.0),                              # 2
            R(P.WAITING, 10, 90, rt=6.0)]                              # 3
    dec, s = P.schedule_step(reqs, unallocated=96, token_budget=1000, **STEP)
    # Nobody is critical.  Demands: request 0: 30 - 29 = 1; requests 2 and 3: 100 each; 201 > 96.
    # Weights RT/sum RT * sp/sum sp with sum RT = 10, sum sp = 70: 2/9, 4/9, 3/9 of 96 -> 21 (capped at 1), 42, 32.
    # Request 2 cannot hold its prompt plus a granule (42 < 48): it is left out and the round repeats with
    # requests 0 and 3: sum RT = 8, sum sp = 30, shares 0.4 and 0.6 of 96 -> 38 (capped at 1) and 57.
    # E_kvc = 101 - 96 = 5.  Request 3 misses 43; it runs 57 - 10 = 47 iterations on its 57 tokens.  Request 1
    # finishes in 3 <= 47 iterations and holds 80 >= 43: the lender.  Request 0 holds only 30.
    assert row(dec[0]) == (1, 0, P.KEEP, 1, 1, -1, 0, -1, 0)
    assert row(dec[1]) == (1, 0, P.KEEP, 0, 0, -1, 0, -1, 0)
    assert row(dec[2]) == (0, 0, P.KEEP, 0, 0, -1, 0, -1, 0)
    assert row(dec[3]) == (1, 0, P.KEEP, 0, 57, -1, 0, 1, 43)
    assert (s.unallocated_after, s.basic_demand, s.excess, s.batch_tokens, s.n_preempted, s.alloc_case) == \
        (38, 0, 5, 12, 0, P.CASE_MORE)


def test_step_adds_waiting_requests_while_kvc_and_slos_allow():
    reqs = [R(P.RUNNING, 10, 10, gen=2, alloc=20, used=12, rt=0.5),
            R(P.WAITING, 30, 10, rt=1.0), R(P.WAITING, 40, 10, rt=2.0), R(P.WAITING, 50, 10, rt=3.0),
            R(P.WAITING, 20, 10, rt=4.0)]
    kw = dict(STEP, iter_time_base=0.1, iter_time_per_token=0.004)
    # token budget 35: the running request (1) + request 1 (30) = 31; request 2 would make 71.  Demand 40 < 200:
    # requests are added in RT order while M_i fits and the modelled iteration stays below every RT in the
    # batch: request 2 -> 71 tokens, 0.1 + 0.284 = 0.384 <= 0.5 fine, sum 90; request 3 -> 121 tokens, 0.584 > 0.5:
    # stop (request 4 is not looked at: the queue is taken in order).
    dec, s = P.schedule_step(reqs, unallocated=200, token_budget=35, **kw)
    assert [d.in_batch for d in dec] == [1, 1, 1, 0, 0] and [d.grant for d in dec] == [0, 40, 50, 0, 0]
    assert (s.unallocated_after, s.batch_tokens, s.alloc_case) == (110, 71, P.CASE_LESS)
    # with 85 tokens of KVC request 2 no longer fits after request 1 (40 + 50 > 85) and stays out
    dec, s = P.schedule_step(reqs, unallocated=85, token_budget=35, **kw)
    assert [d.in_batch for d in dec] == [1, 1, 0, 0, 0] and s.unallocated_after == 45
    # exactly enough: the case sum M = A'
    dec, s = P.schedule_step(reqs, unallocated=40, token_budget=35, **kw)
    assert s.alloc_case == P.CASE_EQUAL and dec[1].grant == 40 and s.unallocated_after == 0


def test_step_returned_request_beyond_its_estimate_asks_for_one_granule():
    # used up its allocation, not time-critical (N'_r), already 4 tokens past sp + so: demand B
    reqs = [R(P.RUNNING, 10, 5, gen=9, alloc=19, used=19, rt=1.0)]
    dec, s = P.schedule_step(reqs, unallocated=100, token_budget=10, **STEP)
    assert row(dec[0]) == (1, 0, P.KEEP, 0, 8, -1, 0, -1, 0) and s.unallocated_after == 92
    # the same request when time-critical gets its granule in the critical phase: D = B
    reqs[0].remaining_time = 0.055
    dec, s = P.schedule_step(reqs, unallocated=100, token_budget=10, **STEP)
    assert row(dec[0]) == (1, 1, P.KEEP, 0, 8, -1, 0, -1, 0) and s.basic_demand == 8


def test_step_hosts_take_one_guest_and_are_not_preempted():
    reqs = [R(P.RUNNING, 10, 300, gen=10, alloc=320, used=20, slo=1.0),    # 0: roomy, loosest SLO
            R(P.WAITING, 20, 10, rt=0.05), R(P.WAITING, 20, 10, rt=0.05)]  # two critical requests
    dec, s = P.schedule_step(reqs, unallocated=0, token_budget=100, **STEP)
    # the first critical request (same basic requirement: index order) is embedded: s0 = 320 - (20+10) - 8 = 282
    # (it starts 38 tokens in, 8 past where request 0 will stand after 10 more iterations);
    # the second finds the host taken, needs 28 from an empty pool, and the only running request is a host:
    # nobody can be preempted, it waits
    assert row(dec[1]) == (1, 1, P.KEEP, 0, 0, 0, 282, -1, 0)
    assert row(dec[2]) == (0, 1, P.KEEP, 0, 0, -1, 0, -1, 0)
    assert dec[0].preempt == P.KEEP and s.n_preempted == 0 and s.basic_demand == 28


def test_step_rejects_bad_arguments_and_accepts_an_empty_queue():
    dec, s = P.schedule_step([], unallocated=5, **STEP)
    assert dec == [] and s.unallocated_after == 5
    for bad in [R(P.WAITING, 0, 5), R(P.WAITING, 5, 0), R(P.WAITING, 5, 5, alloc=8), R(P.RUNNING, 5, 5, alloc=4, used=6),
                R(P.RUNNING, 5, 5, rt=0.0), R(7, 5, 5)]:
        with pytest.raises(ValueError):
            P.schedule_step([bad], unallocated=10, **STEP)
    with pytest.raises(ValueError):
        P.schedule_step([R(P.WAITING, 5, 5)], unallocated=-1, **STEP)


def test_embedding_block_range_rounds_to_whole_blocks():
    # host: 160 tokens allocated, 120 used; guest 16 + 8: s0 = 160 - (120+8) - 8 = 24 tokens of room, so the
    # guest's space begins 160 - 24 = 136 tokens in (= u_j + so_i + b); 16-token blocks: block ceil(136/16) = 9,
    # spanning ceil(24/16) = 2 blocks; the host has 10 blocks: 9 + 2 > 10 does not fit once rounded
    assert P.embedding_block_range(160, 24, 16, 8, 16, 10) is None
    assert P.embedding_block_range(160, 40, 16, 8, 16, 10) == (8, 2)     # begins at token 120 = block 7.5 -> 8
    assert P.embedding_block_range(160, 48, 16, 8, 16, 10) == (7, 2)     # begins at token 112 = block 7
    assert P.embedding_block_range(64, 32, 1, 0, 16, 4) == (2, 1)
    assert P.embedding_block_range(64, 65, 1, 0, 16, 4) is None           # s0 cannot exceed the allocation
