"""The serving loop on the MI355X: every scheduling decision comes from kvcp_schedule_step (the
policy core in C++), the server (paper_2503_13773_amd.serving) turns the decisions into the device calls of the
C ABI - kv_cache_append, paged_attention_decode, paged_attention_prefill for admissions and
recomputation, kv_block_copy to and from pinned host memory for swapping - and every attention
output of every iteration is compared with the oracle's attention over the request's true token
sequence (independent of the server's block tables and of what its swaps and recomputations left
in the cache).  The scenario (tests/serving_scenario.py) contains a victim above the sweet spot
(swapped out and back in), victims below it (dropped and recomputed through the prefill kernel), a
request embedded in another's unused allocation, and the host's overrun into its guest."""
import pytest

import serving_scenario as S
from gpu_util import BF16_TOL

pytestmark = pytest.mark.gpu


def test_policy_core_drives_the_device_calls(oracle_mod):
    from paper_2503_13773_amd.serving import HipOps
    ops = HipOps(S.NUM_BLOCKS, S.SWAP_BLOCKS, S.HQ, S.HKV, S.D, S.BS)
    srv = S.make_server(ops)
    log = S.run(srv, oracle_mod, tol=BF16_TOL, verbose=True)
    st = srv.stats
    print("[serving]", st, flush=True)
    assert srv.all_done()
    assert st["swapped"] >= 1 and st["swap_ins"] == st["swapped"]          # above the sweet spot: swapped
    assert st["recomputed"] >= 1 and any("recompute" in e and "preempt" not in e for e in log)   # below: prefill again
    assert st["embedded"] >= 1 and st["overruns"] >= 1                     # embedding method and its failure mode
    assert srv.bm.free_general == S.NUM_BLOCKS - S.RESERVED and srv.bm.free_reserved == S.RESERVED
    assert sorted(srv.swap_free) == list(range(S.SWAP_BLOCKS))
