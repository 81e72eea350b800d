"""The serving loop's bookkeeping (paper_2503_13773_amd.serving) on the CPU: the policy library decides, the device
calls are replaced by the oracle's functions on host pools, and every attention output is compared
with attention over the request's true token sequence.  The GPU test runs the same scenario on the
HIP library."""
import numpy as np

import serving_scenario as S


def test_scenario_runs_to_completion_and_takes_every_branch(oracle_mod):
    ops = S.OracleOps(oracle_mod, S.NUM_BLOCKS, S.SWAP_BLOCKS)
    srv = S.make_server(ops)
    log = S.run(srv, oracle_mod, tol=1e-9)
    st = srv.stats
    print(st, *log, sep="\n")
    assert srv.all_done()
    assert st["swapped"] >= 1 and st["recomputed"] >= 1 and st["swap_ins"] == st["swapped"]
    assert st["embedded"] >= 1 and st["overruns"] >= 1
    # every block and swap slot came back
    assert srv.bm.free_general == S.NUM_BLOCKS - S.RESERVED and srv.bm.free_reserved == S.RESERVED
    assert sorted(srv.swap_free) == list(range(S.SWAP_BLOCKS))
