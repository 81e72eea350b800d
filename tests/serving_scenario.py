"""A small serving scenario for paper_2503_13773_amd.serving.KvcServer, shared by the CPU test (device
calls replaced by the oracle's functions on numpy pools) and the GPU test (the HIP library).

The model stand-in is a pair of seeded functions giving the K/V and the query of (request,
position); the reference for every output is attention over the request's TRUE token sequence laid
out densely, so it depends neither on the server's block tables nor on what its swaps and
recomputations left in the cache."""
import math

import numpy as np

import kvc_workloads as W
from paper_2503_13773_amd.serving import KvcServer, ServedRequest

HQ, HKV, D, BS = 8, 2, 128, 16
LMAX = 12
SCALE = 1.0 / math.sqrt(D)


def _bits(seed_tuple, shape):
    rng = np.random.default_rng(list(seed_tuple))
    return W.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))


def kv_fn(rid, pos):
    a = _bits((11, rid, pos), (2, HKV, D))
    return a[0], a[1]


def q_fn(rid, pos):
    return _bits((23, rid, pos), (HQ, D))


class OracleOps:
    """Device calls of the server carried out by the oracle on host pools (CPU runs of the loop)."""

    def __init__(self, oracle_mod, num_blocks, swap_blocks):
        self.o = oracle_mod
        self.pool = np.zeros((2, num_blocks, HKV, BS, D), dtype=np.uint16)
        self.swap = np.zeros((2, max(1, swap_blocks), HKV, BS, D), dtype=np.uint16)

    def append(self, k_new, v_new, tables, positions):
        self.o.kv_cache_append(np.ascontiguousarray(k_new), np.ascontiguousarray(v_new), self.pool[0], self.pool[1],
                               tables, positions)

    def decode(self, q, tables, lens):
        return self.o.paged_attention_decode(q, self.pool[0], self.pool[1], tables, lens, SCALE, dtype="bf16")

    def prefill(self, q, tables, lens, q_start):
        return self.o.paged_attention_prefill(q, self.pool[0], self.pool[1], tables, lens, q_start, SCALE, dtype="bf16")

    def copy_out(self, block_ids, slots):
        self.o.kv_block_copy(self.pool, self.swap, np.array(list(zip(block_ids, slots)), dtype=np.int64))

    def copy_in(self, slots, block_ids):
        self.o.kv_block_copy(self.swap, self.pool, np.array(list(zip(slots, block_ids)), dtype=np.int64))

    def poison(self, block_ids):
        if block_ids:
            self.pool[:, list(block_ids)] = np.uint16(0x7FC0)


def reference_decode(oracle_mod, rid, length):
    """Attention of the query at position length-1 over the request's first `length` tokens."""
    nb = (length + BS - 1) // BS
    k = np.zeros((nb, HKV, BS, D), dtype=np.uint16)
    v = np.zeros_like(k)
    for pos in range(length):
        kk, vv = kv_fn(rid, pos)
        k[pos // BS, :, pos % BS] = kk
        v[pos // BS, :, pos % BS] = vv
    table = np.arange(nb, dtype=np.int32)[None]
    return oracle_mod.paged_attention_decode(q_fn(rid, length - 1)[None], k, v, table,
                                             np.array([length], dtype=np.int32), SCALE, dtype="bf16")[0]


def reference_prefill(oracle_mod, rid, length):
    nb = (length + BS - 1) // BS
    k = np.zeros((nb, HKV, BS, D), dtype=np.uint16)
    v = np.zeros_like(k)
    for pos in range(length):
        kk, vv = kv_fn(rid, pos)
        k[pos // BS, :, pos % BS] = kk
        v[pos // BS, :, pos % BS] = vv
    q = np.stack([q_fn(rid, pos) for pos in range(length)])
    return oracle_mod.paged_attention_prefill(q, k, v, np.arange(nb, dtype=np.int32)[None],
                                              np.array([length], dtype=np.int32), np.array([0, length], dtype=np.int32),
                                              SCALE, dtype="bf16")


# (rid, arrival iteration, prompt, estimated output, true output, TTFT SLO, TBT SLO)
ARRIVALS = [
    (0, 0, 20, 150, 70, 1.0, 0.1),    # generously allocated (estimate far above the truth): the host
    (1, 1, 70, 40, 40, 1.0, 1.0),     # long, loose SLO: the victim above the sweet spot -> swapped
    (2, 1, 18, 30, 45, 1.0, 1.5),     # short, loosest SLO: the victim below the sweet spot -> recomputed
    (3, 2, 12, 6, 40, 1.0, 0.4),      # small estimate, long truth: embedded in 0, overrun later
    (4, 6, 130, 20, 20, 0.06, 0.3),   # tight TTFT and too long to embed: critical on arrival, forces preemptions
    (5, 30, 40, 20, 20, 0.06, 0.3),   # another critical arrival
]
NUM_BLOCKS, RESERVED, SWAP_BLOCKS = 22, 2, 16
SWEET_SPOT = 48.0                      # tokens: longer sequences are swapped, shorter recomputed


def make_server(ops):
    return KvcServer(ops, num_blocks=NUM_BLOCKS, reserved_blocks=RESERVED, swap_blocks=SWAP_BLOCKS, block_size=BS,
                     hq=HQ, hkv=HKV, d=D, max_blocks_per_seq=LMAX, kv_fn=kv_fn, q_fn=q_fn, sweet_spot=SWEET_SPOT,
                     token_budget=128, m=2, buffer_tokens=8, iteration_time=0.02, eps=0.0)


def run(server, oracle_mod, tol, max_iterations=400, verbose=False):
    """Drive the scenario to completion, checking every output against the dense reference."""
    pending = sorted(ARRIVALS, key=lambda a: a[1])
    log = []
    for it in range(max_iterations):
        while pending and pending[0][1] <= it:
            rid, _, sp, so, true_out, ttft, tbt = pending.pop(0)
            server.submit(ServedRequest(rid=rid, prompt_len=sp, est_output_len=so, true_output_len=true_out,
                                        ttft_slo=ttft, tbt_slo=tbt))
        before = {rid: r.length for rid, r in server.reqs.items()}
        res = server.step()
        log += [f"{it}: {e}" for e in res["events"]]
        if verbose:
            for e in res["events"]:
                print(f"[serving] {it}: {e}", flush=True)
        for rid, out in res["prefill"].items():
            ref = reference_prefill(oracle_mod, rid, out.shape[0])
            err = np.abs(np.asarray(out, dtype=np.float64) - ref).max()
            assert err <= tol, ("prefill", it, rid, err)
        for rid, out in res["decode"].items():
            r = server.reqs[rid]
            ref = reference_decode(oracle_mod, rid, r.length)
            err = np.abs(np.asarray(out, dtype=np.float64) - ref).max()
            assert err <= tol, ("decode", it, rid, err)
        if not pending and server.all_done():
            break
    return log
