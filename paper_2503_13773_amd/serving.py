"""Iteration-level serving loop that lets the policy core drive the device calls.

Every scheduling decision comes from ``kvcp_schedule_step`` (include/kvc_policy.h: batch
formation, embedding, preemption order, swap-or-recompute, proactive allocation, borrowing:
paper Sections 3.3-3.5); this module only keeps the books the decisions refer to (which request
owns which blocks, who is embedded where, what sits in the swap space) and turns them into the
device calls of include/kvc.h:

    kv_cache_append            the new token of every batched request, and the K/V of a request
                               that is admitted or recomputed
    paged_attention_decode     one decode iteration over the batch
    paged_attention_prefill    the attention of an admitted or recomputed request over all its
                               positions (the recomputation path)
    kv_block_copy              swap-out to / swap-in from pinned host memory

The model around the attention (projections that produce q, k, v; sampling) is outside this
library: the caller supplies it as two functions, ``kv_fn(request id, position)`` and
``q_fn(request id, position)``, returning bf16 bit patterns.  Time is iteration-counted: one call
of ``step`` is one iteration of length ``iteration_time``.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional

import numpy as np

from . import policy as P

NEW, RUNNING, SWAPPED, DROPPED, DONE = "new", "running", "swapped", "dropped", "done"


@dataclass
class ServedRequest:
    rid: int
    prompt_len: int
    est_output_len: int          # s^o after padding (Section 3.2); the policy plans with it
    true_output_len: int         # when the request really finishes (unknown to the policy)
    ttft_slo: float
    tbt_slo: float
    arrival: float = 0.0
    state: str = NEW
    generated: int = 0
    length: int = 0              # tokens whose K/V are in the cache (or in swap space)
    blocks: List[int] = field(default_factory=list)   # block table of the request, in order
    owns_blocks: bool = True     # False while embedded: the blocks belong to the host
    alloc_tokens: int = 0        # a_i as the policy counts it
    host: Optional[int] = None   # rid of the request it is embedded in
    guest: Optional[int] = None  # rid of the request embedded in it
    guest_first_block: int = 0   # index in `blocks` where the guest's range starts
    lender: Optional[int] = None
    swap_slots: List[int] = field(default_factory=list)
    last_token_time: float = 0.0


class HipOps:
    """The device side: pools in HBM, swap space in pinned host memory, calls through the C ABI."""

    def __init__(self, num_blocks: int, swap_blocks: int, hq: int, hkv: int, d: int, block_size: int):
        import torch

        from . import binding as K
        self.K, self.torch = K, torch
        self.pool = torch.zeros((2, num_blocks, hkv, block_size, d), dtype=torch.bfloat16, device="cuda")
        self.swap = torch.zeros((2, max(1, swap_blocks), hkv, block_size, d), dtype=torch.bfloat16, pin_memory=True)
        self.scale = 1.0 / math.sqrt(d)

    def _bf16(self, a: np.ndarray):
        return self.torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(self.torch.bfloat16)

    def _i32(self, a: np.ndarray):
        return self.torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()

    def append(self, k_new, v_new, tables, positions) -> None:
        self.K.kv_cache_append(self._bf16(k_new), self._bf16(v_new), self.pool[0], self.pool[1],
                               self._i32(tables), self._i32(positions))

    def decode(self, q, tables, lens) -> np.ndarray:
        out = self.K.paged_attention_decode(self._bf16(q), self.pool[0], self.pool[1], self._i32(tables),
                                            self._i32(lens), self.scale)
        return out.float().cpu().numpy()

    def prefill(self, q, tables, lens, q_start) -> np.ndarray:
        out = self.K.paged_attention_prefill(self._bf16(q), self.pool[0], self.pool[1], self._i32(tables),
                                             self._i32(lens), self._i32(q_start), self.scale,
                                             max_query_len=int(np.diff(q_start).max()))
        return out.float().cpu().numpy()

    def copy_out(self, block_ids, slots) -> None:
        m = self.torch.tensor(list(zip(block_ids, slots)), dtype=self.torch.int64).cuda()
        self.K.kv_block_copy(self.pool, self.swap, m)
        self.torch.cuda.synchronize()     # the blocks are released to other requests right after

    def copy_in(self, slots, block_ids) -> None:
        m = self.torch.tensor(list(zip(slots, block_ids)), dtype=self.torch.int64).cuda()
        self.K.kv_block_copy(self.swap, self.pool, m)

    def poison(self, block_ids) -> None:
        """Released blocks hold garbage from now on (NaN here, so that a stale reference shows)."""
        if block_ids:
            self.pool[:, self.torch.tensor(list(block_ids)).cuda()] = float("nan")


class KvcServer:
    def __init__(self, ops, *, num_blocks: int, reserved_blocks: int, swap_blocks: int, block_size: int,
                 hq: int, hkv: int, d: int, max_blocks_per_seq: int, kv_fn: Callable, q_fn: Callable,
                 sweet_spot: float, token_budget: int = 512, m: int = 2, buffer_tokens: int = 8,
                 iteration_time: float = 0.02, eps: float = 0.0, slo_edges=(0.2, 0.5), token_bucket: int = 128):
        self.ops, self.bs, self.hq, self.hkv, self.d = ops, block_size, hq, hkv, d
        self.lmax = max_blocks_per_seq
        self.bm = P.BlockManager(num_blocks, reserved_blocks)
        self.kv_fn, self.q_fn = kv_fn, q_fn
        self.params = dict(block_tokens=block_size, buffer_tokens=buffer_tokens, token_budget=token_budget,
                           token_bucket=token_bucket, m=m, slo_edges=tuple(slo_edges), eps=eps,
                           iter_time_base=iteration_time, iter_time_per_token=0.0, sweet_spot=sweet_spot)
        self.dt = iteration_time
        self.now = 0.0
        self.max_iter_latency = iteration_time
        self.reqs: Dict[int, ServedRequest] = {}
        self.swap_free = list(range(swap_blocks))
        self.stats = dict(iterations=0, swapped=0, recomputed=0, swap_ins=0, embedded=0, overruns=0,
                          reserved_blocks_used=0, proactive=0, borrowed=0, allocation_failures=0)

    # ---- bookkeeping -------------------------------------------------------------------------
    def submit(self, r: ServedRequest) -> None:
        r.arrival = self.now
        self.reqs[r.rid] = r

    def _blocks_for(self, tokens: int) -> int:
        return (tokens + self.bs - 1) // self.bs

    def _take_blocks(self, n: int) -> Optional[List[int]]:
        """General pool first; the shared reserved pool serves allocation failures (Section 3.3.3)."""
        if n <= 0:
            return []
        got = self.bm.allocate(n)
        if got is None:
            got = self.bm.allocate_reserved(n)
            if got is not None:
                self.stats["reserved_blocks_used"] += n
        return got

    def _release(self, r: ServedRequest) -> None:
        """Give back what r owns.  Blocks its guest sits in pass to the guest."""
        if not r.owns_blocks:
            h = self.reqs.get(r.host)
            if h is not None and h.guest == r.rid:
                h.guest = None
            r.blocks, r.host, r.owns_blocks = [], None, True
            return
        keep: List[int] = []
        if r.guest is not None:
            g = self.reqs[r.guest]
            keep = list(g.blocks)
            g.owns_blocks, g.host = True, None
            r.guest = None
        gone = [b for b in r.blocks if b not in keep]
        if gone:
            self.ops.poison(gone)
            self.bm.release(gone)
        r.blocks = []

    def _preempt(self, r: ServedRequest, swap: bool) -> None:
        """Take r out of the cache: its KV goes to the swap space, or is dropped for recomputation."""
        if r.guest is not None:                       # the guest loses its place with the host
            g = self.reqs[r.guest]
            self._preempt(g, P.choose_swap(float(g.length), self.params["sweet_spot"]))
        used = r.blocks[:self._blocks_for(r.length)]
        if swap and len(self.swap_free) >= len(used) and used:
            r.swap_slots = [self.swap_free.pop() for _ in used]
            self.ops.copy_out(used, r.swap_slots)
            r.state = SWAPPED
            self.stats["swapped"] += 1
        else:
            r.state = DROPPED
            self.stats["recomputed"] += 1
        self._release(r)
        r.alloc_tokens = 0

    def _policy_request(self, r: ServedRequest) -> P.Request:
        if r.state == RUNNING:
            rt = max(1e-9, r.last_token_time + r.tbt_slo - self.now)
            return P.Request(state=P.RUNNING, reserved=0, prompt_len=r.prompt_len, est_output_len=r.est_output_len,
                             generated=r.generated, allocated=max(r.alloc_tokens, r.length), used=r.length,
                             remaining_time=rt, tbt_slo=r.tbt_slo)
        deadline = r.arrival + r.ttft_slo if r.state == NEW else r.last_token_time + r.tbt_slo
        # a preempted request comes back with everything it had produced as its "prompt"
        sp = r.prompt_len + r.generated
        so = max(1, r.est_output_len - r.generated)
        return P.Request(state=P.WAITING, reserved=0, prompt_len=sp, est_output_len=so, generated=0, allocated=0,
                         used=0, remaining_time=max(1e-9, deadline - self.now), tbt_slo=r.tbt_slo)

    # ---- one iteration ------------------------------------------------------------------------
    def step(self) -> Dict:
        """Schedule, move KV as decided, run one decode iteration.  Returns what was computed:
        {"decode": {rid: out[hq][d]}, "prefill": {rid: out[len][hq][d]}, "events": [...]}."""
        live = [r for r in self.reqs.values() if r.state != DONE]
        events: List[str] = []
        result = {"decode": {}, "prefill": {}, "events": events}
        if not live:
            return result
        order = sorted(live, key=lambda r: r.rid)
        free_tokens = self.bm.free_general * self.bs
        decisions, summary = P.schedule_step([self._policy_request(r) for r in order], unallocated=free_tokens,
                                             max_iteration_latency=self.max_iter_latency, **self.params)
        # 1. preemptions decided by the policy
        for r, dcs in zip(order, decisions):
            if dcs.preempt != P.KEEP and r.state == RUNNING:
                events.append(f"preempt {r.rid} {'swap' if dcs.preempt == P.PREEMPT_SWAP else 'recompute'}")
                self._preempt(r, dcs.preempt == P.PREEMPT_SWAP)
        # 2. grants to running requests (critical, N'_r, proactive) and lenders
        for r, dcs in zip(order, decisions):
            if r.state != RUNNING:
                continue
            if dcs.proactive and dcs.grant:
                self.stats["proactive"] += 1
            if dcs.lender >= 0:
                r.lender = order[dcs.lender].rid
                self.stats["borrowed"] += 1
            if dcs.grant and r.owns_blocks:
                want = self._blocks_for(max(r.alloc_tokens, r.length) + dcs.grant) - len(r.blocks)
                got = self._take_blocks(min(want, self.lmax - len(r.blocks)))
                if got:
                    r.blocks += got
                    r.alloc_tokens = len(r.blocks) * self.bs
        # 3. admissions: embedded, or into blocks of their own
        admitted: List[ServedRequest] = []
        for r, dcs in zip(order, decisions):
            if r.state == RUNNING or not dcs.in_batch:
                continue
            need_now = self._blocks_for(r.length if r.state != NEW else r.prompt_len)
            if dcs.host >= 0:
                h = order[dcs.host]
                rng_ = P.embedding_block_range(len(h.blocks) * self.bs, dcs.s0, r.prompt_len + r.generated,
                                               max(1, r.est_output_len - r.generated), self.bs, len(h.blocks))
                if rng_ is None or h.guest is not None or h.state != RUNNING or rng_[1] < need_now:
                    continue
                first, count = rng_
                r.blocks, r.owns_blocks, r.host = h.blocks[first:first + count], False, h.rid
                h.guest, h.guest_first_block = r.rid, first
                r.alloc_tokens = count * self.bs
                self.stats["embedded"] += 1
                events.append(f"embed {r.rid} in {h.rid} at block {first}")
            else:
                want = min(self.lmax, max(need_now, self._blocks_for(dcs.grant)))
                got = self._take_blocks(want)
                if got is None:
                    self.stats["allocation_failures"] += 1
                    continue
                r.blocks, r.owns_blocks, r.alloc_tokens = got, True, len(got) * self.bs
            if dcs.lender >= 0:
                r.lender = order[dcs.lender].rid
                self.stats["borrowed"] += 1
            admitted.append(r)
        # bring the admitted requests' KV into the cache
        for r in admitted:
            if r.state == SWAPPED:
                self.ops.copy_in(r.swap_slots, r.blocks[:len(r.swap_slots)])
                self.swap_free.extend(r.swap_slots)
                r.swap_slots = []
                self.stats["swap_ins"] += 1
                events.append(f"swap-in {r.rid}")
            else:                                     # new request, or recomputation of a dropped one
                n_tok = r.prompt_len if r.state == NEW else r.length
                table = np.full((1, self.lmax), -1, dtype=np.int32)
                table[0, :len(r.blocks)] = r.blocks
                for pos in range(n_tok):              # K/V of every position, as the model would produce them
                    k, v = self.kv_fn(r.rid, pos)
                    self.ops.append(k[None], v[None], table, np.array([pos], dtype=np.int32))
                q = np.stack([self.q_fn(r.rid, pos) for pos in range(n_tok)])
                result["prefill"][r.rid] = self.ops.prefill(q, table, np.array([n_tok], dtype=np.int32),
                                                            np.array([0, n_tok], dtype=np.int32))
                events.append(f"{'prefill' if r.state == NEW else 'recompute'} {r.rid} over {n_tok} tokens")
                r.length = n_tok
            r.state = RUNNING
            r.last_token_time = self.now
        # 4. the decode iteration: every running request appends one token and attends
        batch: List[ServedRequest] = []
        for r in sorted((x for x in self.reqs.values() if x.state == RUNNING), key=lambda x: x.rid):
            if r.state != RUNNING:                    # preempted as a guest earlier in this loop
                continue
            idx = r.length // self.bs
            if r.guest is not None and idx >= r.guest_first_block:
                g = self.reqs[r.guest]                # the host reached the guest's range: the guest goes
                self.stats["overruns"] += 1
                events.append(f"overrun: {r.rid} reaches its guest {g.rid}")
                self._preempt(g, P.choose_swap(float(g.length), self.params["sweet_spot"]))
                if g in batch:
                    batch.remove(g)
            if idx >= len(r.blocks):                  # out of KVC: borrowed / reserved blocks, else preemption
                got = self._take_blocks(1) if r.owns_blocks and len(r.blocks) < self.lmax else None
                if got is None:
                    self.stats["allocation_failures"] += 1
                    events.append(f"preempt {r.rid} (allocation failure)")
                    self._preempt(r, P.choose_swap(float(r.length), self.params["sweet_spot"]))
                    continue
                r.blocks += got
                r.alloc_tokens = len(r.blocks) * self.bs
            batch.append(r)
        batch = [r for r in batch if r.state == RUNNING]
        if batch:
            n = len(batch)
            tables = np.full((n, self.lmax), -1, dtype=np.int32)
            k_new = np.zeros((n, self.hkv, self.d), dtype=np.uint16)
            v_new = np.zeros_like(k_new)
            q = np.zeros((n, self.hq, self.d), dtype=np.uint16)
            pos = np.zeros(n, dtype=np.int32)
            for i, r in enumerate(batch):
                tables[i, :len(r.blocks)] = r.blocks
                k_new[i], v_new[i] = self.kv_fn(r.rid, r.length)
                q[i] = self.q_fn(r.rid, r.length)
                pos[i] = r.length
            self.ops.append(k_new, v_new, tables, pos)
            out = self.ops.decode(q, tables, pos + 1)
            for i, r in enumerate(batch):
                r.length += 1
                r.generated += 1
                r.last_token_time = self.now + self.dt
                result["decode"][r.rid] = out[i]
                if r.generated >= r.true_output_len:
                    r.state = DONE
                    self._release(r)
                    events.append(f"done {r.rid}")
        self.stats["iterations"] += 1
        self.now += self.dt
        return result

    def all_done(self) -> bool:
        return all(r.state == DONE for r in self.reqs.values())
