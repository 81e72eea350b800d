"""Seeded synthetic inputs for the paged-KV decode path.

This module only *generates inputs*: block tables, context lengths, KV pools,
queries and block-copy mappings.  It holds none of the method's arithmetic (no
dot products, no softmax, no copies of KV data between pools), so the CPU
oracle and the HIP path can both be fed from it without sharing any code that
could hide a common mistake.

The workloads are stand-ins for the serving traces the paper evaluates on
(Section 2.1 / Table 1: three public request traces with mean prompt+output
lengths of roughly 78, 500 and 2600 tokens).  No trace item is reproduced: only
the *length statistics* shape the inputs.  Sequence lengths follow a
prompt+generated lognormal mix that sits between the two longer traces;
values are N(0,1); physical blocks are scattered over the pool the way a
block-based allocator under KV-cache competition leaves them (Section 1:
block-based allocation; Section 3.3.1: requests embedded in other requests'
unused allocation, hence arbitrary interleaved placement).

Layout produced here (row-major, last index fastest):
    q            [num_seqs][num_q_heads][head_dim]
    k_cache      [num_pool_blocks][num_kv_heads][block_size][head_dim]
    v_cache      [num_pool_blocks][num_kv_heads][block_size][head_dim]
    block_tables [num_seqs][max_blocks_per_seq]  int32 (unused entries = -1)
    context_lens [num_seqs]                      int32
bf16 tensors are carried as uint16 bit patterns (numpy has no bf16).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

F32 = "f32"
BF16 = "bf16"


# --------------------------------------------------------------------------
# bf16 <-> f32 bit conversions (storage format only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns uint16 bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    out = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = np.uint16(0x7FC0)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to float32 (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal(rng: np.random.Generator, shape, dtype: str) -> np.ndarray:
    """N(0,1) samples stored in `dtype` (float32 array, or uint16 bf16 bits)."""
    n = int(np.prod(shape))
    if dtype == F32:
        return rng.standard_normal(n, dtype=np.float32).reshape(shape)
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 24
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        out[lo:hi] = f32_to_bf16_bits(rng.standard_normal(hi - lo, dtype=np.float32))
    return out.reshape(shape)


def to_float64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of a stored tensor to float64 (for test-side references)."""
    if dtype == F32:
        return a.astype(np.float64)
    return bf16_bits_to_f32(a).astype(np.float64)


# --------------------------------------------------------------------------
# workload container
# --------------------------------------------------------------------------
@dataclass
class PagedWorkload:
    name: str
    dtype: str
    num_seqs: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    block_size: int
    max_blocks_per_seq: int
    num_pool_blocks: int
    scale: float
    q: np.ndarray
    k_cache: np.ndarray
    v_cache: np.ndarray
    block_tables: np.ndarray
    context_lens: np.ndarray
    extra: Dict = field(default_factory=dict)

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == F32 else 2

    @property
    def max_context_len(self) -> int:
        return int(self.context_lens.max()) if self.num_seqs else 0

    def kv_bytes(self) -> int:
        """Algorithmic K+V bytes one decode step must read (no block padding)."""
        per_tok = 2 * self.num_kv_heads * self.head_dim * self.elem_bytes
        return int(self.context_lens.astype(np.int64).sum()) * per_tok

    def qo_bytes(self) -> int:
        return 2 * self.num_seqs * self.num_q_heads * self.head_dim * self.elem_bytes

    def block_bytes(self) -> int:
        """Bytes of one block of one plane (K or V of one layer)."""
        return self.num_kv_heads * self.block_size * self.head_dim * self.elem_bytes


def blocks_needed(context_lens: np.ndarray, block_size: int) -> np.ndarray:
    return (context_lens.astype(np.int64) + block_size - 1) // block_size


# --------------------------------------------------------------------------
# length mixes
# --------------------------------------------------------------------------
def lognormal_context_lens(rng: np.random.Generator, n: int, cap_each: int,
                           cap_total: Optional[int] = None) -> np.ndarray:
    """context_len = prompt + generated, both lognormal, clipped.

    prompt ~ LN(6.0, 0.8) clipped to [8, cap_each]; generated ~ LN(5.3, 1.0)
    clipped to [1, cap_each]; rounded to the nearest integer; the sum is capped
    at cap_total when given.
    """
    prompt = np.clip(np.rint(rng.lognormal(6.0, 0.8, n)), 8, cap_each)
    gen = np.clip(np.rint(rng.lognormal(5.3, 1.0, n)), 1, cap_each)
    ctx = prompt + gen
    if cap_total is not None:
        ctx = np.minimum(ctx, cap_total)
    return ctx.astype(np.int32)


# --------------------------------------------------------------------------
# generic builder
# --------------------------------------------------------------------------
def build_workload(name: str, rng: np.random.Generator, *, dtype: str,
                   context_lens: np.ndarray, num_q_heads: int, num_kv_heads: int,
                   head_dim: int, block_size: int, max_blocks_per_seq: int,
                   num_pool_blocks: Optional[int] = None, occupancy: float = 1.0,
                   share_groups: Optional[List[Tuple[List[int], int]]] = None,
                   scale: Optional[float] = None) -> PagedWorkload:
    """Scatter each sequence's blocks over a pool by a random permutation.

    share_groups: list of (sequence ids, k): the sequences of a group reference
    the *same* physical block ids for their first k blocks (a shared prefix).
    """
    context_lens = np.asarray(context_lens, dtype=np.int32)
    nseq = int(context_lens.shape[0])
    nblk = blocks_needed(context_lens, block_size)
    assert (nblk <= max_blocks_per_seq).all(), "context longer than the table row"

    shared_from: Dict[int, Tuple[int, int]] = {}  # seq -> (leader seq, k)
    if share_groups:
        for seqs, k in share_groups:
            leader = seqs[0]
            for s in seqs[1:]:
                assert k <= nblk[s] and k <= nblk[leader]
                shared_from[s] = (leader, k)

    private = nblk.copy()
    for s, (_, k) in shared_from.items():
        private[s] -= k
    need = int(private.sum())
    if num_pool_blocks is None:
        num_pool_blocks = max(1, int(math.ceil(need / occupancy)))
    assert num_pool_blocks >= need
    perm = rng.permutation(num_pool_blocks)[:need].astype(np.int32)

    tables = np.full((nseq, max_blocks_per_seq), -1, dtype=np.int32)
    pos = 0
    order = [s for s in range(nseq) if s not in shared_from] + list(shared_from)
    for s in order:
        if s in shared_from:
            leader, k = shared_from[s]
            tables[s, :k] = tables[leader, :k]
            cnt = int(nblk[s]) - k
            tables[s, k:k + cnt] = perm[pos:pos + cnt]
        else:
            cnt = int(nblk[s])
            tables[s, :cnt] = perm[pos:pos + cnt]
        pos += cnt
    assert pos == need

    pool_shape = (num_pool_blocks, num_kv_heads, block_size, head_dim)
    q = _normal(rng, (nseq, num_q_heads, head_dim), dtype)
    k_cache = _normal(rng, pool_shape, dtype)
    v_cache = _normal(rng, pool_shape, dtype)
    if scale is None:
        scale = 1.0 / math.sqrt(head_dim)
    used = np.zeros(num_pool_blocks, dtype=bool)
    used[perm] = True
    return PagedWorkload(name=name, dtype=dtype, num_seqs=nseq, num_q_heads=num_q_heads,
                         num_kv_heads=num_kv_heads, head_dim=head_dim, block_size=block_size,
                         max_blocks_per_seq=max_blocks_per_seq, num_pool_blocks=num_pool_blocks,
                         scale=float(scale), q=q, k_cache=k_cache, v_cache=v_cache,
                         block_tables=tables, context_lens=context_lens,
                         extra={"free_blocks": np.flatnonzero(~used).astype(np.int64),
                                "share_groups": share_groups or []})


# --------------------------------------------------------------------------
# the named configurations
# --------------------------------------------------------------------------
SEEDS = {"cfg1": 1001, "cfg2": 1002, "cfg3": 1003, "cfg3b": 1013, "cfg4": 1004, "cfg5": 1005}


def _share_groups(rng: np.random.Generator, context_lens: np.ndarray, block_size: int,
                  frac: float) -> List[Tuple[List[int], int]]:
    """Pick ~frac of the sequences, in groups of 2-4, sharing k full prefix blocks."""
    nseq = len(context_lens)
    full = context_lens.astype(np.int64) // block_size  # full blocks only
    cand = [int(s) for s in rng.permutation(nseq) if full[s] >= 2]
    want = int(round(frac * nseq))
    groups: List[Tuple[List[int], int]] = []
    i = 0
    while want >= 2 and i + 2 <= len(cand):
        g = int(min(want, rng.integers(2, 5), len(cand) - i))
        if want - g == 1:          # never leave a group of one
            g = g - 1 if g > 2 else g + 1
            g = min(g, len(cand) - i)
        seqs = cand[i:i + g]
        kmax = int(min(full[s] for s in seqs)) - 1
        k = int(rng.integers(1, kmax + 1))
        groups.append((seqs, k))
        i += g
        want -= g
    return groups


def make_config(name: str, *, num_seqs: Optional[int] = None, seed: Optional[int] = None,
                ctx_scale: float = 1.0, block_size: int = 16) -> PagedWorkload:
    """Build one of the named workloads.

    cfg1  tiny fp32 MHA (4 seqs, 8 heads, D 64, ctx U[16,256], pool 128 blocks)
    cfg2  7B-shape MHA bf16, batch 64, 32 heads, D 128, lognormal mix (parts capped 2048)
    cfg3  8B-shape GQA bf16, batch 128, 32/8 heads, lognormal mix capped at 4096,
          pool at 90 % occupancy, random scatter
    cfg3b cfg3 at batch 64 (the headline configuration)
    cfg4  long-context bf16, batch 16, 64/8 heads, ctx U[8192,32768]
    cfg5  8B GQA bf16, batch 96, 25 % of sequences in prefix-sharing groups, pool at
          75 % occupancy (the swap-in needs free slots); extra["swap"] holds the swap-out / swap-in plan for 20 % of sequences

    num_seqs / ctx_scale shrink a config for oracle-sized parity cases
    (ctx_scale multiplies every context length, minimum 1).  block_size other than
    the configs' 16 serves the block-size sweep (the paper's own default is 8, its
    analysis runs use 32); the table rows keep their token capacity.
    """
    rng = np.random.default_rng(SEEDS[name] if seed is None else seed)
    bs = block_size
    assert bs >= 1 and (bs & (bs - 1)) == 0
    rows = lambda tokens: (tokens + bs - 1) // bs   # table row length for a token capacity

    def scaled(c):
        if ctx_scale == 1.0:
            return c
        return np.maximum(1, np.rint(c * ctx_scale)).astype(np.int32)

    if name == "cfg1":
        n = num_seqs or 4
        ctx = scaled(rng.integers(16, 257, n).astype(np.int32))
        return build_workload(name, rng, dtype=F32, context_lens=ctx, num_q_heads=8,
                              num_kv_heads=8, head_dim=64, block_size=bs,
                              max_blocks_per_seq=rows(256), num_pool_blocks=max(128, 16 * n) * 16 // min(bs, 16))
    if name == "cfg2":
        n = num_seqs or 64
        ctx = scaled(lognormal_context_lens(rng, n, 2048))
        return build_workload(name, rng, dtype=BF16, context_lens=ctx, num_q_heads=32,
                              num_kv_heads=32, head_dim=128, block_size=bs,
                              max_blocks_per_seq=rows(4096))
    if name in ("cfg3", "cfg3b"):
        n = num_seqs or (128 if name == "cfg3" else 64)
        ctx = scaled(lognormal_context_lens(rng, n, 4096, 4096))
        return build_workload(name, rng, dtype=BF16, context_lens=ctx, num_q_heads=32,
                              num_kv_heads=8, head_dim=128, block_size=bs,
                              max_blocks_per_seq=rows(4096), occupancy=0.9)
    if name == "cfg4":
        n = num_seqs or 16
        ctx = scaled(rng.integers(8192, 32769, n).astype(np.int32))
        return build_workload(name, rng, dtype=BF16, context_lens=ctx, num_q_heads=64,
                              num_kv_heads=8, head_dim=128, block_size=bs,
                              max_blocks_per_seq=rows(32768))
    if name == "cfg5":
        n = num_seqs or 96
        ctx = scaled(lognormal_context_lens(rng, n, 4096, 4096))
        groups = _share_groups(rng, ctx, bs, 0.25)
        w = build_workload(name, rng, dtype=BF16, context_lens=ctx, num_q_heads=32,
                           num_kv_heads=8, head_dim=128, block_size=bs,
                           max_blocks_per_seq=rows(4096), occupancy=0.75, share_groups=groups)
        w.extra["swap"] = make_swap_plan(rng, w, 0.20)
        return w
    raise KeyError(name)


# --------------------------------------------------------------------------
# block-copy mappings
# --------------------------------------------------------------------------
def make_copy_mapping(rng: np.random.Generator, n_pairs: int, src_blocks: int,
                      dst_blocks: int) -> np.ndarray:
    """n_pairs distinct random src ids -> n_pairs distinct random dst ids; int64 [n][2]."""
    src = rng.permutation(src_blocks)[:n_pairs]
    dst = rng.permutation(dst_blocks)[:n_pairs]
    return np.stack([src, dst], axis=1).astype(np.int64)


def make_swap_plan(rng: np.random.Generator, w: PagedWorkload, frac: float) -> Dict:
    """Swap-out / swap-in plan for ceil(frac * num_seqs) sequences that own their blocks.

    Returns the victim sequence ids, the mapping pool1 -> pool2 (swap-out), the
    mapping pool2 -> pool1 into *different* free slots (swap-in), the size of
    the second pool and the block tables as they read after the swap-in.
    """
    in_group = set()
    for seqs, _ in w.extra.get("share_groups", []):
        in_group.update(seqs)
    cand = [s for s in range(w.num_seqs) if s not in in_group]
    nvict = min(len(cand), int(math.ceil(frac * w.num_seqs)))
    free = rng.permutation(w.extra["free_blocks"])
    nblk = blocks_needed(w.context_lens, w.block_size)
    # the swap-in needs free slots in pool 1: keep victims while they fit
    victims: List[int] = []
    total = 0
    for s in rng.permutation(cand):
        if len(victims) == nvict:
            break
        if total + int(nblk[s]) <= len(free):
            victims.append(int(s))
            total += int(nblk[s])
    src = np.concatenate([w.block_tables[s, :nblk[s]] for s in victims]).astype(np.int64) \
        if victims else np.zeros(0, np.int64)
    pool2_blocks = max(1, int(math.ceil(total * 1.25)))
    slot2 = rng.permutation(pool2_blocks)[:total].astype(np.int64)
    back = free[:total].astype(np.int64)
    tables_after = w.block_tables.copy()
    pos = 0
    for s in victims:
        c = int(nblk[s])
        tables_after[s, :c] = back[pos:pos + c]
        pos += c
    return {"victims": victims, "pool2_blocks": pool2_blocks,
            "out_mapping": np.stack([src, slot2], axis=1).astype(np.int64),
            "in_mapping": np.stack([slot2, back], axis=1).astype(np.int64),
            "tables_after": tables_after}
