"""Profile swap latency against sequence length and fit the linear regressor L_s(S) = gamma * S + delta.

The paper's preemption-strategy selection (Section 3.5) profiles, on the target hardware, the time
to swap a preempted request's KV cache out to CPU memory and back in for a range of sequence
lengths S, fits a linear regressor to it, and later compares it with the recomputation regressor to
find the sweet-spot length above which swapping wins (Section 2.5 reports the crossover at about
4000 tokens on the paper's hardware).  This module does the swap half on MI355X: the KV blocks of
a sequence of S tokens (all layers, K and V planes) are moved between an HBM pool and a pinned
host pool by `kv_block_copy`, timed with HIP events, and the line is fitted by least squares.

    python -m paper_2503_13773_amd.swap_profile [--layers 32] [--kv-heads 8] [--head-dim 128] ...
"""
from __future__ import annotations

import argparse
import json
from typing import Dict, List, Sequence, Tuple


def profile_swap(seq_lens: Sequence[int], *, layers: int = 32, kv_heads: int = 8, head_dim: int = 128,
                 block_size: int = 16, elem_bytes: int = 2, pool_blocks: int = 0, reps: int = 5,
                 seed: int = 0) -> Dict:
    """Time swap-out + swap-in of one sequence's KV blocks for every S in seq_lens.

    Pools are [2 * layers planes][blocks][block_bytes]; the HBM pool holds `pool_blocks` blocks
    (default: twice the longest sequence) from which the sequence's blocks are picked at random,
    the pinned host pool holds exactly the blocks of the longest sequence.
    """
    import torch

    from . import binding as K
    from . import policy

    planes = 2 * layers
    block_bytes = kv_heads * block_size * head_dim * elem_bytes
    max_blocks = (max(seq_lens) + block_size - 1) // block_size
    pool_blocks = pool_blocks or 2 * max_blocks
    gen = torch.Generator(device="cpu").manual_seed(seed)
    hbm = torch.randint(0, 255, (planes, pool_blocks, block_bytes), dtype=torch.uint8, device="cuda")
    host = torch.zeros((planes, max_blocks, block_bytes), dtype=torch.uint8, pin_memory=True)
    stream = torch.cuda.current_stream()
    samples: List[Dict] = []
    for S in seq_lens:
        nb = (S + block_size - 1) // block_size
        src = torch.randperm(pool_blocks, generator=gen)[:nb]
        slot = torch.randperm(max_blocks, generator=gen)[:nb]
        back = torch.randperm(pool_blocks, generator=gen)[:nb]
        out_map = torch.stack([src, slot], dim=1).to(torch.int64).cuda()
        in_map = torch.stack([slot, back], dim=1).to(torch.int64).cuda()
        t_out, t_in = [], []
        for rep in range(reps + 1):
            e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            e[0].record(stream)
            K.kv_block_copy(hbm, host, out_map)
            e[1].record(stream)
            K.kv_block_copy(host, hbm, in_map)
            e[2].record(stream)
            torch.cuda.synchronize()
            if rep:                       # first repetition warms up
                t_out.append(e[0].elapsed_time(e[1]))
                t_in.append(e[1].elapsed_time(e[2]))
        nbytes = nb * block_bytes * planes
        o, i = sorted(t_out)[len(t_out) // 2], sorted(t_in)[len(t_in) // 2]
        samples.append({"S": int(S), "blocks": int(nb), "bytes_each_way": int(nbytes), "swap_out_ms": o,
                        "swap_in_ms": i, "swap_ms": o + i,
                        "out_GBs": nbytes / o / 1e6, "in_GBs": nbytes / i / 1e6})
    Ss = [s["S"] for s in samples]
    gamma, delta, r2 = policy.fit_linear(Ss, [s["swap_ms"] for s in samples])
    return {"model": {"layers": layers, "kv_heads": kv_heads, "head_dim": head_dim, "block_size": block_size,
                      "bytes_per_token": 2 * layers * kv_heads * head_dim * elem_bytes},
            "samples": samples, "gamma_ms_per_token": gamma, "delta_ms": delta,
            "r2": r2}


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--kv-heads", type=int, default=8)
    ap.add_argument("--head-dim", type=int, default=128)
    ap.add_argument("--block-size", type=int, default=16)
    ap.add_argument("--seq-lens", type=int, nargs="+",
                    default=[128, 256, 512, 1024, 2048, 4096, 8192, 16384])
    ap.add_argument("--reps", type=int, default=5)
    args = ap.parse_args()
    res = profile_swap(args.seq_lens, layers=args.layers, kv_heads=args.kv_heads, head_dim=args.head_dim,
                       block_size=args.block_size, reps=args.reps)
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
