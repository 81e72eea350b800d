"""Profile the attention part of recomputation against sequence length on MI355X.

The paper's preemption-strategy selection (Section 3.5) fits a polynomial regressor
L_r(S) = alpha * S^beta + kappa * S + eps to profiled recomputation times and compares it with
the linear swap regressor.  Recomputation re-runs prefill over the preempted request's S tokens;
this module times the part of it that is on this library's path - causal attention over the
paged KV cache, `paged_attention_prefill`, for every layer - reports the achieved MFMA rate and
fits the power law alpha * S^beta by least squares in log-log space.  The dense projections
and MLPs of a full prefill are outside this library, so the figure is a lower bound on L_r.

    python -m paper_2503_13773_amd.recompute_profile [--layers 32] [--q-heads 32] [--kv-heads 8]
"""
from __future__ import annotations

import argparse
import json
import math
from typing import Dict, List, Sequence, Tuple

MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16


def causal_attention_flops(S: int, q_heads: int, head_dim: int) -> float:
    """QK^T and PV multiply-adds over the causal triangle: 4 * D * Hq * S (S + 1) / 2."""
    return 4.0 * head_dim * q_heads * S * (S + 1) / 2.0


def profile_recompute(seq_lens: Sequence[int], *, layers: int = 32, q_heads: int = 32, kv_heads: int = 8,
                      head_dim: int = 128, block_size: int = 16, reps: int = 5, seed: int = 0,
                      fit_from: int = 2048, batch: int = 1, settle_ms: float = 30.0, timed_ms: float = 20.0) -> Dict:
    """Time the causal attention of `batch` requests of S tokens each (recomputed in one launch,
    every request with a block list of its own) for every S in seq_lens.  Each length is launched
    back to back for `settle_ms` first (after an idle spell the device's clocks need 10-20 ms of
    work to settle; a recomputation runs one such launch per layer, so the settled rate is the
    one that counts), then timed over at least `reps` launches and about `timed_ms`."""
    import time

    import torch

    from . import binding as K
    from . import policy

    gen = torch.Generator(device="cpu").manual_seed(seed)
    smax = max(seq_lens)
    per_seq = (smax + block_size - 1) // block_size
    nb = per_seq * batch + 8
    k_cache = torch.randn((nb, kv_heads, block_size, head_dim), generator=gen).to(torch.bfloat16).cuda()
    v_cache = torch.randn((nb, kv_heads, block_size, head_dim), generator=gen).to(torch.bfloat16).cuda()
    q_all = torch.randn((smax * batch, q_heads, head_dim), generator=gen).to(torch.bfloat16).cuda()
    table = torch.randperm(nb, generator=gen)[:per_seq * batch].reshape(batch, per_seq).to(torch.int32).cuda()
    stream = torch.cuda.current_stream()
    samples: List[Dict] = []
    for S in seq_lens:
        q = q_all[:S * batch].contiguous()
        lens = torch.full((batch,), S, dtype=torch.int32, device="cuda")
        qs = (torch.arange(batch + 1, dtype=torch.int32) * S).cuda()
        out = torch.empty_like(q)
        scale = 1.0 / math.sqrt(head_dim)
        fl = causal_attention_flops(S, q_heads, head_dim) * batch
        K.paged_attention_prefill(q, k_cache, v_cache, table, lens, qs, scale, S, out)
        t_end = time.perf_counter() + settle_ms * 1e-3
        while time.perf_counter() < t_end:
            for _ in range(8):
                K.paged_attention_prefill(q, k_cache, v_cache, table, lens, qs, scale, S, out)
            torch.cuda.synchronize()
        n = max(reps, int(timed_ms * 1e-3 / (fl / 1.0e15)))
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record(stream)
        for _ in range(n):
            K.paged_attention_prefill(q, k_cache, v_cache, table, lens, qs, scale, S, out)
        b.record(stream)
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / n
        samples.append({"S": int(S), "batch": int(batch), "layer_ms": ms, "all_layers_ms": ms * layers,
                        "tflops": fl / ms / 1e9, "frac_of_mfma_peak": fl / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS})
    fit = [s for s in samples if s["S"] >= fit_from] if sum(s["S"] >= fit_from for s in samples) >= 2 else samples
    alpha, beta, _ = policy.fit_power_law([s["S"] for s in fit], [s["all_layers_ms"] for s in fit])
    return {"fit_from": fit_from, "model": {"layers": layers, "q_heads": q_heads, "kv_heads": kv_heads, "head_dim": head_dim,
                      "block_size": block_size}, "samples": samples, "alpha_ms": alpha, "beta": beta}


def markdown(res: Dict, swap_gamma_ms: float, swap_delta_ms: float) -> str:
    """The table, the fit and the crossover with the swap regressor L_s = gamma * S + delta."""
    from . import policy

    m = res["model"]
    lines = ["%d request(s) per launch." % res["samples"][0].get("batch", 1), "",
             "| S tokens | per layer ms | all %d layers ms | TFLOP/s | %% of MFMA peak |" % m["layers"], "|---|---|---|---|---|"]
    for s in res["samples"]:
        lines.append("| %d | %.3f | %.2f | %.1f | %.1f |" % (s["S"], s["layer_ms"], s["all_layers_ms"], s["tflops"],
                                                           100 * s["frac_of_mfma_peak"]))
    lines.append("")
    lines.append("Power-law fit over S >= %d (all layers): L_r(S) = %.4g ms * S^%.3f." % (res["fit_from"], res["alpha_ms"],
                                                                                         res["beta"]))
    ss = policy.sweet_spot(swap_gamma_ms, swap_delta_ms, res["alpha_ms"], res["beta"], 0.0, 0.0, 1e6)
    lines.append("Against L_s(S) = %.6g ms * S + %.4g ms the two meet at S_s = %.0f tokens." % (swap_gamma_ms, swap_delta_ms, ss))
    return "\n".join(lines)


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--q-heads", type=int, default=32)
    ap.add_argument("--kv-heads", type=int, default=8)
    ap.add_argument("--seq-lens", type=int, nargs="+", default=[256, 512, 1024, 2048, 4096, 8192, 16384])
    ap.add_argument("--reps", type=int, default=5, help="least number of timed launches per length")
    ap.add_argument("--settle-ms", type=float, default=30.0, help="untimed back-to-back launches before each length")
    ap.add_argument("--batch", type=int, default=1, help="requests of S tokens recomputed in one launch")
    ap.add_argument("--markdown", action="store_true", help="print a table instead of JSON")
    ap.add_argument("--swap-gamma-ms", type=float, default=0.004766, help="slope of the swap regressor (ms per token)")
    ap.add_argument("--swap-delta-ms", type=float, default=0.069, help="offset of the swap regressor (ms)")
    args = ap.parse_args()
    res = profile_recompute(args.seq_lens, layers=args.layers, q_heads=args.q_heads, kv_heads=args.kv_heads,
                            reps=args.reps, batch=args.batch, settle_ms=args.settle_ms)
    print(markdown(res, args.swap_gamma_ms, args.swap_delta_ms) if args.markdown else json.dumps(res))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
