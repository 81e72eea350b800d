#!/usr/bin/env python3
"""Benchmark of the paged-KV decode hot path on one MI355X.

A step = one pass of the whole hot path over one synthetic batch, all inputs resident in
HBM: paged_attention_decode over the batch (with the balanced kernel one launch: split
contexts are merged by the last wavefront to arrive), then kv_block_copy swapping the K and V blocks of 20 % of the batch's sequences out to a second
device pool.  Successive steps rotate over replicas of the KV pools at different addresses
(>= 2 GiB in total), the way successive layers of a model each own a KV pool, so that the
256 MB memory-side cache cannot serve the KV reads.  Block tables, context lengths and the
copy mapping are shared by the replicas, as they are shared by the layers of one decode step.

Before anything is timed the step's results are checked: attention rows against the CPU
oracle and the swapped-out blocks bit for bit; a mismatch ends the run with exit status 4.
Every timed loop is preceded by 30 ms of the same launches, untimed (--clock-ramp-ms): after
an idle spell the device runs its first 10-20 ms of work at lower clocks.  The W warm-up
steps follow, then exactly K timed steps.

Prints ONE JSON line: whole-step throughput in algorithmic GB/s, the roofline record of the
dominant kernel (the attention kernel, timed per launch with HIP events on the launch
stream; with the balanced kernel that launch is the whole paged_attention_decode call) and
the CPU oracle's throughput on the host cores as a baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3b] ...
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
METRIC = "paged-attn decode HBM GB/s (% of MI355X peak) + us per batch decode step"
WORKLOADS = {
    "cfg2": "Llama-2-7B-shape MHA decode, bf16, batch 64, 32 heads, head_dim 128, block 16, lognormal lengths",
    "cfg3": "Llama-3-8B-shape GQA decode, bf16, batch 128, 32q/8kv heads, head_dim 128, block 16, lognormal lengths <= 4096, pool 90% full",
    "cfg3b": "Llama-3-8B-shape GQA decode, bf16, batch 64, 32q/8kv heads, head_dim 128, block 16, lognormal lengths <= 4096, pool 90% full",
    "cfg4": "long-context GQA decode, bf16, batch 16, 64q/8kv heads, head_dim 128, block 16, lengths U[8192,32768]",
    "cfg5": "8B GQA decode, bf16, batch 96, 25% of sequences share prefix blocks",
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def keep_busy(torch, launch, seconds):
    """Launch `launch(i)` back to back for about `seconds` (untimed): after an idle spell the
    device needs 10-20 ms of work before its clocks have settled, and a timed region that starts
    earlier measures that transition instead of the kernels."""
    t_end, i = time.perf_counter() + seconds, 0
    while seconds > 0 and time.perf_counter() < t_end:
        for _ in range(16):
            launch(i)
            i += 1
        torch.cuda.synchronize()


def recompute_attention_detail(args, log):
    """The recompute path (paged causal prefill, the same 8B-shape heads) beside the step: causal attention
    of one preempted request of S tokens over its block list, back-to-back launches for about 20 ms after
    the clocks have settled, against the 2.5 PFLOP/s dense bf16 matrix-core peak; sampled rows are checked
    against the oracle first.  Not part of `value`."""
    import math
    import numpy as np
    import torch
    import kvc_workloads as W
    import paper_2503_13773_amd as K
    hq, hkv, d, bs = 32, 8, 128, 16
    out = {}
    for S in (2048, 4096, 16384):
        rng = np.random.default_rng(7000 + S)
        lens = np.array([S], dtype=np.int32)
        nblk = int(W.blocks_needed(lens, bs).max())
        w = W.build_workload("recompute", rng, dtype=W.BF16, context_lens=lens, num_q_heads=hq, num_kv_heads=hkv,
                             head_dim=d, block_size=bs, max_blocks_per_seq=nblk + 1, num_pool_blocks=nblk + 5)
        q_np = W.f32_to_bf16_bits(rng.standard_normal((S, hq, d)).astype(np.float32))
        q = torch.from_numpy(q_np.view(np.int16)).view(torch.bfloat16).cuda()
        kc = torch.from_numpy(w.k_cache.view(np.int16)).view(torch.bfloat16).cuda()
        vc = torch.from_numpy(w.v_cache.view(np.int16)).view(torch.bfloat16).cuda()
        tbl = torch.from_numpy(w.block_tables).cuda()
        ln = torch.from_numpy(w.context_lens).cuda()
        qs = torch.tensor([0, S], dtype=torch.int32).cuda()
        res = torch.empty_like(q)
        K.paged_attention_prefill(q, kc, vc, tbl, ln, qs, w.scale, S, res)
        torch.cuda.synchronize()
        if not args.no_check:
            import oracle
            got = res.float().cpu().numpy().astype(np.float64)
            for pos in (0, 17, S // 2 + 3, S - 1):
                ref = oracle.paged_attention_decode(q_np[pos:pos + 1], w.k_cache, w.v_cache, w.block_tables,
                                                    np.array([pos + 1], dtype=np.int32), w.scale, dtype="bf16")
                err = float(np.abs(got[pos] - ref[0]).max())
                if not err <= 2e-2:
                    log(f"[bench] recompute attention S={S}: row {pos} differs from the oracle by {err:.3e}")
                    raise SystemExit(4)
        flops = 4.0 * d * hq * S * (S + 1) / 2
        launch = lambda i=0: K.paged_attention_prefill(q, kc, vc, tbl, ln, qs, w.scale, S, res)
        keep_busy(torch, launch, args.clock_ramp_ms * 1e-3)
        n = max(5, int(0.02 / (flops / 1.0e15)))  # about 20 ms of launches
        best = float("inf")
        for _ in range(3):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(n):
                launch()
            b.record()
            torch.cuda.synchronize()
            best = min(best, a.elapsed_time(b) / n)
        out[str(S)] = {"us": round(best * 1e3, 1), "TFLOPs": round(flops / best / 1e9, 1),
                       "frac_of_mfma_peak": round(flops / best / 1e9 / 2500.0, 4)}
    log("[bench] recompute attention (one request, per layer): " +
        ", ".join(f"S={k}: {v['us']} us = {v['TFLOPs']} TFLOP/s ({100 * v['frac_of_mfma_peak']:.1f} %)" for k, v in out.items()))
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="cfg3b", choices=sorted(WORKLOADS))
    ap.add_argument("--kernel", type=int, default=0, help="0 auto, 1 VALU, 2 MFMA fixed partitions, 3 same with LDS-staged K, 4 MFMA balanced")
    ap.add_argument("--partition-tokens", type=int, default=0)
    ap.add_argument("--block-size", type=int, default=16, help="tokens per KV block (the configs use 16)")
    ap.add_argument("--num-seqs", type=int, default=0, help="override the batch size of the workload (0 = as named)")
    ap.add_argument("--replica-bytes", type=float, default=2.2e9,
                    help="rotate over replicas of the batch totalling at least this many KV bytes")
    ap.add_argument("--swap-frac", type=float, default=0.20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-check", action="store_true", help="skip the oracle check before timing (A/B timing runs)")
    ap.add_argument("--no-recompute", action="store_true",
                    help="skip the recompute (paged causal prefill) timing that goes into detail.recompute_attention")
    ap.add_argument("--cpu-threads", type=int, default=0)
    ap.add_argument("--clock-ramp-ms", type=float, default=30.0,
                    help="untimed back-to-back launches for this long before each warm-up (0: none)")
    args = ap.parse_args()

    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              f"--gpus {args.gpus} is not supported, use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np

    oracle = None
    if not (args.no_cpu_baseline and args.no_check):
        import oracle          # test infrastructure: the check before timing and the cpu_baseline leg only
        oracle.build()         # compiles only when missing or stale, and before the GPU is touched

    import torch

    import kvc_workloads as W
    import paper_2503_13773_amd as K

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    lib = K.lib()

    t0 = time.time()
    w = W.make_config(args.workload, block_size=args.block_size, **({"num_seqs": args.num_seqs} if args.num_seqs else {}))
    log(f"[bench] workload {args.workload}: {w.num_seqs} seqs, mean ctx {w.context_lens.mean():.0f}, "
        f"max {w.max_context_len}, pool {w.num_pool_blocks} blocks, KV {w.kv_bytes()/1e6:.1f} MB "
        f"(generated in {time.time()-t0:.1f}s)")

    # ---- swap-out plan: ceil(frac * batch) sequences, all their blocks, K and V planes ----
    rng = np.random.default_rng(4242)
    nblk = W.blocks_needed(w.context_lens, w.block_size)
    victims = sorted(int(s) for s in rng.permutation(w.num_seqs)[:int(math.ceil(args.swap_frac * w.num_seqs))])
    src_ids = np.unique(np.concatenate([w.block_tables[s, :nblk[s]] for s in victims])).astype(np.int64)
    pool2_blocks = int(len(src_ids))
    mapping_np = np.stack([src_ids, rng.permutation(pool2_blocks).astype(np.int64)], axis=1)
    block_bytes = w.block_bytes()
    copy_bytes = 2 * 2 * len(src_ids) * block_bytes          # read + write, K and V planes
    attn_bytes = w.kv_bytes() + w.qo_bytes()                 # K+V once, q in, out
    step_bytes = attn_bytes + copy_bytes

    # ---- device replicas ----
    def dev_bf16(a):
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)

    pool_np = np.stack([w.k_cache, w.v_cache])                # [2][NB][Hkv][Bs][D]
    n_rep = max(2, int(math.ceil(args.replica_bytes / max(1, w.kv_bytes()))))
    base_pool = dev_bf16(pool_np)
    base = dict(q=dev_bf16(w.q), tables=torch.from_numpy(w.block_tables).cuda(),
                lens=torch.from_numpy(w.context_lens).cuda(),
                mapping=torch.from_numpy(mapping_np).cuda())
    desc = K.attn_desc(base["q"], base_pool[0], base["tables"], max_context_len=w.max_context_len,
                       partition_tokens=args.partition_tokens, kernel=args.kernel)
    plan = K.attn_plan(desc)
    ws_bytes = K.workspace_bytes(desc)
    reps = []
    for r in range(n_rep):
        pool1 = base_pool if r == 0 else base_pool.clone()
        rep = dict(pool1=pool1, k=pool1[0], v=pool1[1],
                   q=base["q"].clone(), tables=base["tables"], lens=base["lens"],
                   mapping=base["mapping"], out=torch.empty_like(base["q"]),
                   ws=K.new_workspace(desc),
                   pool2=torch.zeros((2, pool2_blocks) + tuple(pool1.shape[2:]), dtype=pool1.dtype,
                                     device="cuda"))
        rep["src_pool"] = K.pool_of(rep["pool1"])
        rep["dst_pool"] = K.pool_of(rep["pool2"])
        reps.append(rep)
    torch.cuda.synchronize()
    log(f"[bench] {n_rep} replicas, plan: kernel {plan.kernel}, partition {plan.partition_tokens} tokens, "
        f"partial grid {plan.partial_grid}, merge grid {plan.merge_grid}, workspace {ws_bytes/1e6:.1f} MB; "
        f"swap {len(victims)} seqs / {len(src_ids)} blocks")

    import ctypes
    stream = torch.cuda.current_stream()
    sh = int(stream.cuda_stream)
    dref = ctypes.byref(desc)

    def attn(rep):
        rc = lib.kvc_paged_attention_decode(rep["q"].data_ptr(), rep["k"].data_ptr(), rep["v"].data_ptr(),
                                            rep["tables"].data_ptr(), rep["lens"].data_ptr(), w.scale,
                                            rep["out"].data_ptr(), dref, rep["ws"].data_ptr(), ws_bytes, sh)
        assert rc == 0, K.status_string(rc)

    def partial(rep):
        rc = lib.kvc_paged_attention_decode_partial(rep["q"].data_ptr(), rep["k"].data_ptr(), rep["v"].data_ptr(),
                                                    rep["tables"].data_ptr(), rep["lens"].data_ptr(), w.scale,
                                                    rep["out"].data_ptr(), dref, rep["ws"].data_ptr(), ws_bytes, sh)
        assert rc == 0, K.status_string(rc)

    # the same attention from a schedule built once per iteration (what the layers of a model share)
    sched = None
    if K.schedule_bytes(desc) > 0:
        sched = K.attn_schedule_build(base["tables"], base["lens"], desc)
        sched_bytes = sched.numel()

    def attn_scheduled(rep):
        rc = lib.kvc_paged_attention_decode_scheduled(rep["q"].data_ptr(), rep["k"].data_ptr(), rep["v"].data_ptr(),
                                                      sched.data_ptr(), sched_bytes, w.scale, rep["out"].data_ptr(),
                                                      dref, rep["ws"].data_ptr(), ws_bytes, sh)
        assert rc == 0, K.status_string(rc)

    def build_schedule(rep):
        rc = lib.kvc_attn_schedule_build(rep["tables"].data_ptr(), rep["lens"].data_ptr(), dref, sched.data_ptr(),
                                         sched_bytes, sh)
        assert rc == 0, K.status_string(rc)

    def copy(rep):
        rc = lib.kvc_kv_block_copy(ctypes.byref(rep["src_pool"]), ctypes.byref(rep["dst_pool"]),
                                   rep["mapping"].data_ptr(), len(src_ids), sh)
        assert rc == 0, K.status_string(rc)

    def step(rep):
        attn(rep)
        copy(rep)

    # ---- check before timing: every replica runs one step; attention rows of the first and
    # last replica against the oracle, the swapped-out blocks of the last bit for bit ----
    for rep in reps:
        step(rep)
    torch.cuda.synchronize()
    if not args.no_check:
        crng = np.random.default_rng(99)
        order = np.argsort(w.context_lens)
        seqs = sorted(set(int(x) for x in order[:2]) | set(int(x) for x in order[-2:]) |
                      set(int(x) for x in crng.integers(0, w.num_seqs, 12)))
        rows = [(sq, h) for sq in seqs for h in range(w.num_q_heads)]
        ref = oracle.attention_of_workload(w, rows=rows, num_threads=min(8, os.cpu_count() or 1))
        for rep in (reps[0], reps[-1]):
            got = rep["out"].float().cpu().numpy().astype(np.float64)
            err = max(float(np.abs(got[sq, h] - ref[sq, h]).max()) for sq, h in rows)
            if not (err <= 2e-2):
                print(f"bench.py: attention differs from the oracle (max abs err {err:.3e} > 2e-2)", file=sys.stderr)
                return 4
        want2 = np.zeros((2, pool2_blocks) + pool_np.shape[2:], dtype=np.uint16)
        oracle.kv_block_copy(pool_np, want2, mapping_np)
        got2 = reps[-1]["pool2"].view(torch.int16).cpu().numpy().view(np.uint16)
        if not np.array_equal(got2, want2):
            print("bench.py: swapped-out blocks differ from the oracle copy", file=sys.stderr)
            return 4
        log(f"[bench] check before timing: {len(rows)} attention rows within 2e-2 of the oracle (max abs err {err:.2e}), "
            f"{len(src_ids)} swapped blocks bit-exact")

    ramp_s = args.clock_ramp_ms * 1e-3

    def timed_wall(fn, steps, warmup):
        keep_busy(torch, lambda i: fn(reps[i % n_rep]), ramp_s)
        for i in range(warmup):
            fn(reps[i % n_rep])
        torch.cuda.synchronize()
        t = time.perf_counter()
        for i in range(steps):
            fn(reps[i % n_rep])
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / steps

    def timed_region(fn, steps, warmup):
        """Average duration of one fn launch: HIP events on the launch stream around `steps`
        back-to-back launches."""
        keep_busy(torch, lambda i: fn(reps[i % n_rep]), ramp_s)
        for i in range(warmup):
            fn(reps[i % n_rep])
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record(stream)
        for i in range(steps):
            fn(reps[i % n_rep])
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e-3 / steps

    def timed_events(fn, steps, warmup, hot=False):
        """Duration of single fn launches, HIP events on the launch stream around each call
        (includes the event overhead of a few microseconds)."""
        pick = (lambda i: reps[0]) if hot else (lambda i: reps[i % n_rep])
        keep_busy(torch, lambda i: fn(pick(i)), ramp_s)
        for i in range(warmup):
            fn(pick(i))
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(steps)]
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(ev):
            a.record(stream)
            fn(pick(i))
            b.record(stream)
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) * 1e-3 for a, b in ev)
        return sum(ts) / len(ts), ts[len(ts) // 2], ts[len(ts) // 10], ts[(9 * len(ts)) // 10]

    K_, W_ = args.steps, args.warmup
    step_s = timed_wall(step, K_, W_)                      # the headline: exactly K steps, wall clock
    attn_avg, attn_med, attn_p10, attn_p90 = timed_events(attn, K_, W_)
    part_pair_avg, part_med, _, _ = timed_events(partial, K_, W_)
    part_avg = timed_region(partial, K_, W_)
    attn_region = timed_region(attn, K_, W_)
    copy_region = timed_region(copy, K_, W_)
    copy_avg, copy_med, _, _ = timed_events(copy, K_, W_)
    hot_avg, hot_med, _, _ = timed_events(attn, K_, W_, hot=True)
    sched_region = sched_build = None
    if sched is not None:
        sched_region = timed_region(attn_scheduled, K_, W_)
        sched_build = timed_region(build_schedule, min(K_, 100), 10)
        if not args.no_check:   # same bits as the stateless call on the same replica
            attn(reps[0]); a_bits = reps[0]["out"].view(torch.int16).clone()
            attn_scheduled(reps[0]); torch.cuda.synchronize()
            if not torch.equal(a_bits, reps[0]["out"].view(torch.int16)):
                print("bench.py: scheduled attention differs from the stateless call", file=sys.stderr)
                return 4
        log(f"[bench] attention from a prebuilt schedule {sched_region*1e6:.1f} us back-to-back "
            f"({100.0 * attn_bytes / sched_region / 1e9 / HBM_PEAK_GBS:.1f} % of peak); building the schedule "
            f"{sched_build*1e6:.1f} us, once per iteration")
    log(f"[bench] step {step_s*1e6:.1f} us | attention avg {attn_avg*1e6:.1f} med {attn_med*1e6:.1f} us "
        f"(hot {hot_med*1e6:.1f}) | partial kernel {part_avg*1e6:.1f} us back-to-back, {part_pair_avg*1e6:.1f} us "
        f"event pairs | attention back-to-back {attn_region*1e6:.1f} us | copy avg {copy_avg*1e6:.1f} us, "
        f"back-to-back {copy_region*1e6:.1f} us")

    # ---- CPU baseline: the oracle as it stands, on the host cores, same inputs ----
    cpu = None
    if not args.no_cpu_baseline:
        threads = args.cpu_threads or min(oracle.num_threads_available(), os.cpu_count() or 1)
        h2 = np.zeros((2, pool2_blocks) + pool_np.shape[2:], dtype=np.uint16)
        # bounded sample: whole steps of the same batch, repeated until ~10 s of CPU time
        t_cpu, passes = 0.0, 0
        while True:
            t = time.perf_counter()
            oracle.attention_of_workload(w, num_threads=threads)
            oracle.kv_block_copy(pool_np, h2, mapping_np)
            t_cpu += time.perf_counter() - t
            passes += 1
            if t_cpu >= 10.0 or t_cpu + t_cpu / passes > 30.0:
                break
        cpu_s = t_cpu / passes
        # the same step on one thread (a few passes, about 2 s)
        t1, n1 = 0.0, 0
        while t1 < 2.0 and n1 < 20:
            t = time.perf_counter()
            oracle.attention_of_workload(w, num_threads=1)
            oracle.kv_block_copy(pool_np, h2, mapping_np)
            t1 += time.perf_counter() - t
            n1 += 1
        model = ""
        try:
            with open("/proc/cpuinfo") as f:
                model = next((l.split(":", 1)[1].strip() for l in f if l.startswith("model name")), "")
        except OSError:
            pass
        cpu = {"value": round(step_bytes / cpu_s / 1e9, 4), "unit": "GB/s", "cores": int(threads),
               "kind": "oracle", "sample": f"{passes} full step(s) of the same batch ({w.num_seqs} seqs x "
               f"{w.num_q_heads} heads fp64 attention + {len(src_ids)}-block memcpy copy), "
               f"{cpu_s:.2f} s per step", "s_per_step": round(cpu_s, 4),
               "single_thread_s_per_step": round(t1 / n1, 4), "cpu_model": model, "os_cpu_count": os.cpu_count()}
        log(f"[bench] cpu oracle: {cpu_s:.3f} s/step on {threads} threads, {t1 / n1:.3f} s/step on 1 thread ({model})")

    # ---- measured HBM traffic of the dominant kernel, if a rocprofv3 --pmc summary is committed ----
    traffic = None
    tfile = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tfile):
        try:
            with open(tfile) as f:
                t = json.load(f)
            key = f"{args.workload}:kernel{plan.kernel}:pt{plan.partition_tokens}"
            if key in t:
                traffic = t[key]["bytes_per_launch"]
        except Exception:
            traffic = None

    recompute = None if args.no_recompute else recompute_attention_detail(args, log)

    part_bytes = attn_bytes  # what one launch of the attention kernel must move (K+V once, q, out; partials not counted)
    achieved = part_bytes / part_avg / 1e9
    value = step_bytes / step_s / 1e9
    result = {
        "metric": METRIC, "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": K_,
        "warmup": W_, "ms_per_step": round(step_s * 1e3, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {WORKLOADS[args.workload]}",
                   "batch": w.num_seqs, "num_q_heads": w.num_q_heads, "num_kv_heads": w.num_kv_heads,
                   "head_dim": w.head_dim, "block_size": w.block_size,
                   "mean_context_len": round(float(w.context_lens.mean()), 1),
                   "max_context_len": w.max_context_len,
                   "step": "paged_attention_decode (" + ("one launch" if plan.merge_grid == 0 else "partial + merge launches") + ") + kv_block_copy swap-out of "
                           f"{len(victims)} sequences ({len(src_ids)} blocks, K and V planes)",
                   "replicas": n_rep, "kernel": int(plan.kernel),
                   "partition_tokens": int(plan.partition_tokens)},
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "detail": {
            "step_bytes": int(step_bytes), "attention_bytes": int(attn_bytes), "copy_bytes": int(copy_bytes),
            "clock_ramp_ms": args.clock_ramp_ms,
            "attention_us_back_to_back": round(attn_region * 1e6, 2),
            "copy_us_back_to_back": round(copy_region * 1e6, 2),
            "partial_kernel_us_event_pairs": round(part_pair_avg * 1e6, 2),
            "attention_us": round(attn_avg * 1e6, 2), "attention_us_median": round(attn_med * 1e6, 2),
            "attention_us_p10": round(attn_p10 * 1e6, 2), "attention_us_p90": round(attn_p90 * 1e6, 2),
            "attention_GBs": round(attn_bytes / attn_avg / 1e9, 1),
            "attention_pct_of_peak": round(100.0 * attn_bytes / attn_avg / 1e9 / HBM_PEAK_GBS, 2),
            "attention_us_hot_same_replica": round(hot_med * 1e6, 2),
            "tokens_per_s": round(w.num_seqs / attn_avg, 1),
            "copy_us": round(copy_avg * 1e6, 2), "copy_GBs": round(copy_bytes / copy_avg / 1e9, 1),
            "attention_pct_of_peak_back_to_back": round(100.0 * attn_bytes / attn_region / 1e9 / HBM_PEAK_GBS, 2),
            "attention_scheduled_us_back_to_back": None if sched_region is None else round(sched_region * 1e6, 2),
            "attention_scheduled_pct_of_peak_back_to_back":
                None if sched_region is None else round(100.0 * attn_bytes / sched_region / 1e9 / HBM_PEAK_GBS, 2),
            "schedule_build_us": None if sched_build is None else round(sched_build * 1e6, 2),
            "recompute_attention": recompute,
        },
        "roofline": {"bound": "hbm", "kernel": {1: "pa_partial_valu_kernel", 2: "pa_partial_mfma_kernel", 3: "pa_partial_mfma_kernel", 4: "pa_stream_mfma_kernel"}[int(plan.kernel)],
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "bytes_per_launch": int(part_bytes), "avg_launch_us": round(part_avg * 1e6, 2),
                     "covers": "whole paged_attention_decode call" if plan.merge_grid == 0 else "partial kernel only (a merge launch follows)"},
        "cpu_baseline": cpu,
    }
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
