"""A decode iteration (KV append, paged attention, swap-out block copy) recorded into a HIP graph
and replayed: the library allocates nothing, never synchronises and records no memset, so its
launches can be captured.  Every replay runs on inputs rewritten in place between replays, with
eager work and synchronisations in between, and is compared with the eager result bit for bit and
with the fp64 oracle."""
import numpy as np
import pytest
import torch

import kvc_workloads as W
from gpu_util import BF16_TOL, dev_tensor, out_bits, out_to_f64

pytestmark = pytest.mark.gpu


def test_decode_iteration_graph_replays_match_eager_and_oracle(oracle_mod):
    import paper_2503_13773_amd as K
    rng = np.random.default_rng(77)
    w = W.make_config("cfg3", num_seqs=10, ctx_scale=0.4)
    nseq, hq, d = w.q.shape
    hkv, bs = w.k_cache.shape[1], w.k_cache.shape[2]
    # every sequence gets room for 3 more tokens (its table row and the pool have spare blocks)
    lens0 = w.context_lens.copy()
    nblk = W.blocks_needed(lens0 + 3, bs)
    free = sorted(set(range(w.k_cache.shape[0])) - set(int(b) for b in w.block_tables[w.block_tables >= 0]))
    for n in range(nseq):
        have = int(W.blocks_needed(lens0[n:n + 1], bs)[0])
        for j in range(have, int(nblk[n])):
            w.block_tables[n, j] = free.pop()

    pool = torch.stack([dev_tensor(w.k_cache, W.BF16), dev_tensor(w.v_cache, W.BF16)])  # planes K, V
    kc, vc = pool[0], pool[1]
    tables = torch.from_numpy(w.block_tables).cuda()
    lens = torch.from_numpy(lens0).cuda()          # rewritten before every replay
    pos = torch.full((nseq,), -1, dtype=torch.int32, device="cuda")   # the warm-up run appends nothing
    q = dev_tensor(w.q, W.BF16)
    k_new = torch.zeros((nseq, hkv, d), dtype=torch.bfloat16, device="cuda")
    v_new = torch.zeros_like(k_new)
    out = torch.empty_like(q)
    desc = K.attn_desc(q, kc, tables, max_context_len=int(lens0.max()) + 3)
    ws = K.new_workspace(desc)      # counter header zeroed once; every call leaves it zeroed, replays too
    # swap-out of the first two sequences' blocks into a second pool
    victims = [b for n in (0, 1) for b in w.block_tables[n, :int(nblk[n])]]
    pool2 = torch.zeros((2, len(victims)) + tuple(kc.shape[1:]), dtype=kc.dtype, device="cuda")
    mapping = torch.tensor([[int(b), i] for i, b in enumerate(victims)], dtype=torch.int64, device="cuda")

    def iteration():
        K.kv_cache_append(k_new, v_new, kc, vc, tables, pos)
        K.paged_attention_decode(q, kc, vc, tables, lens, w.scale, out, desc=desc, workspace=ws)
        K.kv_block_copy(pool, pool2, mapping)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        iteration()                                 # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        iteration()

    host_k, host_v = w.k_cache.copy(), w.v_cache.copy()
    for step in range(1, 4):
        new_lens = lens0 + step
        kn = W.f32_to_bf16_bits(rng.standard_normal((nseq, hkv, d)).astype(np.float32))
        vn = W.f32_to_bf16_bits(rng.standard_normal((nseq, hkv, d)).astype(np.float32))
        qn = W.f32_to_bf16_bits(rng.standard_normal((nseq, hq, d)).astype(np.float32))
        lens.copy_(torch.from_numpy(new_lens).cuda())
        pos.copy_(torch.from_numpy(new_lens - 1).cuda())
        k_new.copy_(dev_tensor(kn, W.BF16))
        v_new.copy_(dev_tensor(vn, W.BF16))
        q.copy_(dev_tensor(qn, W.BF16))
        print(f"[case] graph replay {step}", flush=True)
        graph.replay()
        torch.cuda.synchronize()
        replayed, swapped = out_bits(out).copy(), pool2.cpu().view(torch.int16).numpy().copy()
        # eager work between replays: the same iteration again (the append rewrites the same slot)
        out.zero_()
        pool2.zero_()
        iteration()
        torch.cuda.synchronize()
        assert np.array_equal(replayed, out_bits(out)), step
        assert np.array_equal(swapped, pool2.cpu().view(torch.int16).numpy()), step
        # oracle on the host copy of the cache after the same append
        oracle_mod.kv_cache_append(kn, vn, host_k, host_v, w.block_tables, (new_lens - 1).astype(np.int32))
        ref = oracle_mod.paged_attention_decode(qn, host_k, host_v, w.block_tables, new_lens.astype(np.int32),
                                                w.scale, dtype="bf16", num_threads=8)
        got = W.bf16_bits_to_f32(replayed.view(np.uint16)).astype(np.float64)
        assert np.abs(got - ref).max() <= BF16_TOL, step
        for i, b in enumerate(victims):
            assert np.array_equal(swapped[0, i].view(np.uint16), host_k[b]) and \
                np.array_equal(swapped[1, i].view(np.uint16), host_v[b]), (step, i)
