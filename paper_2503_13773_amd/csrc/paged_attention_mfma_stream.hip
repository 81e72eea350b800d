// Load-balanced persistent partial kernel of paged decode attention on the matrix cores
// (gfx950, bf16, head_dim 128, block_size a multiple of 16, group <= 16, <= 1024 sequences).
//
// The serving traces this path sees have heavily skewed context lengths (a lognormal mix:
// median ~700 tokens, tail to 4096), and the whole batch is only ~30 us of HBM streaming.
// Fixed-length partitions then lose to per-workgroup start-up latency, idle workgroups and
// a ragged tail.  Here instead the work is flattened and cut into equal pieces:
//
//   rows  = (sequence n, KV head g), each with t_n = ceil(context_len_n / 16) tiles
//   flat  = [row 0 tiles][row 1 tiles]...   T = num_kv_heads * sum_n t_n tiles in all
//   every WAVEFRONT of the (fixed-size, one-wave-per-SIMD-slot) grid is a worker that takes
//   C = max(C_min, ceil(T / workers)) consecutive flat tiles.
//
// A worker's range may start and end inside a row; each (row, tile range) it covers is a
// "segment".  A segment that is a whole row is normalised and written to `out`; otherwise
// the worker writes (max, sum, accumulator) to partial slot (worker - first worker of the
// row), and the worker that owns tile 0 of a row records how many partials the row has.  The
// merge kernel reads that count.  Wavefronts never synchronise with each other: no LDS
// reduction, no barrier after the start-up prefix sum, and every loop is bounded by the
// worker's static range, so every wavefront exits.
//
// Start-up (once per workgroup): prefix sum of t_n over the batch in LDS (<= 1024 sequences),
// then a binary search places each worker.  Per tile the arithmetic is pa_mfma_tile.h.
#include <math.h>

#include "kvc_internal.h"
#include "pa_mfma_tile.h"

namespace kvc {

namespace {

using namespace mfma;

__device__ inline int uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }

__global__ __launch_bounds__(kThreads, 3) void pa_stream_mfma_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k_cache,
    const uint16_t *__restrict__ v_cache, const int32_t *__restrict__ block_tables,
    const int32_t *__restrict__ context_lens, uint16_t *__restrict__ out, Workspace ws,
    AttnParams p, int tiles_per_block_log2) {
    __shared__ int s_pref[kMaxStreamSeqs + 1];  // exclusive prefix of tiles per sequence
    __shared__ int s_wave_tot[kWaves];

    const int tid = threadIdx.x;
    const int wave = uniform(tid >> 6), lane = tid & 63;
    const int quad = lane >> 4, r = lane & 15;
    const int nseq = p.num_seqs;

    // ---- prefix sum of 16-token tiles per sequence (thread t owns sequences t*spt .. +spt-1)
    {
        const int spt = (nseq + kThreads - 1) / kThreads;  // <= 4
        int local[4], sum = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int n = tid * spt + i;
            int t = 0;
            if (i < spt && n < nseq) t = (max(context_lens[n], 0) + kTileTokens - 1) >> 4;
            local[i] = sum;
            sum += t;
        }
        int inc = sum;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int v = __shfl_up(inc, off);
            if (lane >= off) inc += v;
        }
        if (lane == 63) s_wave_tot[wave] = inc;
        __syncthreads();
        int base = 0;
        for (int w = 0; w < wave; ++w) base += s_wave_tot[w];
        const int excl = base + inc - sum;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int n = tid * spt + i;
            if (i < spt && n < nseq) s_pref[n] = excl + local[i];
        }
        if (tid == kThreads - 1) s_pref[nseq] = excl + sum;
        __syncthreads();
    }

    const int Hkv = p.num_kv_heads;
    const int G = p.group;
    const int T = uniform(s_pref[nseq]) * Hkv;
    const int workers = gridDim.x * kWaves;
    const int C = max(p.min_chunk_tiles, (T + workers - 1) / workers);
    const int worker = blockIdx.x * kWaves + wave;
    if (int64_t(worker) * C >= T) return;
    const int f0 = worker * C;
    const int f1 = min(T, f0 + C);

    // ---- place the worker: largest n with s_pref[n] * Hkv <= f0 (that sequence is not empty)
    int n;
    {
        int lo = 0, hi = nseq;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (uniform(s_pref[mid]) * Hkv <= f0) lo = mid; else hi = mid;
        }
        n = lo;
    }
    int pref_n = uniform(s_pref[n]);
    int t_n = uniform(s_pref[n + 1]) - pref_n;
    int kvh = (f0 - pref_n * Hkv) / t_n;
    int tile = (f0 - pref_n * Hkv) - kvh * t_n;

    const size_t head_elems = size_t(p.block_size) * D;
    const size_t block_elems = head_elems * Hkv;
    const int sub_mask = (1 << tiles_per_block_log2) - 1;

    int f = f0;
    while (f < f1) {
        // ---- one segment: tiles [ta, tb) of row (n, kvh)
        const int ta = tile;
        const int tb = min(t_n, ta + (f1 - f));
        const int ctx = uniform(context_lens[n]);
        const int row_f = pref_n * Hkv + kvh * t_n;          // flat index of the row's tile 0
        const int j0 = row_f / C;
        const int cnt = (row_f + t_n - 1) / C - j0 + 1;      // workers that touch this row
        const int slot = worker - j0;                        // my partial index within the row
        const int32_t *table = block_tables + size_t(n) * p.max_blocks_per_seq;
        const size_t head_off = size_t(kvh) * head_elems;

        bf16x8 qb[4];
        load_q_operand(qb, q + (size_t(n) * p.num_q_heads + kvh * G + (r < G ? r : 0)) * D, quad, r < G);
        HeadState st;
        st.reset();

        for (int c0 = ta; c0 < tb; c0 += 64) {
            const int nt = min(64, tb - c0);
            int my_blk = 0;  // physical block of tile c0 + lane
            if (lane < nt) my_blk = table[(c0 + lane) >> tiles_per_block_log2];

            auto issue = [&](uint4(&kr)[4], uint4(&vr)[4], int it) __attribute__((always_inline)) {
                const int blk = __builtin_amdgcn_readlane(my_blk, it);
                const size_t base = size_t(blk) * block_elems + head_off + size_t((c0 + it) & sub_mask) * kTileElems;
                issue_tile_direct(kr, vr, k_cache + base, v_cache + base, quad, r);
            };
            auto compute = [&](uint4(&kr)[4], uint4(&vr)[4], int it) __attribute__((always_inline)) {
                bf16x8 ka[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) ka[j] = __builtin_bit_cast(bf16x8, kr[j]);
                compute_tile(st, ka, vr, qb, p.scale_log2e, ctx - (c0 + it) * kTileTokens, quad);
            };

            uint4 kA[4], vA[4], kB[4], vB[4];
            issue(kA, vA, 0);
            for (int it = 0; it < nt; it += 2) {
                const bool has1 = it + 1 < nt;
                if (has1) issue(kB, vB, it + 1);
                compute(kA, vA, it);
                if (has1) {
                    if (it + 2 < nt) issue(kA, vA, it + 2);
                    compute(kB, vB, it + 1);
                }
            }
        }
        st.finish();

        // ---- write the segment: lane (quad, r < G) holds O[head r][32*quad .. +31]
        if (r < G) {
            const size_t orow = size_t(n) * p.num_q_heads + kvh * G + r;
            if (cnt == 1) {
                const float inv = 1.0f / st.l;
                uint16_t *dst = out + orow * D + 32 * quad;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    uint4 w;
                    w.x = pack_bf16(st.acc[0][i] * inv, st.acc[1][i] * inv);
                    w.y = pack_bf16(st.acc[2][i] * inv, st.acc[3][i] * inv);
                    w.z = pack_bf16(st.acc[4][i] * inv, st.acc[5][i] * inv);
                    w.w = pack_bf16(st.acc[6][i] * inv, st.acc[7][i] * inv);
                    *reinterpret_cast<uint4 *>(dst + 8 * i) = w;
                }
            } else if (slot < p.max_partitions) {
                const size_t ps = orow * p.max_partitions + slot;
                float *dst = ws.acc + ps * D + 32 * quad;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    *reinterpret_cast<float4 *>(dst + 8 * i) = float4{st.acc[0][i], st.acc[1][i], st.acc[2][i], st.acc[3][i]};
                    *reinterpret_cast<float4 *>(dst + 8 * i + 4) = float4{st.acc[4][i], st.acc[5][i], st.acc[6][i], st.acc[7][i]};
                }
                if (quad == 0) *reinterpret_cast<float2 *>(ws.ml + ps * 2) = float2{st.m, st.l};
            }
        }
        if (ta == 0 && lane == 0) ws.cnt[n * Hkv + kvh] = cnt;

        // ---- advance to the next row
        f += tb - ta;
        tile = 0;
        if (tb == t_n && f < f1) {
            if (++kvh == Hkv) {
                kvh = 0;
                do { ++n; } while (n < nseq - 1 && uniform(s_pref[n + 1]) == uniform(s_pref[n]));
                pref_n = uniform(s_pref[n]);
                t_n = uniform(s_pref[n + 1]) - pref_n;
            }
        }
    }
}

}  // namespace

hipError_t launch_partial_mfma_stream(const void *q, const void *k_cache, const void *v_cache,
                                      const int32_t *block_tables, const int32_t *context_lens,
                                      void *out, Workspace ws, const AttnParams &p, int grid,
                                      hipStream_t stream) {
    int tpb_log2 = 0;
    while ((16 << tpb_log2) < p.block_size) ++tpb_log2;
    pa_stream_mfma_kernel<<<dim3(grid), dim3(kThreads), 0, stream>>>(
        static_cast<const uint16_t *>(q), static_cast<const uint16_t *>(k_cache),
        static_cast<const uint16_t *>(v_cache), block_tables, context_lens,
        static_cast<uint16_t *>(out), ws, p, tpb_log2);
    return hipGetLastError();
}

}  // namespace kvc
