// Load-balanced persistent partial kernel of paged decode attention on the matrix cores
// (gfx950, bf16, head_dim 128, block_size >= 4, group <= 16, <= 4096 sequences).
//
// The serving traces this path sees have heavily skewed context lengths (a lognormal mix:
// median ~700 tokens, tail to 4096), and the whole batch is only ~30 us of HBM streaming.
// Fixed-length partitions then lose to per-workgroup start-up latency, idle workgroups and
// a ragged tail.  Here instead the work is flattened and cut into equal pieces:
//
//   rows  = (sequence n, KV head g), each with t_n = ceil(context_len_n / 16) tiles
//   flat  = [row 0 tiles][row 0 cost][row 1 tiles][row 1 cost]...
//           T = num_kv_heads * sum_n (t_n + kRowCost) units in all
//   every WAVEFRONT of the grid is a worker that takes C = max(C_min, ceil(T / workers))
//   consecutive flat units.
// The kRowCost units after a row's tiles stand for the work of leaving the row (writing the
// segment, switching the softmax state, loading the next Q: measured at about half a tile's
// time each; a worker that crossed 9 short rows finished 6 us after the rest); nothing is
// computed for them, they only make a worker that crosses rows take fewer tiles.
//
// The grid is ONE wavefront per SIMD (256 CUs x 4).  Measured on MI355X: with 2 or 3
// wavefronts per SIMD the older wavefronts win the memory-issue arbitration, the younger
// ones starve until the older exit, and the kernel ends with a long, thinly populated
// tail; one wavefront per SIMD with its loads kept in flight across row changes streams at
// the same rate and all workers finish within a few percent of each other.
//
// A worker's range may start and end inside a row; each (row, tile range) it covers is a
// "segment".  A segment that is a whole row is normalised and written to `out`; otherwise
// the worker writes (max, sum, accumulator) to partial slot (worker - first worker of the
// row), and the worker that owns tile 0 of a row records how many partials the row has.  The
// merge kernel reads that count.  Wavefronts never synchronise with each other after the
// start-up prefix sum, and every loop is bounded by the worker's static range, so every
// wavefront exits.
//
// The worker's tiles form one continuous stream, software-pipelined over two register sets:
// the loads of tile i+1 are issued before tile i is consumed, also when tile i+1 belongs to
// the next row.  An "issue cursor" (row, tile, block ids) runs one tile ahead of the
// "compute cursor" (row, tile, softmax state, Q operand); block ids and the Q operand of
// the row after the current one are prefetched when a cursor enters a row, so a row change
// costs no dependent-load bubble.
//
// Start-up (once per workgroup): prefix sum of t_n over the batch in LDS (<= 4096 sequences),
// then a binary search places each worker.  Per tile the arithmetic is pa_mfma_tile.h.
#include <math.h>

#include "kvc_internal.h"
#include "pa_mfma_tile.h"

namespace kvc {

namespace {

using namespace mfma;

__device__ inline int uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }

constexpr int kStageTiles = 256;  // tiles whose addresses are staged in LDS per wavefront at a time
constexpr int kMaxUnits = 4;      // a 16-token tile spans up to 4 blocks (block_size 4)
constexpr int kRowCost = 1;       // flat units charged for leaving a row

// A row of the flattened work: (sequence, KV head); all fields wavefront-uniform.
struct RowCursor {
    int n;       // sequence
    int kvh;     // KV head
    int pref;    // flat units (per KV head) of all sequences before n
    int tiles;   // t_n (the row spans t_n + kRowCost flat units)
};

// MAXSPT: sequences per thread in the start-up prefix sum (batches up to MAXSPT * 256 sequences);
// the small instance keeps the start-up of ordinary batches short.
template <int MAXSPT>
__global__ __launch_bounds__(kThreads, 1) void pa_stream_mfma_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k_cache,
    const uint16_t *__restrict__ v_cache, const int32_t *__restrict__ block_tables,
    const int32_t *__restrict__ context_lens, uint16_t *__restrict__ out, Workspace ws,
    AttnParams p, int unit_log2, int units_per_block_log2) {
    constexpr int kSeqs = MAXSPT * kThreads;
    __shared__ int s_pref[kSeqs + 2];  // exclusive prefix of flat units (tiles + row cost) per sequence (+ guard)
    __shared__ int s_ctx[kSeqs];       // context length per sequence
    __shared__ int s_wave_tot[kWaves];
    __shared__ int s_tile[kWaves][kStageTiles * kMaxUnits];  // per worker: pool index of each unit of its next tiles

    const int tid = threadIdx.x;
    const int wave = uniform(tid >> 6), lane = tid & 63;
    const int quad = lane >> 4, r = lane & 15;
    const int nseq = p.num_seqs;

    // ---- prefix sum of 16-token tiles per sequence (thread t owns sequences t*spt .. +spt-1)
    {
        constexpr int kMaxSpt = MAXSPT;
        const int spt = (nseq + kThreads - 1) / kThreads;  // <= kMaxSpt
        int local[kMaxSpt], sum = 0;
#pragma unroll
        for (int i = 0; i < kMaxSpt; ++i) {
            const int n = tid * spt + i;
            int t = 0;
            if (i < spt && n < nseq) {
                const int c = max(context_lens[n], 0);
                s_ctx[n] = c;
                t = (c + kTileTokens - 1) >> 4;
                if (t > 0) t += kRowCost;
            }
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
        for (int i = 0; i < kMaxSpt; ++i) {
            const int n = tid * spt + i;
            if (i < spt && n < nseq) s_pref[n] = excl + local[i];
        }
        if (tid == kThreads - 1) {
            s_pref[nseq] = excl + sum;
            s_pref[nseq + 1] = excl + sum + 1 + kRowCost;  // guard: "sequence nseq" looks non-empty, stops row walks
        }
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
    const int f1 = min(T, f0 + C);       // the worker's flat units are [f0, f1)


    // Row after `c` in flat order, skipping empty sequences.  Past the last row it parks on
    // the guard entry (n == nseq), which is never dereferenced: a cursor only moves there
    // when the worker has no tile left.
    auto next_row = [&](const RowCursor &c) __attribute__((always_inline)) {
        RowCursor o = c;
        if (o.n < nseq && ++o.kvh == Hkv) {
            o.kvh = 0;
            do { ++o.n; } while (uniform(s_pref[o.n + 1]) == uniform(s_pref[o.n]));
            o.pref = uniform(s_pref[o.n]);
            o.tiles = uniform(s_pref[o.n + 1]) - o.pref - kRowCost;
        }
        return o;
    };
    auto load_q = [&](bf16x8(&qb)[4], const RowCursor &c) __attribute__((always_inline)) {
        const bool active = r < G && c.n < nseq;
        const int n = c.n < nseq ? c.n : 0;
        load_q_operand(qb, q + (size_t(n) * p.num_q_heads + c.kvh * G + (r < G ? r : 0)) * D, quad, active);
    };

    // ---- place the worker: largest n with s_pref[n] * Hkv <= f0 (that sequence is not empty)
    RowCursor first;
    int first_tile;
    {
        int lo = 0, hi = nseq;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (uniform(s_pref[mid]) * Hkv <= f0) lo = mid; else hi = mid;
        }
        first.n = lo;
        first.pref = uniform(s_pref[lo]);
        const int units = uniform(s_pref[lo + 1]) - first.pref;  // per KV head
        first.tiles = units - kRowCost;
        first.kvh = (f0 - first.pref * Hkv) / units;
        first_tile = (f0 - first.pref * Hkv) - first.kvh * units;
        if (first_tile >= first.tiles) {  // the range starts in the row's cost units: begin with the next row
            first = next_row(first);
            first_tile = 0;
        }
    }
    // tiles of this worker: the part of [f0, f1) that falls on tiles rather than cost units
    int NT = 0;
    {
        RowCursor c = first;
        int t0 = first_tile;
        while (c.n < nseq) {
            const int row0 = c.pref * Hkv + c.kvh * (c.tiles + kRowCost);  // flat unit of the row's tile 0
            if (row0 + t0 >= f1) break;
            NT += min(row0 + c.tiles, f1) - (row0 + t0);
            if (row0 + c.tiles + kRowCost >= f1) break;
            c = next_row(c);
            t0 = 0;
        }
    }
    if (NT == 0) return;  // the range covered cost units only; no row counts this worker

    // ---- tile addresses of the worker's range, staged in LDS
    // A "unit" is the part of a 16-token tile that lies in one block: min(block_size, 16)
    // tokens, so a tile is U = 1, 2 or 4 units.  Entry (k, u) holds the index, in units, of
    // unit u of the worker's k-th tile inside the KV pools:
    //   (block * Hkv + kv head) * units_per_block + unit-in-block.
    // Units past the end of the context (ragged last tile, blocks never allocated) repeat the
    // last valid unit: they are loaded and masked, never taken from the block table.
    // Staging the addresses up front keeps the steady-state loop free of dependent
    // block-table loads: the issue side needs two LDS reads per tile and no row bookkeeping.
    const int U_log2 = 4 - unit_log2;                 // log2(units per tile)
    const int unit_tokens = 1 << unit_log2;
    const int upb_mask = (1 << units_per_block_log2) - 1;
    RowCursor rf = first;           // fill cursor
    int tf = first_tile;            // next tile of row rf to stage
    int staged_base = 0;            // worker-relative index of the first staged tile
    auto stage_tiles = [&](int from) __attribute__((always_inline)) {
        const int count = min(kStageTiles, NT - from);
        int off = 0;
        while (off < count) {
            if (tf == rf.tiles) {
                rf = next_row(rf);
                tf = 0;
            }
            if (rf.n >= nseq) break;  // cannot happen for a consistent batch; never walk past the last row
            const int seg = min(rf.tiles - tf, count - off);  // >= 1
            const int32_t *table = block_tables + size_t(rf.n) * p.max_blocks_per_seq;
            const int last_unit = ((uniform(s_ctx[rf.n]) + unit_tokens - 1) >> unit_log2) - 1;
            for (int e = lane; e < (seg << U_log2); e += 64) {
                const int unit = min(((tf << U_log2) + e), last_unit);   // unit index within the row
                const int blk = table[unit >> units_per_block_log2];
                s_tile[wave][(off << U_log2) + e] =
                    ((blk * Hkv + rf.kvh) << units_per_block_log2) + (unit & upb_mask);
            }
            off += seg;
            tf += seg;
        }
        staged_base = from;
    };
    stage_tiles(0);

    // Per-lane constants of the tile loads: K wants token r, V wants tokens 4*quad + i.
    const size_t unit_elems = size_t(unit_tokens) * D;
    const int k_unit = r >> unit_log2, k_row = r & (unit_tokens - 1);
    const int v_unit = (4 * quad) >> unit_log2, v_row = (4 * quad) & (unit_tokens - 1);
    const uint16_t *k_lane = k_cache + k_row * D + 8 * quad;
    const uint16_t *v_lane = v_cache + v_row * D + 8 * r;

    int ki = 0;  // worker-relative index of the next tile to load
    auto issue_next = [&](uint4(&kr)[4], uint4(&vr)[4]) __attribute__((always_inline)) {
        if (ki - staged_base == kStageTiles) stage_tiles(ki);  // very long ranges only
        const int *e = &s_tile[wave][(ki - staged_base) << U_log2];
        const uint16_t *kp = k_lane + size_t(e[k_unit]) * unit_elems;
        const uint16_t *vp = v_lane + size_t(e[v_unit]) * unit_elems;
#pragma unroll
        for (int j = 0; j < 4; ++j) kr[j] = load16_stream(kp + 32 * j);
#pragma unroll
        for (int i = 0; i < 4; ++i) vr[i] = load16_stream(vp + i * D);
        ++ki;
    };

    // ---- compute cursor
    RowCursor rc = first;
    int tc = first_tile;             // next tile of row rc to consume
    int seg_first = first_tile;      // first tile of the current segment
    int ctx_c = uniform(s_ctx[rc.n]);
    bf16x8 qb[4], qb_next[4];
    load_q(qb, rc);
    load_q(qb_next, next_row(rc));
    HeadState st;
    st.reset();

    // Write the finished segment [seg_first, tc) of row rc.
    auto finalize = [&]() __attribute__((always_inline)) {
        st.finish();
        const int row_f = rc.pref * Hkv + rc.kvh * (rc.tiles + kRowCost);  // flat unit of the row's tile 0
        const int j0 = row_f / C;
        const int cnt = (row_f + rc.tiles - 1) / C - j0 + 1;  // workers that touch this row
        const int slot = worker - j0;                         // my partial index within the row
        if (r < G) {  // lane (quad, r) holds O[head r][32*quad .. +31]
            const size_t orow = size_t(rc.n) * p.num_q_heads + rc.kvh * G + r;
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
        if (seg_first == 0 && lane == 0) ws.cnt[rc.n * Hkv + rc.kvh] = cnt;
    };

    // Consumes the tile under the compute cursor.  When it was the last tile of the row the
    // segment is written and the state switches to the next row at once: the stores and the
    // Q prefetch are then issued as early as possible before the next wait on tile data.
    auto compute_next = [&](uint4(&kr)[4], uint4(&vr)[4], bool more) __attribute__((always_inline)) {
        bf16x8 ka[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) ka[j] = __builtin_bit_cast(bf16x8, kr[j]);
        compute_tile(st, ka, vr, qb, p.scale_log2e, ctx_c - tc * kTileTokens, quad);
        ++tc;
        if (tc == rc.tiles && more) {  // row finished and the worker has more tiles
            finalize();
            rc = next_row(rc);
            tc = 0;
            seg_first = 0;
            ctx_c = uniform(s_ctx[rc.n]);
            st.reset();
#pragma unroll
            for (int j = 0; j < 4; ++j) qb[j] = qb_next[j];
            load_q(qb_next, next_row(rc));
        }
    };

    // Two register sets; the steady-state loop has no branch around the tile loads, so the
    // compiler's wait counts let the newest 8 loads stay in flight while the older tile is
    // consumed.  The 1- or 2-tile tail is peeled.
    uint4 kA[4], vA[4], kB[4], vB[4];
    issue_next(kA, vA);
    int it = 0;
    for (; it + 2 < NT; it += 2) {
        issue_next(kB, vB);
        compute_next(kA, vA, true);
        issue_next(kA, vA);
        compute_next(kB, vB, true);
    }
    if (it + 1 < NT) {
        issue_next(kB, vB);
        compute_next(kA, vA, true);
        compute_next(kB, vB, false);
    } else {
        compute_next(kA, vA, false);
    }
    finalize();
}

}  // namespace

hipError_t launch_partial_mfma_stream(const void *q, const void *k_cache, const void *v_cache,
                                      const int32_t *block_tables, const int32_t *context_lens,
                                      void *out, Workspace ws, const AttnParams &p, int grid,
                                      hipStream_t stream) {
    // unit = min(block_size, 16) tokens; blocks hold block_size / unit units
    int unit_log2 = 4, upb_log2 = 0;
    if (p.block_size < 16) {
        unit_log2 = p.block_size_log2;
    } else {
        while ((16 << upb_log2) < p.block_size) ++upb_log2;
    }
    if (p.num_seqs <= 4 * kThreads)
        pa_stream_mfma_kernel<4><<<dim3(grid), dim3(kThreads), 0, stream>>>(
            static_cast<const uint16_t *>(q), static_cast<const uint16_t *>(k_cache),
            static_cast<const uint16_t *>(v_cache), block_tables, context_lens,
            static_cast<uint16_t *>(out), ws, p, unit_log2, upb_log2);
    else
        pa_stream_mfma_kernel<kMaxStreamSeqs / kThreads><<<dim3(grid), dim3(kThreads), 0, stream>>>(
            static_cast<const uint16_t *>(q), static_cast<const uint16_t *>(k_cache),
            static_cast<const uint16_t *>(v_cache), block_tables, context_lens,
            static_cast<uint16_t *>(out), ws, p, unit_log2, upb_log2);
    return hipGetLastError();
}

}  // namespace kvc
