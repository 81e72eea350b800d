// Load-balanced persistent kernel of paged decode attention on the matrix cores, one launch
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
// "segment".  A segment that is a whole row is normalised and written to `out`.  Otherwise it
// is a partial (max, sum, accumulator) of a cut row: the H partial when the segment does not
// start at the row's tile 0 (only a worker's first segment can), the T partial when it starts
// at tile 0 but stops before the row ends (only its last segment can).  A row cut over workers
// j0 .. j0+cnt-1 therefore has its partials in T[j0], H[j0+1], ..., H[j0+cnt-1], and the
// workspace needs two partial slots per worker whatever the batch looks like.
//
// Cut rows are finished inside this kernel, with no second launch.  Which rows a worker holds
// a piece of follows from its placement alone.  Per cut row there is one counter word (indexed
// by j0: a worker is the first of at most one cut row; arrivals in the lower half of the word,
// publications in the upper half).  A worker
//   1. announces its arrival (adds 1 to the word of each of its cut rows) right after it has
//      issued the loads of its last tile, so the counter's answer travels while the last one or
//      two tiles are consumed; the H partial was parked in registers meanwhile;
//   2. where the add returned cnt-1 it is the last to arrive and finishes the row: it waits
//      until the upper half shows the other cnt-1 pieces published (a poll, usually short),
//      fetches them with device-scope loads, merges all cnt partials in slot order by the
//      log-sum-exp rule (its own from registers: the same values its slot would hold, so the
//      result does not depend on who arrived last), writes `out` and resets the word to 0;
//   3. elsewhere it writes its partial to its slot with device-scope stores, waits for them to
//      complete and adds 0x10000 (published).
// The only wait on another wavefront is the poll in 2: the wavefronts polled for have already
// arrived, which they do one or two tiles before the end of their range; what they have left
// (those tiles, their stores, one add) needs nothing from anyone, so the poll ends.  The
// counter words must be 0 when the kernel starts and are 0 again when it ends.
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

// Partials cross from one wavefront to another inside a launch, between XCDs whose L2 caches
// are not coherent with each other.  They are therefore written and read with device-scope
// accesses (the sc1 cache policy: each access goes to the point of coherence of the whole
// device by itself), 16 bytes per lane, through raw buffer instructions, instead of ordinary
// stores followed by a write-back of the whole L2: that write-back, issued by 1024 wavefronts,
// doubled the kernel time when it was measured.
constexpr int kDeviceScope = 16;  // cache-policy operand of the buffer builtins: sc1
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
__device__ inline __amdgpu_buffer_rsrc_t raw_buffer(const void *base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}
__device__ inline void store4_device_scope(__amdgpu_buffer_rsrc_t b, uint32_t byte_off, float x, float y, float z, float w) {
    const u32x4 v = {__float_as_uint(x), __float_as_uint(y), __float_as_uint(z), __float_as_uint(w)};
    __builtin_amdgcn_raw_buffer_store_b128(v, b, byte_off, 0, kDeviceScope);
}
__device__ inline float4 load4_device_scope(__amdgpu_buffer_rsrc_t b, uint32_t byte_off) {
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(b, byte_off, 0, kDeviceScope);
    return float4{__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w)};
}
__device__ inline void store2_device_scope(__amdgpu_buffer_rsrc_t b, uint32_t byte_off, float x, float y) {
    const u32x2 v = {__float_as_uint(x), __float_as_uint(y)};
    __builtin_amdgcn_raw_buffer_store_b64(v, b, byte_off, 0, kDeviceScope);
}
__device__ inline float2 load2_device_scope(__amdgpu_buffer_rsrc_t b, uint32_t byte_off) {
    const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(b, byte_off, 0, kDeviceScope);
    return float2{__uint_as_float(v.x), __uint_as_float(v.y)};
}

constexpr int kStageTiles = 256;  // tiles whose addresses are staged in LDS per wavefront at a time
constexpr int kMaxUnits = 4;      // a 16-token tile spans up to 4 blocks (block_size 4)
constexpr int kRowCost = 1;       // flat units charged for leaving a row
static_assert(size_t(kNumCUs) * kWaves * sizeof(int32_t) <= kWorkspaceHeaderBytes,
              "one arrival counter per worker must fit the workspace header");

// ---- finishing cut rows --------------------------------------------------------------------
// A cut row as seen by the worker that arrived last at it.
struct CutRow {
    bool active;
    int n, kvh;   // sequence, KV head
    int j0, cnt;  // first worker of the row, number of workers on it
    int own;      // which of the cnt partials is this worker's own
};


// Partial slot layout (fp32): [8 vectors][quad][head][4]; vector v of (quad, head) = dims
// 32*quad + 4v .. +3 of the head's accumulator; (max, sum) per head in a second array.  One
// store or load instruction of a wavefront then covers whole 128-byte lines.  Offsets in bytes.
__device__ inline uint32_t slot_vec(int slot, int G, int v, int quad, int head) {
    return (uint32_t(slot) * uint32_t(G * mfma::D) + uint32_t(((v * 4 + quad) * G + head) * 4)) * 4u;
}
__device__ inline uint32_t slot_ml(int slot, int G, int head) { return uint32_t(slot * G + head) * 8u; }
__device__ inline int slot_of_partial(int j0, int i) { return i == 0 ? 2 * j0 + 1 : 2 * (j0 + i); }
// vector v of a lane's accumulator registers: dims 4v .. 4v+3 of its 32-dim slice
__device__ inline float4 acc_vec(const mfma::HeadState &x, int v) {
    const int e = 4 * (v & 1), i = v >> 1;
    return float4{x.acc[e][i], x.acc[e + 1][i], x.acc[e + 2][i], x.acc[e + 3][i]};
}

// Log-sum-exp merge of the partials of up to two cut rows, in slot order, and the write of the
// rows.  The loads of both rows are issued before anything is consumed (device-scope loads
// are slow, ~40 ns each per wavefront when measured, so only partials that exist and are not
// the worker's own are fetched).  PV = 4-dim vectors per lane: with PV = 8 lane (quad, r)
// merges all 32 dims of head r (lanes r >= G idle); with PV = 2 or 4 (G <= 2 PV) the 32 dims
// are spread over the 8 / PV lanes (quad, head + 2 PV * sub), so all lanes work and a lane has
// 8 / PV times fewer loads in flight.  The worker's own partial comes from its registers
// (`mine`, re-distributed through `lds`, >= 128 * G floats private to the wavefront, when
// PV < 8): the same values its slot holds, so the result does not depend on which worker merges.
template <int PV, typename Await>
__device__ inline void merge_cut_rows(__amdgpu_buffer_rsrc_t acc_buf, __amdgpu_buffer_rsrc_t ml_buf,
                                      uint16_t *out, int G, int num_q_heads, int lane, float *lds,
                                      const CutRow (&row)[2], const mfma::HeadState &mine0,
                                      const mfma::HeadState &mine1, Await await_row) {
    using namespace mfma;
    constexpr int HP = 2 * PV;  // heads a quad row of 16 lanes can carry: 4, 8 or 16
    const int quad = lane >> 4, r = lane & 15;
    const int head = PV == 8 ? r : (r & (HP - 1)), sub = PV == 8 ? 0 : r / HP;
    const bool active = head < G;
    const int hd = active ? head : 0;

    float4 own_x[2][PV];
    float2 own_ml[2];
#pragma unroll
    for (int w = 0; w < 2; ++w) {
        const HeadState &mine = w == 0 ? mine0 : mine1;
        if (!row[w].active) continue;
        if constexpr (PV == 8) {
#pragma unroll
            for (int v = 0; v < 8; ++v) own_x[w][v] = acc_vec(mine, v);
            own_ml[w] = float2{mine.m, mine.l};
        } else {
            if (r < G) {
#pragma unroll
                for (int v = 0; v < 8; ++v)
                    *reinterpret_cast<float4 *>(lds + slot_vec(0, G, v, quad, r) / 4) = acc_vec(mine, v);
            }
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int vv = 0; vv < PV; ++vv)
                own_x[w][vv] = *reinterpret_cast<const float4 *>(lds + slot_vec(0, G, PV * sub + vv, quad, hd) / 4);
            own_ml[w] = float2{__shfl(mine.m, (lane & 48) | hd), __shfl(mine.l, (lane & 48) | hd)};
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    }

    constexpr int kMergeBatch = 16 / PV;  // partials of a row fetched together (64 registers per row)
    float2 ml[2][kMergeBatch];
    float4 x[2][kMergeBatch][PV];
    auto issue = [&](int w, int c0) __attribute__((always_inline)) {
        if (active) {
#pragma unroll
            for (int u = 0; u < kMergeBatch; ++u) {
                // wavefront-uniform: nothing is fetched past the row's partials, nor this worker's own
                if (c0 + u >= row[w].cnt || c0 + u == row[w].own) continue;
                const int slot = slot_of_partial(row[w].j0, c0 + u);
                ml[w][u] = load2_device_scope(ml_buf, slot_ml(slot, G, hd));
#pragma unroll
                for (int vv = 0; vv < PV; ++vv)
                    x[w][u][vv] = load4_device_scope(acc_buf, slot_vec(slot, G, PV * sub + vv, quad, hd));
            }
        }
    };
    // a row's pieces are fetched as soon as all of them are published: the other row's poll and
    // the hand-over of the own pieces above run under the first row's loads
#pragma unroll
    for (int w = 0; w < 2; ++w)
        if (row[w].active) {
            await_row(w);
            issue(w, 0);
        }

#pragma unroll
    for (int w = 0; w < 2; ++w) {
        if (!row[w].active) continue;
        const int cnt = row[w].cnt;
        float M = -INFINITY, L = 0.f;
        float4 a[PV];
#pragma unroll
        for (int vv = 0; vv < PV; ++vv) a[vv] = float4{0.f, 0.f, 0.f, 0.f};
        for (int c0 = 0; c0 < cnt; c0 += kMergeBatch) {
            if (c0 > 0) issue(w, c0);
            float mc = M;
#pragma unroll
            for (int u = 0; u < kMergeBatch; ++u) {
                if (c0 + u == row[w].own) {  // wavefront-uniform
                    ml[w][u] = own_ml[w];
#pragma unroll
                    for (int vv = 0; vv < PV; ++vv) x[w][u][vv] = own_x[w][vv];
                }
                if (c0 + u >= cnt) {         // past the row's partials: weight 0 below
                    ml[w][u] = float2{-INFINITY, 0.f};
#pragma unroll
                    for (int vv = 0; vv < PV; ++vv) x[w][u][vv] = float4{0.f, 0.f, 0.f, 0.f};
                }
                mc = fmaxf(mc, ml[w][u].x);  // finite: every partial holds at least one token
            }
            const float alpha = __builtin_amdgcn_exp2f(M - mc);
            M = mc;
            L *= alpha;
#pragma unroll
            for (int vv = 0; vv < PV; ++vv) { a[vv].x *= alpha; a[vv].y *= alpha; a[vv].z *= alpha; a[vv].w *= alpha; }
#pragma unroll
            for (int u = 0; u < kMergeBatch; ++u) {
                const float wgt = c0 + u < cnt ? __builtin_amdgcn_exp2f(ml[w][u].x - M) : 0.f;
                L = fmaf(wgt, ml[w][u].y, L);
#pragma unroll
                for (int vv = 0; vv < PV; ++vv) {
                    a[vv].x = fmaf(wgt, x[w][u][vv].x, a[vv].x);
                    a[vv].y = fmaf(wgt, x[w][u][vv].y, a[vv].y);
                    a[vv].z = fmaf(wgt, x[w][u][vv].z, a[vv].z);
                    a[vv].w = fmaf(wgt, x[w][u][vv].w, a[vv].w);
                }
            }
        }
        if (active) {
            const float inv = 1.0f / L;
            uint16_t *dst = out + (size_t(row[w].n) * num_q_heads + row[w].kvh * G + head) * D + 32 * quad + 4 * PV * sub;
#pragma unroll
            for (int v = 0; v < PV / 2; ++v) {
                uint4 o;
                o.x = pack_bf16(a[2 * v].x * inv, a[2 * v].y * inv);
                o.y = pack_bf16(a[2 * v].z * inv, a[2 * v].w * inv);
                o.z = pack_bf16(a[2 * v + 1].x * inv, a[2 * v + 1].y * inv);
                o.w = pack_bf16(a[2 * v + 1].z * inv, a[2 * v + 1].w * inv);
                *reinterpret_cast<uint4 *>(dst + 8 * v) = o;
            }
        }
    }
}

// A row of the flattened work: (sequence, KV head); all fields wavefront-uniform.
struct RowCursor {
    int n;       // sequence
    int kvh;     // KV head
    int pref;    // flat units (per KV head) of all sequences before n
    int tiles;   // t_n (the row spans t_n + kRowCost flat units)
};

// What a launch does with the placement of the workers (the start-up work that depends only on
// block_tables and context_lens, which all layers of one decode step share):
//   kDirect     computes it and streams (the stateless call);
//   kBuild      computes it and writes it to a schedule buffer, nothing else;
//   kScheduled  reads it from a schedule buffer and streams: the prefix table, the worker's plan
//               and its first tile addresses arrive in one memory round trip instead of the
//               three dependent ones (context lengths, block table, first tile) of kDirect.
enum : int { kDirect = 0, kBuild = 1, kScheduled = 2 };
constexpr int kPlanInts = 16;  // a worker's plan in the schedule buffer

// MAXSPT: sequences per thread in the start-up prefix sum (batches up to MAXSPT * 256 sequences);
// the small instance keeps the start-up of ordinary batches short.
template <int MAXSPT, int MODE>
__global__ __launch_bounds__(kThreads, 1) void pa_stream_mfma_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k_cache,
    const uint16_t *__restrict__ v_cache, const int32_t *__restrict__ block_tables,
    const int32_t *__restrict__ context_lens, uint16_t *__restrict__ out, Workspace ws,
    AttnParams p, int unit_log2, int units_per_block_log2, Schedule sched) {
    constexpr int kSeqs = MAXSPT * kThreads;
    __shared__ int s_pref[kSeqs + 2];  // exclusive prefix of flat units (tiles + row cost) per sequence (+ guard)
    __shared__ int s_ctx[kSeqs];       // context length per sequence
    __shared__ int s_wave_tot[kWaves];
    __shared__ int s_tile[kWaves][kStageTiles * kMaxUnits];  // per worker: pool index of each unit of its next tiles

    const int tid = threadIdx.x;
    const int wave = uniform(tid >> 6), lane = tid & 63;
    const int quad = lane >> 4, r = lane & 15;
    const int nseq = p.num_seqs;

    const int worker = blockIdx.x * kWaves + wave;
    const int U_log2 = 4 - unit_log2;                 // log2(units per tile)
    int plan_word = 0;                                // kScheduled: lane i < kPlanInts holds word i of the plan
    if constexpr (MODE == kScheduled) {
        // one round trip: the worker's plan, its first tile addresses (as many as the staging
        // window or its share of the schedule holds; entries past its tiles are never used) and
        // the prefix table of the batch
        if (lane < kPlanInts) plan_word = sched.plans[size_t(worker) * kPlanInts + lane];
        const int *mine = sched.tiles + size_t(worker) * sched.stride;
        const int window = min(kStageTiles << U_log2, sched.stride);
        for (int e = lane; e < window; e += 64) s_tile[wave][e] = mine[e];
        for (int n = tid; n < nseq + 2; n += kThreads) s_pref[n] = sched.pref[n];
        for (int n = tid; n < nseq; n += kThreads) s_ctx[n] = sched.ctx[n];
        __syncthreads();
    } else
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
                const int c = min(max(context_lens[n], 0), p.max_context_len);
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

    if constexpr (MODE == kBuild) {
        if (blockIdx.x == 0) {  // every workgroup has the same table: one of them keeps it
            for (int n = tid; n < nseq + 2; n += kThreads) sched.pref[n] = s_pref[n];
            for (int n = tid; n < nseq; n += kThreads) sched.ctx[n] = s_ctx[n];
        }
    } else {
        // empty contexts give rows of zeros; workgroup b looks after sequences b, b + grid, ...
        for (int n = blockIdx.x; n < nseq; n += gridDim.x) {
            if (s_ctx[n] == 0) {
                uint4 *row = reinterpret_cast<uint4 *>(out + size_t(n) * p.num_q_heads * D);
                for (int i = tid; i < p.num_q_heads * (D / 8); i += kThreads) row[i] = uint4{0u, 0u, 0u, 0u};
            }
        }
    }

    const int Hkv = p.num_kv_heads;
    const int G = p.group;
    // the plan of a worker with nothing to do
    auto write_empty_plan = [&]() __attribute__((always_inline)) {
        if (MODE == kBuild && lane < kPlanInts) sched.plans[size_t(worker) * kPlanInts + lane] = 0;
    };
    const int T = uniform(s_pref[nseq]) * Hkv;
    const int workers = gridDim.x * kWaves;
    const int C = max(p.min_chunk_tiles, (T + workers - 1) / workers);
    if (MODE != kScheduled && int64_t(worker) * C >= T) {
        write_empty_plan();
        return;
    }
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
    int NT = 0;
    // Cut rows this worker holds a piece of (at most one through slot H: its first segment, when
    // that starts past the row's tile 0; at most one through slot T: its last segment, when that
    // starts at tile 0 and stops before the row's end): sequence, KV head, first worker of the
    // row, number of workers on the row (0 = none).  Known from the worker's placement alone, so
    // that it can announce its arrival before its last tiles are consumed.
    int h_n = 0, h_kvh = 0, h_j0 = 0, h_cnt = 0;
    int t_n = 0, t_kvh = 0, t_j0 = 0, t_cnt = 0;
    if constexpr (MODE == kScheduled) {
        auto word = [&](int i) { return __builtin_amdgcn_readlane(plan_word, i); };
        NT = word(0);
        first.n = word(1); first.kvh = word(2); first.pref = word(3); first.tiles = word(4);
        first_tile = word(5);
        h_n = word(6); h_kvh = word(7); h_j0 = word(8); h_cnt = word(9);
        t_n = word(10); t_kvh = word(11); t_j0 = word(12); t_cnt = word(13);
    } else {
        int lo = 0;
        if (nseq <= 4 * 64) {  // every lane tests one entry: the table is sorted, so the count is the position
            int below = 0;
            for (int base = 0; base < nseq; base += 64) {
                const int n = base + lane;
                below += __popcll(__ballot(n < nseq && s_pref[min(n, nseq)] * Hkv <= f0));
            }
            lo = uniform(below) - 1;  // s_pref[0] = 0 is never above f0
        } else {
            int hi = nseq;
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (uniform(s_pref[mid]) * Hkv <= f0) lo = mid; else hi = mid;
            }
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
    // tiles of this worker: the part of [f0, f1) that falls on tiles rather than cost units;
    // the walk also finds the last row it touches and where its piece of that row ends
    if constexpr (MODE != kScheduled) {
        RowCursor last = first;
        int last_t0 = first_tile, last_end = first_tile;
        RowCursor c = first;
        int t0 = first_tile;
        while (c.n < nseq) {
            const int row0 = c.pref * Hkv + c.kvh * (c.tiles + kRowCost);  // flat unit of the row's tile 0
            if (row0 + t0 >= f1) break;
            const int e = min(row0 + c.tiles, f1) - row0;
            NT += e - t0;
            last = c; last_t0 = t0; last_end = e;
            if (row0 + c.tiles + kRowCost >= f1) break;
            c = next_row(c);
            t0 = 0;
        }
        // x / C for 0 <= x < 2^30 with a quotient below 2^16 (a worker index): the float product
        // is off by less than one, so one correction step either way makes it exact - a handful
        // of instructions against the forty of an integer division, four times, on the path
        // every wavefront walks before it can request its first tile
        const float inv_c = 1.0f / float(C);
        auto div_c = [&](int x) __attribute__((always_inline)) {
            int qt = int(float(x) * inv_c);
            const int rem = x - qt * C;
            qt += (rem >= C) - (rem < 0);
            return qt;
        };
        if (first_tile > 0) {
            const int row_f = first.pref * Hkv + first.kvh * (first.tiles + kRowCost);
            h_n = first.n; h_kvh = first.kvh; h_j0 = div_c(row_f);
            h_cnt = div_c(row_f + first.tiles - 1) - h_j0 + 1;
        }
        if (NT > 0 && last_t0 == 0 && last_end < last.tiles) {
            const int row_f = last.pref * Hkv + last.kvh * (last.tiles + kRowCost);
            t_n = last.n; t_kvh = last.kvh; t_j0 = div_c(row_f);
            t_cnt = div_c(row_f + last.tiles - 1) - t_j0 + 1;
        }
    }
    if (NT == 0) {  // the range covered cost units only; no row counts this worker
        write_empty_plan();
        return;
    }
    if constexpr (MODE == kBuild) {
        const int words[kPlanInts] = {NT, first.n, first.kvh, first.pref, first.tiles, first_tile, h_n, h_kvh,
                                      h_j0, h_cnt, t_n, t_kvh, t_j0, t_cnt, 0, 0};
        int mine = 0;
#pragma unroll
        for (int i = 0; i < kPlanInts; ++i) mine = lane == i ? words[i] : mine;
        if (lane < kPlanInts) sched.plans[size_t(worker) * kPlanInts + lane] = mine;
    }

    // ---- tile addresses of the worker's range, staged in LDS
    // A "unit" is the part of a 16-token tile that lies in one block: min(block_size, 16)
    // tokens, so a tile is U = 1, 2 or 4 units.  Entry (k, u) holds the index, in units, of
    // unit u of the worker's k-th tile inside the KV pools:
    //   (block * Hkv + kv head) * units_per_block + unit-in-block.
    // Units past the end of the context (ragged last tile, blocks never allocated) repeat the
    // last valid unit: they are loaded and masked, never taken from the block table.
    // Staging the addresses up front keeps the steady-state loop free of dependent
    // block-table loads: the issue side needs two LDS reads per tile and no row bookkeeping.
    const int unit_tokens = 1 << unit_log2;
    const int upb_mask = (1 << units_per_block_log2) - 1;
    RowCursor rf = first;           // fill cursor
    int tf = first_tile;            // next tile of row rf to stage
    int staged_base = 0;            // worker-relative index of the first staged tile
    auto stage_tiles = [&](int from) __attribute__((always_inline)) {
        const int count = min(kStageTiles, NT - from);
        if constexpr (MODE == kScheduled) {  // copied from the schedule
            const int *mine = sched.tiles + size_t(worker) * sched.stride + (size_t(from) << U_log2);
            for (int e = lane; e < (count << U_log2); e += 64) s_tile[wave][e] = mine[e];
            staged_base = from;
            return;
        }
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
    if constexpr (MODE == kBuild) {
        // every tile address of the worker, window by window, into its share of the schedule
        int *mine = sched.tiles + size_t(worker) * sched.stride;
        for (int from = 0; from < NT; from += kStageTiles) {
            stage_tiles(from);
            const int count = min(kStageTiles, NT - from);
            for (int e = lane; e < (count << U_log2); e += 64) mine[(size_t(from) << U_log2) + e] = s_tile[wave][e];
        }
        return;
    }
    if constexpr (MODE == kDirect) stage_tiles(0);  // kScheduled: the first window came with the plan

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

    // The H partial is parked in `hp` until the worker's end; the T partial is still in `st` then.
    HeadState hp;
    hp.reset();

    // The segment [seg_first, tc) of row rc is finished: a whole row goes to `out`, a piece of a
    // cut row is kept for the publication at the end of the worker.
    auto finalize = [&]() __attribute__((always_inline)) {
        st.finish();
        if (seg_first > 0) {            // H piece
            hp = st;
        } else if (tc == rc.tiles) {    // whole row
            if (r < G) {  // lane (quad, r) holds O[head r][32*quad .. +31]
                const size_t orow = size_t(rc.n) * p.num_q_heads + rc.kvh * G + r;
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
            }
        }                               // else: T piece, stays in `st`
    };

    const uint32_t slots = 2u * gridDim.x * kWaves;
    const __amdgpu_buffer_rsrc_t acc_buf = raw_buffer(ws.acc, slots * uint32_t(G * D) * 4u);
    const __amdgpu_buffer_rsrc_t ml_buf = raw_buffer(ws.ml, slots * uint32_t(G) * 8u);
    auto store_partial = [&](int slot, const HeadState &x) __attribute__((always_inline)) {
        if (r < G) {
#pragma unroll
            for (int v = 0; v < 8; ++v) {
                const float4 f = acc_vec(x, v);
                store4_device_scope(acc_buf, slot_vec(slot, G, v, quad, r), f.x, f.y, f.z, f.w);
            }
            if (quad == 0) store2_device_scope(ml_buf, slot_ml(slot, G, r), x.m, x.l);
        }
    };

    // Arrival at the cut rows: 1 is added to the lower half of their counter words.
    int oh = 0, ot = 0;
    auto arrive = [&]() __attribute__((always_inline)) {
        if (lane == 0) {
            if (h_cnt) oh = __hip_atomic_fetch_add(ws.cnt + h_j0, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (t_cnt) ot = __hip_atomic_fetch_add(ws.cnt + t_j0, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    };

    // The last worker to arrive at a cut row finishes it.  `seen` is the counter word its
    // arrival returned: when some earlier arrival has not published yet (upper half below
    // cnt - 1) it polls.  The workers polled for have already arrived: they have at most two
    // tiles to consume, their stores to wait for and one add to make, none of which depends on
    // another wavefront, so the poll ends; the cap only keeps a wavefront from spinning forever
    // should that reasoning ever be wrong.
    auto await_publications = [&](int j0, int cnt, int seen) __attribute__((always_inline)) {
        int spins = 0;
        while ((seen >> 16) != cnt - 1 && ++spins < (1 << 22)) {
            __builtin_amdgcn_s_sleep(2);
            seen = uniform(__hip_atomic_load(ws.cnt + j0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        }
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
    // consumed.  The last 1 to 3 tiles are peeled; the worker announces its arrival at its cut
    // rows right after the loads of its last tile have been issued, so that the counter's
    // answer travels while the last tiles are consumed.
    uint4 kA[4], vA[4], kB[4], vB[4];
    issue_next(kA, vA);
    int it = 0;
    for (; it + 3 < NT; it += 2) {
        issue_next(kB, vB);
        compute_next(kA, vA, true);
        issue_next(kA, vA);
        compute_next(kB, vB, true);
    }
    if (it + 3 == NT) {
        issue_next(kB, vB);
        compute_next(kA, vA, true);
        issue_next(kA, vA);
        arrive();
        compute_next(kB, vB, true);
        compute_next(kA, vA, false);
    } else if (it + 2 == NT) {
        issue_next(kB, vB);
        arrive();
        compute_next(kA, vA, true);
        compute_next(kB, vB, false);
    } else {
        arrive();
        compute_next(kA, vA, false);
    }
    finalize();

    // ---- cut rows: publish, and finish the rows this worker was the last to arrive at.
    // Counter word of a row (indexed by its first worker): arrivals in the lower half,
    // publications in the upper half.  If the worker's arrival was the last it merges, taking
    // its own piece from registers and polling for pieces that arrived but are not published
    // yet.  Otherwise it waits until its partial stores (device-scope accesses) have completed
    // (an explicit wait on the vector memory counter) and adds 0x10000.
    if (h_cnt | t_cnt) {
        oh = uniform(oh);
        ot = uniform(ot);
        const bool last_h = h_cnt && (oh & 0xffff) == h_cnt - 1, last_t = t_cnt && (ot & 0xffff) == t_cnt - 1;
        if ((h_cnt && !last_h) || (t_cnt && !last_t)) {
            if (h_cnt && !last_h) store_partial(2 * worker, hp);
            if (t_cnt && !last_t) store_partial(2 * worker + 1, st);
            // The publication may become visible only after the partial has: wait until every
            // store above has completed.  The fence alone does not do it (at workgroup scope
            // it compiles to no wait at all on this target); it keeps the compiler from moving
            // the stores.
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            if (lane == 0) {
                if (h_cnt && !last_h) __hip_atomic_fetch_add(ws.cnt + h_j0, 0x10000, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (t_cnt && !last_t) __hip_atomic_fetch_add(ws.cnt + t_j0, 0x10000, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        if (last_t | last_h) {
            const CutRow rows[2] = {{last_t, t_n, t_kvh, t_j0, t_cnt, 0}, {last_h, h_n, h_kvh, h_j0, h_cnt, worker - h_j0}};
            auto await_row = [&](int w) __attribute__((always_inline)) {
                if (w == 0) await_publications(t_j0, t_cnt, ot);
                else await_publications(h_j0, h_cnt, oh);
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");  // the fetches stay behind the poll
            };
            float *lds = reinterpret_cast<float *>(&s_tile[wave][0]);  // the tile addresses are no longer needed
            if (G <= 4) merge_cut_rows<2>(acc_buf, ml_buf, out, G, p.num_q_heads, lane, lds, rows, st, hp, await_row);
            else if (G <= 8) merge_cut_rows<4>(acc_buf, ml_buf, out, G, p.num_q_heads, lane, lds, rows, st, hp, await_row);
            else merge_cut_rows<8>(acc_buf, ml_buf, out, G, p.num_q_heads, lane, lds, rows, st, hp, await_row);
            // every arrival and publication of these rows has happened: leave their counters at 0
            if (lane == 0) {
                if (last_t) __hip_atomic_store(ws.cnt + t_j0, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (last_h) __hip_atomic_store(ws.cnt + h_j0, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

}  // namespace

hipError_t launch_partial_mfma_stream(const void *q, const void *k_cache, const void *v_cache,
                                      const int32_t *block_tables, const int32_t *context_lens,
                                      void *out, Workspace ws, const AttnParams &p, int grid,
                                      int mode, Schedule sched, hipStream_t stream) {
    // unit = min(block_size, 16) tokens; blocks hold block_size / unit units
    int unit_log2 = 4, upb_log2 = 0;
    if (p.block_size < 16) {
        unit_log2 = p.block_size_log2;
    } else {
        while ((16 << upb_log2) < p.block_size) ++upb_log2;
    }
    const auto *q_ = static_cast<const uint16_t *>(q), *k_ = static_cast<const uint16_t *>(k_cache),
               *v_ = static_cast<const uint16_t *>(v_cache);
    auto *o_ = static_cast<uint16_t *>(out);
    const dim3 g(grid), b(kThreads);
    constexpr int kBig = kMaxStreamSeqs / kThreads;
    const bool small = p.num_seqs <= 4 * kThreads;
#define KVC_LAUNCH_STREAM(SPT, MODE) \
    pa_stream_mfma_kernel<SPT, MODE><<<g, b, 0, stream>>>(q_, k_, v_, block_tables, context_lens, o_, ws, p, \
                                                          unit_log2, upb_log2, sched)
    if (mode == kDirect) {
        if (small) KVC_LAUNCH_STREAM(4, kDirect); else KVC_LAUNCH_STREAM(kBig, kDirect);
    } else if (mode == kBuild) {
        if (small) KVC_LAUNCH_STREAM(4, kBuild); else KVC_LAUNCH_STREAM(kBig, kBuild);
    } else {
        if (small) KVC_LAUNCH_STREAM(4, kScheduled); else KVC_LAUNCH_STREAM(kBig, kScheduled);
    }
#undef KVC_LAUNCH_STREAM
    return hipGetLastError();
}

}  // namespace kvc
