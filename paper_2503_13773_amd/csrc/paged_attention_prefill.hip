// Causal attention of many query positions per sequence over the block-allocated KV cache on
// the matrix cores (gfx950, bf16, head_dim 128, any power-of-two block_size): the recomputation
// path of a preempted request (prefill re-run over prompt + generated tokens, quadratic in the
// sequence length: paper Section 2.5 and 3.5) and chunked prefill.
//
// Bound: MFMA (4 * D * Hq * sum over query rows of (position + 1) flops), not HBM: every K/V
// tile is used by 64 query positions x the query heads that share the KV head.
//
// One workgroup = (sequence, chunk of NG query heads sharing one KV head, 64 consecutive query
// rows); each of its 4 wavefronts owns 16 query rows (the 16 columns of its MFMA tiles) for the
// NG heads.  The workgroup walks the context in steps of 32 tokens.  The K and V rows of a
// step are fetched from the cache once per workgroup (4 x 16 bytes per lane, 1 KiB contiguous
// per load instruction), parked in LDS, and read from there by all four wavefronts as MFMA
// operands: measured with one private copy per wavefront, the vector memory pipeline (about 40
// cache look-ups per 16-byte-per-lane load instruction) was busy 92 % of the time and bound the
// kernel.  LDS holds three steps of K and four of V, so that global loads, LDS writes, LDS reads
// and the arithmetic of four consecutive steps overlap; one barrier per step.
//
// Per step and head: S = K . Q^T for the two 16-token tiles (8 x v_mfma_f32_16x16x32_bf16),
// one online-softmax update over the 32 tokens, and O^T += V^T . P^T with the 32 tokens as the
// depth of 8 more 32-deep MFMAs: the C layout of the two score tiles (lane holds tokens
// 4*quad + i of each) is taken as the B operand as it stands, which fixes the order in which
// the 32 tokens fill the depth slots (slot 8*quad + i = token 4*quad + i of the first tile,
// slot 8*quad + 4 + i the same of the second); the A operand V^T (shared by the NG heads) comes
// from LDS in that order by transposing reads (ds_read_b64_tr_b16; V rows are padded to 288
// bytes so that the 8 rows a half-wavefront touches fall into different banks).  The running
// sum of the weights is one more MFMA against an all-ones A operand, so it adds up exactly the
// bf16-rounded weights that multiply V and needs no cross-lane reduction.  K rows are stored in
// LDS with their 16-byte chunks XOR-permuted by the row number, which makes the A-operand reads
// (16 lanes = 16 rows, same columns) conflict free.
//
// The steps are software-pipelined: a turn of the loop issues the score MFMAs of step s+1 (the
// K operands of its first tile were read from LDS during the previous turn, so they start
// without an LDS wait) together with the exponentials, the P.V MFMAs of step s and the max tree
// of step s+1, so matrix-core and vector work of neighbouring steps overlap inside a wavefront
// as well as between the two wavefronts of a SIMD.
//
// The causal mask only bites in the last one or two steps of a wavefront: steps entirely
// below the diagonal of all 16 rows run code without mask or range checks.  Token 0 is visible
// to every query row and steps are walked in order, so every column has a finite running max
// after the first step.  Workgroups with the most steps (the last query rows) are dispatched
// first.
//
// Block sizes below 16 (SMALL): a 16-token tile spans several blocks, so every thread looks up
// the block of the one row it fetches (its table entry comes one turn ahead, like the scalar
// ids of the large-block path); rows past the workgroup's last needed token re-read that token
// (their blocks may not be allocated), they are masked and their V rows zeroed like any row past
// the diagonal.
#include <math.h>

#include "kvc_internal.h"
#include "pa_mfma_tile.h"

namespace kvc {

namespace {

using namespace mfma;

constexpr int kStepTiles = 2;
constexpr int kStepTokens = kStepTiles * kTileTokens;
constexpr int kStepElems = kStepTiles * kTileElems;
constexpr float kLazyLog2 = 8.0f;
constexpr int kKStages = 3;   // K rows of steps s+1 .. s+3 during turn s
constexpr int kVStages = 4;   // V rows of steps s .. s+3
constexpr int kPreTiles = 1;   // tiles of the next step whose K operands are read one turn ahead (2 measured the same)
constexpr int kVRow = D + 16;                     // padded V row in LDS (288 bytes): see the transpose reads
constexpr int kVStepElems = kStepTokens * kVRow;

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// Online-softmax state of one head: 16 query rows (columns r) x 128 dims; lane (quad, r) holds
// O[row r][16*e + 4*quad + j] in acc[e][j] (MFMA number e covers dims 16e .. 16e+15).
struct PrefillState {
    floatx4 acc[8];
    floatx4 lsum;  // every entry: running sum of the rounded weights of column r
    float m;       // reference point of the weights (base-2 units): within 2^kLazyLog2 of the running max of column r

    __device__ inline void reset() {
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = floatx4{0.f, 0.f, 0.f, 0.f};
        lsum = floatx4{0.f, 0.f, 0.f, 0.f};
        m = -INFINITY;
    }
};

// max over the four lanes that share r (lane = 16*quad + r): the two row swaps exchange 16-lane
// rows between the two copies of the operand, no LDS round trip.
__device__ inline float max_over_quads(float x) {
    const unsigned u = __float_as_uint(x);
    const u32x2 a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    const float a0 = __uint_as_float(a[0]), a1 = __uint_as_float(a[1]);
    const float y = a0 > a1 ? a0 : a1;  // inputs are never NaN; a select needs no quieting moves
    const unsigned w = __float_as_uint(y);
    const u32x2 b = __builtin_amdgcn_permlane32_swap(w, w, false, false);
    const float b0 = __uint_as_float(b[0]), b1 = __uint_as_float(b[1]);
    return b0 > b1 ? b0 : b1;
}

// K operands of one 16-token tile from LDS (sk_tile: [16 tokens][128], 16-byte chunks
// XOR-permuted by the row number).
__device__ inline void read_k_tile(bf16x8 (&ka)[4], const uint16_t *sk_tile, int quad, int r) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
        ka[j] = *reinterpret_cast<const bf16x8 *>(sk_tile + r * D + (((4 * j + quad) ^ r) << 3));
}

// Scores of one tile for every head: S = K . Q^T.
template <int NG>
__device__ inline void tile_scores(floatx4 (&s)[NG][kStepTiles], int t, const bf16x8 (&ka)[4],
                                   const bf16x8 (&qb)[NG][4]) {
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        s[g][t] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j) s[g][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[j], qb[g][j], s[g][t], 0, 0, 0);
    }
}

// Scaled (and, if MASKED, causally masked) scores of one head and the max over this lane's 8
// tokens of the step (the column's other 24 tokens sit in the lanes r + 16, r + 32, r + 48).  The multiply also leaves canonical values, so the max tree compiles to bare
// v_max3/v_max without one quieting move per input.  `limit` = tokens of the step visible to
// this lane's column (may be <= 0).
template <bool MASKED>
__device__ inline float scale_mask_max(float (&x)[8], const floatx4 (&s)[kStepTiles], float scale_log2e,
                                       int limit, int quad) {
#pragma unroll
    for (int t = 0; t < kStepTiles; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[4 * t + i] = s[t][i] * scale_log2e;
            if (MASKED && t * kTileTokens + 4 * quad + i >= limit) x[4 * t + i] = -INFINITY;
        }
    return fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
}

// Lazy rebase: the reference point m only moves when some column's max has grown by more than
// 2^kLazyLog2 over it (always in the first step, m = -inf), so weights are at most 2^kLazyLog2
// and the 36 multiplies of the rebase are rare.  Every column sees token 0 in its first step,
// so m - m_new is never inf - inf.
__device__ inline void rebase(PrefillState &st, float lane_max) {
    // the test needs no cross-lane max: if no lane holds a score above m + 2^kLazyLog2, none exists
    if (__builtin_amdgcn_ballot_w64(lane_max > st.m + kLazyLog2) != 0) {
        const float m_new = fmaxf(st.m, max_over_quads(lane_max));
        const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);
        st.m = m_new;
#pragma unroll
        for (int e = 0; e < 8; ++e) st.acc[e] *= alpha;
        st.lsum *= alpha;
    }
}

// A operands of O^T += V^T . P^T straight from LDS: the transpose read hands lane i of a 16-lane
// block the i-th 16-bit element of each of the four 16-element groups that lanes 4k .. 4k+3 of
// the block point at (8 bytes each).  Lanes 4k .. 4k+3 of block `quad` point at dims 16e + 0, 4,
// 8, 12 of token 4*quad + k, so lane r receives dim 16e + r of tokens 4*quad .. +3: the depth
// slots in the order the score layout fixed.  MASKED: rows at or past `vlim` (tokens of the step
// visible to any column of this wavefront) are zeroed: their weights are zero for every column
// and the rows may hold NaN.
template <bool MASKED>
__device__ inline void read_v_operands(uint2 (&va)[8][kStepTiles], const uint16_t *sv, int vlim, int quad, int r) {
    typedef short v4i16 __attribute__((ext_vector_type(4)));
    typedef v4i16 __attribute__((address_space(3))) * lds_v4i16_ptr;
    const uint16_t *vlane = sv + (4 * quad + (r >> 2)) * kVRow + 4 * (r & 3);
#pragma unroll
    for (int e = 0; e < 8; ++e)
#pragma unroll
        for (int t = 0; t < kStepTiles; ++t)
            va[e][t] = __builtin_bit_cast(uint2, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                                                     (lds_v4i16_ptr)(vlane + t * kTileTokens * kVRow + 16 * e)));
    if (MASKED) {
#pragma unroll
        for (int t = 0; t < kStepTiles; ++t) {
            const int tok = t * kTileTokens + 4 * quad;
            const uint32_t m01 = (tok < vlim ? 0xffffu : 0u) | (tok + 1 < vlim ? 0xffff0000u : 0u);
            const uint32_t m23 = (tok + 2 < vlim ? 0xffffu : 0u) | (tok + 3 < vlim ? 0xffff0000u : 0u);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                va[e][t].x &= m01;
                va[e][t].y &= m23;
            }
        }
    }
}

// O^T += V^T . P^T for every head, and the running weight sums as one more MFMA against an
// all-ones A operand.
template <int NG>
__device__ inline void accumulate_pv(PrefillState (&st)[NG], const uint2 (&va)[8][kStepTiles], const bf16x8 (&pb)[NG]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint4 aw = {va[e][0].x, va[e][0].y, va[e][1].x, va[e][1].y};
        const bf16x8 av = __builtin_bit_cast(bf16x8, aw);
#pragma unroll
        for (int g = 0; g < NG; ++g)
            st[g].acc[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, pb[g], st[g].acc[e], 0, 0, 0);
    }
    const uint4 one_bits = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};  // bf16 1.0 x 8
    const bf16x8 ones = __builtin_bit_cast(bf16x8, one_bits);
#pragma unroll
    for (int g = 0; g < NG; ++g) st[g].lsum = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pb[g], st[g].lsum, 0, 0, 0);
}

// Weights of a step from its scaled scores, rounded to bf16: the B operand of P.V as they stand.
__device__ inline bf16x8 step_weights(const float (&x)[8], float m) {
    float pf[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) pf[i] = __builtin_amdgcn_exp2f(x[i] - m);
    const uint4 pw = {pack_bf16(pf[0], pf[1]), pack_bf16(pf[2], pf[3]), pack_bf16(pf[4], pf[5]), pack_bf16(pf[6], pf[7])};
    return __builtin_bit_cast(bf16x8, pw);
}

// One turn of the software pipeline: the weights and the P.V accumulation of step `cur` (scaled
// scores in x, V rows in sv_cur) together with the scores, scaling and max of step `next` (K rows
// in sk_next), in one straight-line region so that the matrix-core work of one step runs under
// the vector work of the other.  On return x holds the scaled scores of step `next`, the
// reference points are rebased for it, and ka_pre holds K operands of the step after `next`.
// MASKED: `vlim_cur` = tokens of step cur visible to any column of this wavefront (V rows past
// it are zeroed: their weights are zero for every column and the rows may hold NaN);
// `limit_next` = tokens of step next visible to this lane's column.
template <int NG, bool MASKED>
__device__ inline void pipeline_turn(PrefillState (&st)[NG], float (&x)[NG][8], bf16x8 (&ka_pre)[kStepTiles][4],
                                     const uint16_t *sk_next, const uint16_t *sk_next2, const uint16_t *sv_cur,
                                     const bf16x8 (&qb)[NG][4], float scale_log2e, int vlim_cur, int limit_next,
                                     int quad, int r) {
    uint2 va[8][kStepTiles];
    read_v_operands<MASKED>(va, sv_cur, vlim_cur, quad, r);

    // scores of step next: the first kPreTiles tiles from operands read during the previous turn
    // (no LDS wait in front of the first MFMAs), the rest from LDS now; then the operands of the
    // step after next are read for the coming turn
    floatx4 s[NG][kStepTiles];
#pragma unroll
    for (int t = 0; t < kStepTiles; ++t) {
        if (t < kPreTiles) {
            tile_scores<NG>(s, t, ka_pre[t], qb);
        } else {
            bf16x8 ka[4];
            read_k_tile(ka, sk_next + t * kTileElems, quad, r);
            tile_scores<NG>(s, t, ka, qb);
        }
    }
#pragma unroll
    for (int t = 0; t < kPreTiles; ++t) read_k_tile(ka_pre[t], sk_next2 + t * kTileElems, quad, r);

    bf16x8 pb[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) pb[g] = step_weights(x[g], st[g].m);
    accumulate_pv<NG>(st, va, pb);

    float mx[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) mx[g] = scale_mask_max<MASKED>(x[g], s[g], scale_log2e, limit_next, quad);
#pragma unroll
    for (int g = 0; g < NG; ++g) rebase(st[g], mx[g]);
}

template <int NG, bool SMALL>
__global__ __launch_bounds__(kThreads, 2) void pa_prefill_mfma_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k_cache,
    const uint16_t *__restrict__ v_cache, const int32_t *__restrict__ block_tables,
    const int32_t *__restrict__ context_lens, const int32_t *__restrict__ q_start,
    uint16_t *__restrict__ out, PrefillParams p) {
    __shared__ __attribute__((aligned(16))) uint16_t s_k[kKStages][kStepElems];
    __shared__ __attribute__((aligned(16))) uint16_t s_v[kVStages][kVStepElems];

    // blockIdx.x = head chunk + chunks * (seq + num_seqs * reversed query tile)
    const int chunks = p.num_q_heads / NG;
    const int item = blockIdx.x;
    const int chunk = item % chunks;
    const int n = (item / chunks) % p.num_seqs;
    const int qtile = p.max_query_tiles - 1 - item / (chunks * p.num_seqs);
    const int head0 = chunk * NG;
    const int kvh = head0 / p.group;

    const int S = context_lens[n];
    const int qs = q_start[n];
    const int Qn = q_start[n + 1] - qs;
    if (qtile * 64 >= Qn || Qn > S) return;  // uniform over the workgroup

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int quad = lane >> 4, r = lane & 15;

    // tiles and steps this workgroup walks (up to the position of its last query row)
    const int last_pos = S - Qn + min(Qn, qtile * 64 + 64) - 1;
    const int wg_tiles = (last_pos >> 4) + 1;
    const int wg_steps = (wg_tiles + kStepTiles - 1) / kStepTiles;
    const int32_t *table = block_tables + size_t(n) * p.max_blocks_per_seq;

    // wavefronts past the last query row still fetch and synchronise, they just never compute
    const int i0 = qtile * 64 + 16 * wave;  // first query row of this wavefront
    const bool active = i0 < Qn;
    const int ncols = active ? min(16, Qn - i0) : 1;
    const int col = min(r, ncols - 1);      // lanes past the last query row shadow it
    const int p0 = S - Qn + (active ? i0 : 0);  // position of column 0
    const int my_pos = p0 + col;
    const int wave_vis = p0 + ncols;        // tokens visible to some column of this wavefront
    const int free_steps = (p0 + 1) / kStepTokens;  // steps whose every token every column sees

    bf16x8 qb[NG][4];
#pragma unroll
    for (int g = 0; g < NG; ++g)
        load_q_operand(qb[g], q + (size_t(qs + (active ? i0 : 0) + col) * p.num_q_heads + head0 + g) * D, quad, true);

    PrefillState st[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) st[g].reset();

    const size_t head_elems = size_t(p.block_size) * D;
    const size_t block_elems = head_elems * p.num_kv_heads;
    const int sub_mask = (1 << p.tiles_per_block_log2) - 1;

    // this thread's share of a step: 16 bytes of row (tid >> 4), chunk (tid & 15), of each of the
    // two K tiles and the two V tiles; tiles past the last one re-read it (never used unmasked)
    const int lrow = tid >> 4, lchunk = tid & 15;
    const int k_dst = lrow * D + ((lchunk ^ lrow) << 3);
    const int v_dst = lrow * kVRow + (lchunk << 3);
    struct Share { uint4 k0, k1, v0, v1; };
    const int lane_off = lrow * D + (lchunk << 3);  // elements inside a tile
    const uint16_t *k_head = k_cache + size_t(kvh) * head_elems;
    const uint16_t *v_head = v_cache + size_t(kvh) * head_elems;
    // Large blocks: block ids are uniform over the workgroup, they come through the scalar cache
    // one turn before the fetch that uses them, and the tile bases live in scalar registers.
    // Tiles past the last one repeat it (never used unmasked).  Small blocks: b0 / b1 are the
    // blocks of this thread's row in the two tiles, t0 / t1 the row's slot inside its block.
    struct Ids { int t0, t1, b0, b1; };
    auto ids_of = [&](int step) __attribute__((always_inline)) -> Ids {
        Ids id;
        if (SMALL) {
            const int tok0 = min(step * kStepTokens + lrow, last_pos);
            const int tok1 = min(step * kStepTokens + kTileTokens + lrow, last_pos);
            id.t0 = tok0 & (p.block_size - 1);
            id.t1 = tok1 & (p.block_size - 1);
            id.b0 = table[tok0 >> p.block_size_log2];
            id.b1 = table[tok1 >> p.block_size_log2];
        } else {
            id.t0 = min(step * kStepTiles, wg_tiles - 1);
            id.t1 = min(step * kStepTiles + 1, wg_tiles - 1);
            id.b0 = __builtin_amdgcn_readfirstlane(table[id.t0 >> p.tiles_per_block_log2]);
            id.b1 = __builtin_amdgcn_readfirstlane(table[id.t1 >> p.tiles_per_block_log2]);
        }
        return id;
    };
    auto fetch = [&](const Ids &id) __attribute__((always_inline)) -> Share {
        size_t b0, b1;
        if (SMALL) {
            b0 = size_t(id.b0) * block_elems + size_t(id.t0) * D + (lchunk << 3);
            b1 = size_t(id.b1) * block_elems + size_t(id.t1) * D + (lchunk << 3);
        } else {
            b0 = size_t(id.b0) * block_elems + size_t(id.t0 & sub_mask) * kTileElems + lane_off;
            b1 = size_t(id.b1) * block_elems + size_t(id.t1 & sub_mask) * kTileElems + lane_off;
        }
        Share sh;
        sh.k0 = *reinterpret_cast<const uint4 *>(k_head + b0);
        sh.k1 = *reinterpret_cast<const uint4 *>(k_head + b1);
        sh.v0 = *reinterpret_cast<const uint4 *>(v_head + b0);
        sh.v1 = *reinterpret_cast<const uint4 *>(v_head + b1);
        return sh;
    };
    auto park = [&](int kstage, int vstage, const Share &sh) __attribute__((always_inline)) {
        *reinterpret_cast<uint4 *>(&s_k[kstage][k_dst]) = sh.k0;
        *reinterpret_cast<uint4 *>(&s_k[kstage][kTileElems + k_dst]) = sh.k1;
        *reinterpret_cast<uint4 *>(&s_v[vstage][v_dst]) = sh.v0;
        *reinterpret_cast<uint4 *>(&s_v[vstage][kTileTokens * kVRow + v_dst]) = sh.v1;
    };

    // K rows of step j live in K stage j % 3, V rows in V stage j % 4.  Turn s parks step s+3
    // (fetched during turn s-1) over K(s) and V(s-1), whose last readers passed the barrier that
    // ended turn s-1, and issues the fetch of step s+4; it computes the scores of step s+1
    // (operands read during turn s-1, or from K stage (s+1) % 3), reads operands of step s+2 for
    // the next turn and the V rows of step s.  The barrier at its end publishes step s+3.  Past
    // the last step the last one is fetched and parked again (unused): the loop stays branch free.
    {
        const Share d0 = fetch(ids_of(0));
        const Share d1 = fetch(ids_of(min(1, wg_steps - 1)));
        park(0, 0, d0);
        park(1, 1, d1);
    }
    Share next = fetch(ids_of(min(2, wg_steps - 1)));
    __syncthreads();

    float x[NG][8];
    bf16x8 ka_pre[kStepTiles][4];
    if (active) {  // scores of step 0, then the operands turn 0 starts from
        floatx4 s[NG][kStepTiles];
#pragma unroll
        for (int t = 0; t < kStepTiles; ++t) {
            bf16x8 ka[4];
            read_k_tile(ka, s_k[0] + t * kTileElems, quad, r);
            tile_scores<NG>(s, t, ka, qb);
        }
#pragma unroll
        for (int g = 0; g < NG; ++g) rebase(st[g], scale_mask_max<true>(x[g], s[g], p.scale_log2e, my_pos + 1, quad));
#pragma unroll
        for (int t = 0; t < kPreTiles; ++t) read_k_tile(ka_pre[t], s_k[1] + t * kTileElems, quad, r);
    }
    park(2, 2, next);  // K stage 2 and V stage 2 have not been used yet
    next = fetch(ids_of(min(3, wg_steps - 1)));
    Ids ids = ids_of(min(4, wg_steps - 1));
    __syncthreads();

    int k0 = 0, k1 = 1, k2 = 2;  // K stages of steps s, s+1, s+2
    for (int s = 0; s < wg_steps; ++s) {
        park(k0, (s + 3) & 3, next);
        next = fetch(ids);
        ids = ids_of(min(s + 5, wg_steps - 1));
        if (active) {
            if (s + 1 < free_steps)
                pipeline_turn<NG, false>(st, x, ka_pre, s_k[k1], s_k[k2], s_v[s & 3], qb, p.scale_log2e, kStepTokens,
                                         kStepTokens, quad, r);
            else
                pipeline_turn<NG, true>(st, x, ka_pre, s_k[k1], s_k[k2], s_v[s & 3], qb, p.scale_log2e,
                                        wave_vis - s * kStepTokens, my_pos + 1 - (s + 1) * kStepTokens, quad, r);
        }
        __syncthreads();
        const int t = k0;
        k0 = k1;
        k1 = k2;
        k2 = t;
    }

    if (!active) return;
    // lane (quad, r < ncols) holds O[query row i0 + r][head0 + g][16*e + 4*quad .. +3] in acc[e]
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        if (r < ncols) {
            const float inv = 1.0f / st[g].lsum[0];
            uint16_t *dst = out + (size_t(qs + i0 + r) * p.num_q_heads + head0 + g) * D + 4 * quad;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                uint2 w;
                w.x = pack_bf16(st[g].acc[e][0] * inv, st[g].acc[e][1] * inv);
                w.y = pack_bf16(st[g].acc[e][2] * inv, st[g].acc[e][3] * inv);
                *reinterpret_cast<uint2 *>(dst + 16 * e) = w;
            }
        }
    }
}

}  // namespace

hipError_t launch_prefill_mfma(const void *q, const void *k_cache, const void *v_cache,
                               const int32_t *block_tables, const int32_t *context_lens,
                               const int32_t *q_start, void *out, const PrefillParams &p,
                               hipStream_t stream) {
    const auto *qq = static_cast<const uint16_t *>(q);
    const auto *kk = static_cast<const uint16_t *>(k_cache);
    const auto *vv = static_cast<const uint16_t *>(v_cache);
    auto *oo = static_cast<uint16_t *>(out);
    const int ng = p.heads_per_chunk;
    const bool small = p.block_size < kTileTokens;
    const unsigned grid = unsigned(int64_t(p.num_q_heads / ng) * p.num_seqs * p.max_query_tiles);
    const dim3 g(grid), b(kThreads);
    if (ng == 2 && !small) pa_prefill_mfma_kernel<2, false><<<g, b, 0, stream>>>(qq, kk, vv, block_tables, context_lens, q_start, oo, p);
    else if (ng == 2) pa_prefill_mfma_kernel<2, true><<<g, b, 0, stream>>>(qq, kk, vv, block_tables, context_lens, q_start, oo, p);
    else if (!small) pa_prefill_mfma_kernel<1, false><<<g, b, 0, stream>>>(qq, kk, vv, block_tables, context_lens, q_start, oo, p);
    else pa_prefill_mfma_kernel<1, true><<<g, b, 0, stream>>>(qq, kk, vv, block_tables, context_lens, q_start, oo, p);
    return hipGetLastError();
}

}  // namespace kvc
