// Causal attention of many query positions per sequence over the block-allocated KV cache on
// 32x32x16 matrix-core tiles (gfx950, bf16, head_dim 128, positive scale): the
// recomputation path of a preempted request (prefill re-run over prompt + generated tokens,
// quadratic in the sequence length: paper Section 2.5 and 3.5) and chunked prefill.
//
// Why 32x32 tiles.  Measured on this chip, a vector instruction holds a SIMD's vector issue
// port for 4 cycles, an exponential for 8 and a matrix instruction for 8, whatever its shape;
// a 16x16x32 tile then runs 16 cycles in the matrix pipe, a 32x32x16 tile 32 cycles with twice
// the work.  Attention at head_dim 128 needs per 32 tokens x 32 score columns about 60 vector
// instructions and 16 exponentials of softmax arithmetic (16 scores per lane).  With 34 small
// tiles that adds up to about 800 port cycles against 544 matrix cycles; with 16 large tiles it
// is about 500 port cycles against 512.
//
// One workgroup = (sequence, 2 query heads sharing one KV head, 64 or 128 consecutive query
// rows); each of its 4 or 8 wavefronts owns 16 query rows x 2 heads = the 32 columns of its
// tiles (column c = 16 * head + row).  Odd GQA group sizes take one head and 32 query rows per
// wavefront instead (workgroups of 128 or 256 rows); everything below is written for two heads
// and holds for one with "row" = c.  The workgroup walks the context in steps of 32 tokens
// (the 32 rows of a score tile).  With 8 wavefronts the two groups of four run half a turn
// apart, so that the two wavefronts of a SIMD are in opposite halves of their turns.
//
// K and V rows travel from the cache straight into LDS (global_load_lds_dwordx4: lane l of a
// wavefront writes its 16 bytes at M0 + 16 * l, no register staging), requested two turns
// before their first use (K rows four steps ahead, V rows three); which bytes a
// lane fetches is chosen so that the LDS image is
//   K rows: 16-byte chunks XOR-permuted by the row number (A-operand reads of 16 rows x the
//           same dims then touch every bank once);
//   V rows: 64-byte granules rotated by the row number (the 4 rows x 64 bytes that a
//           half-wavefront reads in one transposing access then fall into disjoint banks).
// Four steps of K and four of V are in LDS (64 KiB).
//
// Per step, with lane = 32 * half + c:
//   S^T = K . Q^T      8 x v_mfma_f32_32x32x16_bf16 (depth = the 128 dims).  A: K row c of the
//                      step, dims 16j + 8*half .. +7; B: the same dims of column c's query row.
//                      The lane receives the 16 scores of column c against tokens
//                      8*(v/4) + 4*half + v%4, v < 16.
//   softmax            all 16 scores of a lane belong to one column: in-lane max (raw scores,
//                      the scale is positive), one fused multiply-add and one exponential per
//                      score (weight = exp2(score * scale - m)); the weights are rounded to
//                      bf16 for P.V and added up in fp32 for the normaliser.  The two halves of
//                      a column meet only when the reference point m moves (lazily: when some
//                      score exceeds it by more than 2^8) and once at the end.
//   O^T += V^T . P^T   8 x v_mfma_f32_32x32x16_bf16: 4 blocks of 32 dims x 2 slices of 16
//                      tokens.  B is the weight registers as they stand (slice n = registers
//                      8n .. 8n+7, depth slot 8*half + i = token 16n + 8*(i/4) + 4*half + i%4);
//                      A = V^T comes from LDS in that token order by transposing reads
//                      (ds_read_b64_tr_b16: 4 consecutive tokens of the lane's dim per read).
//
// The causal mask only bites in the last one or two steps of a wavefront: steps entirely below
// the diagonal of all 16 rows run code without mask or range checks.  Token 0 is visible to
// every query row and steps are walked in order, so every column has a finite reference point
// after the first step.  Workgroups with the most steps (the last query rows) are dispatched
// first.
#include <math.h>

#include "kvc_internal.h"
#include "pa_mfma_tile.h"

namespace kvc {

namespace {

using namespace mfma;

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kStepTokens = 32;
constexpr int kStageBytes = kStepTokens * D * 2;  // K (or V) rows of a step: 32 rows x 256 bytes
constexpr float kLazyLog2 = 8.0f;
constexpr int kKStages = 4;   // K rows of steps s+1 .. s+4 during turn s
constexpr int kVStages = 4;   // V rows of steps s .. s+3

// Online-softmax state of one column (query row x head); lane (half, c) holds
// O[column c][32*b + 8*(v/4) + 4*half + v%4] in acc[b][v].
struct ColumnState {
    floatx16 acc[4];
    float lsum;  // sum of the rounded weights of this lane's tokens (the other half's lane holds the rest)
    float m;     // reference point of the weights (base-2 units): within 2^kLazyLog2 of the column's running max

    __device__ inline void reset() {
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;
        lsum = 0.f;
        m = -INFINITY;
    }
};

// The value lane l ^ 32 holds, next to this lane's: one swap of the two 32-lane halves.
__device__ inline float max_over_halves(float x) {
    const unsigned u = __float_as_uint(x);
    const u32x2 b = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const float b0 = __uint_as_float(b[0]), b1 = __uint_as_float(b[1]);
    return b0 > b1 ? b0 : b1;  // inputs are never NaN
}
__device__ inline float sum_over_halves(float x) {
    const unsigned u = __float_as_uint(x);
    const u32x2 b = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// max of three without the quieting moves the compiler puts in front of a max whose inputs
// come out of the matrix pipe (they are never NaN here: finite scores or -inf)
__device__ inline float max3(float a, float b, float c) {
    float d;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}

// Raw scores of a step into x (if MASKED, -inf where the token is not visible to the lane's
// column: `limit` = tokens of the step it sees, may be <= 0) and their max over the lane.
template <bool MASKED>
__device__ inline float take_scores(float (&x)[16], const floatx16 &s, int limit, int half) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        x[v] = s[v];
        if (MASKED && 8 * (v >> 2) + 4 * half + (v & 3) >= limit) x[v] = -INFINITY;
    }
    const float a = max3(x[0], x[1], x[2]), b = max3(x[3], x[4], x[5]), c = max3(x[6], x[7], x[8]);
    const float d = max3(x[9], x[10], x[11]), e = max3(x[12], x[13], x[14]);
    const float f = max3(a, b, c), g = max3(d, e, x[15]);
    float h;
    asm("v_max_f32 %0, %1, %2" : "=v"(h) : "v"(f), "v"(g));
    return h;
}

// Lazy rebase: the reference point m only moves when some column's scaled max has grown by more
// than 2^kLazyLog2 over it (always in the first step, m = -inf), so weights are at most
// 2^kLazyLog2 and the 65 multiplies of the rebase are rare.  Every column sees token 0 in its
// first step, so m - m_new is never inf - inf.
__device__ inline void rebase(ColumnState &st, float lane_max, float scale_log2e) {
    const float scaled = lane_max * scale_log2e;
    // the test needs no cross-lane max: if no lane holds a score above m + 2^kLazyLog2, none exists
    if (__builtin_amdgcn_ballot_w64(scaled > st.m + kLazyLog2) != 0) {
        const float m_new = fmaxf(st.m, max_over_halves(scaled));
        const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);
        st.m = m_new;
#pragma unroll
        for (int b = 0; b < 4; ++b) st.acc[b] *= alpha;
        st.lsum *= alpha;
    }
}

// A operands of O^T += V^T . P^T straight from LDS.  The transposing read hands lane i of a
// 16-lane block the i-th 16-bit element of each of the four 16-element groups that lanes
// 4k .. 4k+3 of the block point at (8 bytes each).  Block (half, w) of this wavefront covers
// dims 32b + 16w .. +15; its lanes 4k .. 4k+3 point at dims +0, 4, 8, 12 of token
// 16n + 8g + 4*half + k, so the lane of dim 32b + c receives that dim of the four tokens
// 16n + 8g + 4*half .. +3: depth slots 8*half + 4g .. +3 of slice n, the order the score layout
// fixed.  Row R of a V stage keeps its 64-byte granule b at granule position (b + R) % 4, and
// R % 4 = k for the row a lane points at, so the byte offset of the lane inside a stage for
// dim block b is v_lane_offset(b) + (16n + 8g) rows.
__device__ inline int v_lane_offset(int b, int half, int c) {
    const int i16 = c & 15, k = i16 >> 2;
    return (4 * half + k) * 256 + ((b + k) & 3) * 64 + 32 * (c >> 4) + 8 * (i16 & 3);
}
template <int N>
__device__ inline void read_v_operand(uint2 (&va)[2], const unsigned char *vlane) {
    typedef short v4i16 __attribute__((ext_vector_type(4)));
    typedef v4i16 __attribute__((address_space(3))) * lds_v4i16_ptr;
#pragma unroll
    for (int g = 0; g < 2; ++g)
        va[g] = __builtin_bit_cast(uint2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_ptr)(vlane + (16 * N + 8 * g) * 256)));
}

// V rows at or past `vlim` (tokens of the step visible to any column of this wavefront) are
// zeroed in the operand of slice N: their weights are zero for every column and the rows may
// hold NaN.
template <int N>
__device__ inline void mask_v_operand(uint2 (&va)[2], int vlim, int half) {
#pragma unroll
    for (int g = 0; g < 2; ++g) {
        const int tok = 16 * N + 8 * g + 4 * half;
        va[g].x &= (tok < vlim ? 0xffffu : 0u) | (tok + 1 < vlim ? 0xffff0000u : 0u);
        va[g].y &= (tok + 2 < vlim ? 0xffffu : 0u) | (tok + 3 < vlim ? 0xffff0000u : 0u);
    }
}

__device__ inline bf16x8 v_operand(const uint2 (&va)[2]) {
    const uint4 aw = {va[0].x, va[0].y, va[1].x, va[1].y};
    return __builtin_bit_cast(bf16x8, aw);
}

// K operand j of a step from LDS (a stage is 32 rows of 256 bytes, 16-byte chunks XOR-permuted
// by row % 16); lane (half, c) reads row c, dims 16j + 8*half .. +7.
template <int J>
__device__ inline bf16x8 read_k_operand(const unsigned char *krow, int half, int c) {
    return *reinterpret_cast<const bf16x8 *>(krow + (((2 * J + half) ^ (c & 15)) << 4));
}

// 16 bytes per lane from global memory straight into LDS: lane l's bytes land at lds_addr +
// 16 * l (lds_addr uniform).  The two-instruction forms load a second 1 KiB from 1 KiB further
// on both sides.  The compiler does not see these accesses: the caller orders them against LDS
// reads with barriers and waits for them with wait_loads_but().
__device__ inline void load_rows_to_lds(const void *base, uint32_t off0, uint32_t off1_minus_1k, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %3\n\tglobal_load_lds_dwordx4 %2, %3 offset:1024"
                 :: "s"(lds_addr), "v"(off0), "v"(off1_minus_1k), "s"(base) : "memory");
}
__device__ inline void load_row_group_to_lds(const void *base, uint32_t off, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" :: "s"(lds_addr), "v"(off), "s"(base) : "memory");
}
__device__ inline void load_lane_to_lds(const void *addr, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" :: "s"(lds_addr), "v"(addr) : "memory");
}
template <int N>
__device__ inline void wait_loads_but() {
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// The barrier that ends a turn.  The wavefront first waits for its own LDS reads (operands
// requested for the next turn): the loads of the next turn overwrite the stages they come from.
__device__ inline void turn_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// The barrier in the middle of a turn orders no data (see the kernel): it only keeps the two
// groups of wavefronts half a turn apart.
__device__ inline void phase_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// Nothing moves across this point when the compiler orders the instructions of a turn.
#define KVC_PIN() __builtin_amdgcn_sched_barrier(0)

// One turn of the software pipeline: the weights and the P.V accumulation of step `cur` (raw
// scores in x) together with the scores and the max of step `next`.  The order of the turn is
// pinned chunk by chunk, one matrix instruction (32 cycles in the matrix pipe, 8 on the issue
// port) per chunk together with the vector work that fits under it and the LDS reads of operands
// that are due half a turn or more later:
//     chunks  0 ..  3   S(next) += K operand j . Q, j < 4       2 weights of cur each (fma, exp2), rounding, sum
//                       reads K operand 4 + j of step next
//     chunks  4 ..  7   O block b += V slice 0 . weights 0..7   2 weights each (scores 8 .. 15), rounding, sum
//                       reads V operand b, slice 1, of step cur
//     chunks  8 .. 11   S(next) += K operand j . Q, j >= 4      block id of the following turn's loads (`lookup`)
//                       reads K operand j - 4 of the step after next and V operand j - 4, slice 0, of step next
//     chunks 12 .. 15   O block b += V slice 1 . weights 8..15  max of S(next)
//                       requests the K and V rows of the step four ahead (`issue_k`, `issue_v`)
// so the turn starts with ka_lo = K operands 0 .. 3 of step next and va0 = the slice-0 V
// operands of step cur in registers and ends with those of the following turn.
// On return x holds the raw scores of step `next` and the reference point is rebased for it.
// MASKED: `vlim_cur` = tokens of step cur visible to any column of this wavefront,
// `limit_next` = tokens of step next visible to this lane's column.
template <bool MASKED, class IssueK, class IssueV, class Mid, class Lookup>
__device__ inline void pipeline_turn(ColumnState &st, float (&x)[16], bf16x8 (&ka_lo)[4], uint2 (&va0)[4][2],
                                     const unsigned char *krow1, const unsigned char *krow2,
                                     const unsigned char *sv_cur, const unsigned char *sv_next, const int (&voff)[4],
                                     const bf16x8 (&qb)[8], float scale_log2e, int vlim_cur, int limit_next, int half,
                                     int c, const IssueK &issue_k, const IssueV &issue_v, const Mid &mid, const Lookup &lookup) {
    const float neg_m = -st.m;
    float arg[16], pf[16], pair[8];
    uint32_t w[8];
    bf16x8 ka_hi[4];
    uint2 va1[4][2];
    floatx16 s;
#pragma unroll
    for (int v = 0; v < 16; ++v) s[v] = 0.f;

    // The softmax arithmetic of score pair P goes through four stages placed in different chunks,
    // so that no instruction waits for the result of the one in front of it: exponent arguments,
    // exponentials, rounding to bf16 plus the pair's sum, and the addition to the normaliser.
#define KVC_ARG(P)                                                           \
    arg[2 * (P)] = __builtin_fmaf(x[2 * (P)], scale_log2e, neg_m);           \
    arg[2 * (P) + 1] = __builtin_fmaf(x[2 * (P) + 1], scale_log2e, neg_m)
#define KVC_EXP(P)                                        \
    pf[2 * (P)] = __builtin_amdgcn_exp2f(arg[2 * (P)]);   \
    pf[2 * (P) + 1] = __builtin_amdgcn_exp2f(arg[2 * (P) + 1])
#define KVC_ROUND(P)                                \
    w[P] = pack_bf16(pf[2 * (P)], pf[2 * (P) + 1]); \
    pair[P] = pf[2 * (P)] + pf[2 * (P) + 1]
#define KVC_SUM(P) st.lsum += pair[P]
#define KVC_QK_LO(J)                                                          \
    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka_lo[J], qb[J], s, 0, 0, 0); \
    ka_hi[J] = read_k_operand<4 + (J)>(krow1, half, c)
#define KVC_QK_HI(J)                                                                \
    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka_hi[J], qb[4 + (J)], s, 0, 0, 0); \
    ka_lo[J] = read_k_operand<J>(krow2, half, c);                                   \
    read_v_operand<0>(va0[J], sv_next + voff[J])

    KVC_PIN();
    KVC_QK_LO(0); KVC_ARG(0); KVC_ARG(1); KVC_EXP(0);
    KVC_PIN();
    KVC_QK_LO(1); KVC_ARG(2); KVC_EXP(1); KVC_ROUND(0);
    KVC_PIN();
    KVC_QK_LO(2); KVC_ARG(3); KVC_EXP(2); KVC_ROUND(1); KVC_SUM(0);
    KVC_PIN();
    KVC_QK_LO(3); KVC_EXP(3); KVC_ROUND(2); KVC_SUM(1); KVC_ARG(4);
    KVC_PIN();
    KVC_ROUND(3);
    const uint4 pw0 = {w[0], w[1], w[2], w[3]};
    const bf16x8 pb0 = __builtin_bit_cast(bf16x8, pw0);

#define KVC_PV0(B)                                                                                        \
    if (MASKED) mask_v_operand<0>(va0[B], vlim_cur, half);                                                \
    st.acc[B] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_operand(va0[B]), pb0, st.acc[B], 0, 0, 0);     \
    read_v_operand<1>(va1[B], sv_cur + voff[B])
    KVC_PV0(0); KVC_SUM(2); KVC_ARG(5); KVC_EXP(4); KVC_SUM(3);
    KVC_PIN();
    KVC_PV0(1); KVC_ARG(6); KVC_EXP(5); KVC_ROUND(4);
    KVC_PIN();
    KVC_PV0(2); KVC_ARG(7); KVC_EXP(6); KVC_ROUND(5); KVC_SUM(4);
    KVC_PIN();
    KVC_PV0(3); KVC_EXP(7); KVC_ROUND(6); KVC_SUM(5);
    KVC_PIN();
    mid();  // the workgroup's half-turn barrier: the other group of wavefronts changes phase here too
    KVC_PIN();

    lookup();  // block id for the loads of the next turn: half a turn for the scalar load to return
    KVC_QK_HI(0); KVC_ROUND(7); KVC_SUM(6);
    KVC_PIN();
    const uint4 pw1 = {w[4], w[5], w[6], w[7]};
    const bf16x8 pb1 = __builtin_bit_cast(bf16x8, pw1);
    KVC_QK_HI(1); KVC_SUM(7);
    KVC_PIN();
    KVC_QK_HI(2);
    KVC_PIN();
    KVC_QK_HI(3);
    KVC_PIN();

    // chunks 12 .. 15 also take the raw scores of step next (masked if need be) and their max
#define KVC_PV1(B)                                                                                        \
    if (MASKED) mask_v_operand<1>(va1[B], vlim_cur, half);                                                \
    st.acc[B] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_operand(va1[B]), pb1, st.acc[B], 0, 0, 0)
    KVC_PV1(0);
    issue_k();
    KVC_PIN();
    KVC_PV1(1);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        x[v] = s[v];
        if (MASKED && 8 * (v >> 2) + 4 * half + (v & 3) >= limit_next) x[v] = -INFINITY;
    }
    const float m0 = max3(x[0], x[1], x[2]), m1 = max3(x[3], x[4], x[5]), m2 = max3(x[6], x[7], x[8]);
    KVC_PIN();
    KVC_PV1(2);
    issue_v();
    const float m3 = max3(x[9], x[10], x[11]), m4 = max3(x[12], x[13], x[14]);
    KVC_PIN();
    KVC_PV1(3);
    const float m5 = max3(m0, m1, m2), m6 = max3(m3, m4, x[15]);
    float lane_max;
    asm("v_max_f32 %0, %1, %2" : "=v"(lane_max) : "v"(m5), "v"(m6));
    rebase(st, lane_max, scale_log2e);
#undef KVC_ARG
#undef KVC_EXP
#undef KVC_SUM
#undef KVC_ROUND
#undef KVC_QK_LO
#undef KVC_QK_HI
#undef KVC_PV0
#undef KVC_PV1
}

// HEADS = 2: the 32 columns of a wavefront are 16 query rows x 2 heads of one KV head (even GQA
// groups); HEADS = 1: 32 query rows of one head.  GROUPS = 1: workgroups of four wavefronts, two
// per compute unit.  GROUPS = 2: workgroups of two groups of four wavefronts, one per compute
// unit; the groups run half a turn apart (see below).  Either way a SIMD holds two wavefronts.
template <bool SMALL, int GROUPS, int HEADS>
__global__ __launch_bounds__(256 * GROUPS, 3 - GROUPS) void pa_prefill_mfma32_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k_cache,
    const uint16_t *__restrict__ v_cache, const int32_t *__restrict__ block_tables,
    const int32_t *__restrict__ context_lens, const int32_t *__restrict__ q_start,
    uint16_t *__restrict__ out, PrefillParams p, int query_tiles, int fold_at) {
    __shared__ __attribute__((aligned(1024))) unsigned char s_k[kKStages][kStageBytes];
    __shared__ __attribute__((aligned(1024))) unsigned char s_v[kVStages][kStageBytes];
    constexpr int kWaveRows = 32 / HEADS;           // query rows of a wavefront: column c = kWaveRows * head + row
    constexpr int kTileRows = 4 * kWaveRows * GROUPS;  // query rows of a workgroup
    constexpr int kLoads = 2 / GROUPS;              // 1 KiB loads of K (and of V) per wavefront and step
    constexpr int kWavesPerTile = 2 * GROUPS;       // wavefronts that share a 16-row tile of a step

    // blockIdx.x = head chunk + chunks * (seq + num_seqs * order); the longest query tiles come
    // first, and from `fold_at` on the shortest: when every workgroup is resident at once, the two
    // that share a compute unit are then a long and a short one
    const int chunks = p.num_q_heads / HEADS;
    const int item = blockIdx.x;
    const int chunk = item % chunks;
    const int n = (item / chunks) % p.num_seqs;
    const int order = item / (chunks * p.num_seqs);
    const int qtile = order < fold_at ? query_tiles - 1 - order : order - fold_at;
    const int head0 = chunk * HEADS;
    const int kvh = head0 / p.group;

    const int S = context_lens[n];
    const int qs = q_start[n];
    const int Qn = q_start[n + 1] - qs;
    if (qtile * kTileRows >= Qn || Qn > S) return;  // uniform over the workgroup

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int group = wave >> 2;  // GROUPS = 2: wavefronts w and w + 4 share a SIMD; group 1 runs half a turn behind group 0
    const int half = lane >> 5, c = lane & 31;
    const int r = c % kWaveRows;  // query row of the column inside the wavefront's rows
    const int my_head = head0 + c / kWaveRows;

    // tiles and steps this workgroup walks (up to the position of its last query row)
    const int last_pos = S - Qn + min(Qn, qtile * kTileRows + kTileRows) - 1;
    const int wg_tiles = (last_pos >> 4) + 1;
    const int wg_steps = (wg_tiles + 1) / 2;
    const int32_t *table = block_tables + size_t(n) * p.max_blocks_per_seq;

    // wavefronts past the last query row still load and synchronise, they just never compute
    const int i0 = qtile * kTileRows + kWaveRows * wave;  // first query row of this wavefront
    const bool active = i0 < Qn;
    const int nrows = active ? min(kWaveRows, Qn - i0) : 1;
    const int row = min(r, nrows - 1);      // lanes past the last query row shadow it
    const int p0 = S - Qn + (active ? i0 : 0);  // position of row 0
    const int my_pos = p0 + row;
    const int wave_vis = p0 + nrows;        // tokens visible to some column of this wavefront
    const int free_steps = (p0 + 1) / kStepTokens;  // steps whose every token every column sees

    bf16x8 qb[8];
    {
        const uint16_t *qrow = q + (size_t(qs + (active ? i0 : 0) + row) * p.num_q_heads + my_head) * D + 8 * half;
#pragma unroll
        for (int j = 0; j < 8; ++j) qb[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(qrow + 16 * j));
    }

    ColumnState st;
    st.reset();

    // ---- this wavefront's share of a step's rows: 4 * kLoads consecutive rows of the 32 (inside
    // one 16-row tile of the step), kLoads loads of 4 rows for K and as many for V.  Lane l of
    // load i writes LDS chunk l % 16 of the share's row 4 * i + l / 16; the chunk it fetches for
    // that place follows from the stage layouts.
    const size_t head_bytes = size_t(p.block_size) * D * 2;
    const size_t block_bytes = head_bytes * p.num_kv_heads;
    const unsigned char *k_head = reinterpret_cast<const unsigned char *>(k_cache) + size_t(kvh) * head_bytes;
    const unsigned char *v_head = reinterpret_cast<const unsigned char *>(v_cache) + size_t(kvh) * head_bytes;
    const int sub_mask = (1 << p.tiles_per_block_log2) - 1;
    const int my_tile = wave / kWavesPerTile;       // tile of the step this wavefront loads from
    const int lrow = 4 * kLoads * (wave % kWavesPerTile) + (lane >> 4);  // row inside the tile of load 0 (load 1: + 4)
    const int lchunk = lane & 15;
    const uint32_t k_off = lrow * 256 + ((lchunk ^ lrow) << 4);
    const uint32_t k_off1 = (lrow + 4) * 256 + ((lchunk ^ (lrow + 4)) << 4);
    const uint32_t v_off = lrow * 256 + ((4 * (((lchunk >> 2) - lrow) & 3) + (lchunk & 3)) << 4);  // load 1: + 1024
    const uint32_t lds_k0 = uint32_t(reinterpret_cast<uintptr_t>(&s_k[0][0])) + 1024 * kLoads * wave;
    const uint32_t lds_v0 = uint32_t(reinterpret_cast<uintptr_t>(&s_v[0][0])) + 1024 * kLoads * wave;

    // Large blocks: the block id of the wavefront's tile is uniform, it comes through the scalar
    // cache one turn before the loads that use it.  Tiles past the last one repeat it (never
    // used unmasked).  Small blocks: a / b are the blocks of this lane's row in loads 0 / 1.
    struct Ids { int a, b; };
    auto ids_of = [&](int step) __attribute__((always_inline)) -> Ids {
        Ids id;
        if (SMALL) {
            const int tok = min((2 * step + my_tile) * kTileTokens + lrow, last_pos);
            id.a = table[tok >> p.block_size_log2];
            id.b = kLoads == 2 ? table[min(tok + 4, last_pos) >> p.block_size_log2] : 0;
        } else {
            const int t = min(2 * step + my_tile, wg_tiles - 1);
            id.a = __builtin_amdgcn_readfirstlane(table[t >> p.tiles_per_block_log2]);
            id.b = t & sub_mask;
        }
        return id;
    };
    // load this wavefront's K (V) rows of step `src` (the one `id` was looked up for) into a stage
    auto issue_rows = [&](const unsigned char *head, uint32_t dst, uint32_t off, uint32_t off1, int src, const Ids &id)
                          __attribute__((always_inline)) {
        if (SMALL) {
            const int tok = min((2 * src + my_tile) * kTileTokens + lrow, last_pos);
            load_lane_to_lds(head + size_t(id.a) * block_bytes + size_t(tok & (p.block_size - 1)) * 256 + (off & 255), dst);
            if (kLoads == 2) {
                const int tok1 = min(tok + 4, last_pos);
                load_lane_to_lds(head + size_t(id.b) * block_bytes + size_t(tok1 & (p.block_size - 1)) * 256 + (off1 & 255),
                                 dst + 1024);
            }
        } else {
            const unsigned char *tile = head + size_t(unsigned(id.a)) * block_bytes + size_t(id.b) * (kTileTokens * 256);
            if (kLoads == 2) load_rows_to_lds(tile, off, off1 - 1024, dst);
            else load_row_group_to_lds(tile, off, dst);
        }
    };
    auto issue_k = [&](int kst, int src, const Ids &id) __attribute__((always_inline)) {
        issue_rows(k_head, __builtin_amdgcn_readfirstlane(lds_k0 + kst * kStageBytes), k_off, k_off1, src, id);
    };
    auto issue_v = [&](int vst, int src, const Ids &id) __attribute__((always_inline)) {
        issue_rows(v_head, __builtin_amdgcn_readfirstlane(lds_v0 + vst * kStageBytes), v_off, v_off + 1024, src, id);
    };

    // Rows of step j live in K stage j % 4 and V stage j % 4.  Turn s requests the K rows of step
    // s+4 (over those of step s) and the V rows of step s+3 (over those of step s-1), multiplies
    // with operands of steps s+1 (K) and s (V) and reads operands of steps s+1, s+2 (K) and s, s+1
    // (V).  Before the barrier that ends it, a wavefront waits for its own loads of turn s-1 and
    // for its LDS reads.  The workgroup meets at a barrier twice per turn, and group 1 of its
    // wavefronts runs half a turn behind group 0: while one wavefront of a SIMD is in the first,
    // vector-heavy half of a turn the other is in the second, matrix-heavy half.  A stage is
    // overwritten, at the earliest, two barriers after the last wavefront has waited for its
    // reads of it, and read, at the earliest, after the barrier that follows the wait of the last
    // wavefront for its loads into it.  Past the last step the last one is loaded again (unused):
    // the loops stay branch free.
    Ids ids_v;
    {
        const Ids i0s = ids_of(0), i1s = ids_of(min(1, wg_steps - 1)), i2s = ids_of(min(2, wg_steps - 1));
        ids_v = ids_of(min(3, wg_steps - 1));
        issue_k(0, 0, i0s);
        issue_v(0, 0, i0s);
        issue_k(1, min(1, wg_steps - 1), i1s);
        issue_v(1, min(1, wg_steps - 1), i1s);
        issue_k(2, min(2, wg_steps - 1), i2s);
        issue_v(2, min(2, wg_steps - 1), i2s);
        issue_k(3, min(3, wg_steps - 1), ids_v);
    }
    Ids ids_k = ids_of(min(4, wg_steps - 1));
    wait_loads_but<kLoads>();  // steps 0 .. 2 have arrived
    // A use of the Q operand on this side of the barrier: without one the compiler sinks its
    // loads into the path of the active wavefronts, behind the barrier, where nothing hides them.
#pragma unroll
    for (int j = 0; j < 8; ++j) asm volatile("" : "+v"(qb[j]));
    __syncthreads();

    int s = 0;
    // PH = s % 4 (a literal in the unrolled loop: every LDS address of the turn is then a per-lane
    // register plus an immediate)
#define KVC_TURN_BEGIN(PH)                                                                        \
    const int ph = (PH);                                                                          \
    const int src_k = min(s + 4, wg_steps - 1), src_v = min(s + 3, wg_steps - 1);                 \
    const Ids idk = ids_k, idv = ids_v;                                                           \
    auto turn_k = [&]() __attribute__((always_inline)) { issue_k(ph, src_k, idk); };              \
    auto turn_v = [&]() __attribute__((always_inline)) {                                          \
        issue_v((ph + 3) & 3, src_v, idv);                                                        \
        ids_v = idk;                                                                              \
    };                                                                                            \
    auto turn_lookup = [&]() __attribute__((always_inline)) { ids_k = ids_of(min(s + 5, wg_steps - 1)); }
#define KVC_TURN_END()     \
    wait_loads_but<2 * kLoads>();   \
    turn_barrier()

    // Every wavefront of the workgroup passes one more barrier here, two per turn, and one to
    // set group 1 back by half a turn (group 0 passes its counterpart after its last turn).  A
    // wavefront without query rows only loads and synchronises.
    if (!active) {
        __syncthreads();
        if (GROUPS == 2 && group == 1) phase_barrier();
        for (; s < wg_steps; ++s) {
            KVC_TURN_BEGIN(s & 3);
            if (GROUPS == 2) phase_barrier();
            turn_lookup();
            turn_k();
            turn_v();
            KVC_TURN_END();
        }
        if (GROUPS == 2 && group == 0) phase_barrier();
        wait_loads_but<0>();
        return;
    }

    const unsigned char *k_lane = &s_k[0][0] + c * 256;  // this lane's K row inside a stage
    int voff[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) voff[b] = v_lane_offset(b, half, c);
    float x[16];
    bf16x8 ka_lo[4];
    uint2 va0[4][2];
    {  // scores of step 0, then the operands turn 0 starts from
        floatx16 sc;
#pragma unroll
        for (int v = 0; v < 16; ++v) sc[v] = 0.f;
        bf16x8 ka[8];
        ka[0] = read_k_operand<0>(k_lane, half, c); ka[1] = read_k_operand<1>(k_lane, half, c);
        ka[2] = read_k_operand<2>(k_lane, half, c); ka[3] = read_k_operand<3>(k_lane, half, c);
        ka[4] = read_k_operand<4>(k_lane, half, c); ka[5] = read_k_operand<5>(k_lane, half, c);
        ka[6] = read_k_operand<6>(k_lane, half, c); ka[7] = read_k_operand<7>(k_lane, half, c);
#pragma unroll
        for (int j = 0; j < 8; ++j) sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[j], qb[j], sc, 0, 0, 0);
        rebase(st, take_scores<true>(x, sc, my_pos + 1, half), p.scale_log2e);
        const unsigned char *krow = k_lane + kStageBytes;
        ka_lo[0] = read_k_operand<0>(krow, half, c); ka_lo[1] = read_k_operand<1>(krow, half, c);
        ka_lo[2] = read_k_operand<2>(krow, half, c); ka_lo[3] = read_k_operand<3>(krow, half, c);
#pragma unroll
        for (int b = 0; b < 4; ++b) read_v_operand<0>(va0[b], &s_v[0][0] + voff[b]);
    }
    __syncthreads();  // K stage 0 has been read: turn 0 may load step 4 over it
    if (GROUPS == 2 && group == 1) phase_barrier();

    // The turns below the diagonal first (no mask), unrolled by the four phases of the stage
    // rings, then the one to three turns that the causal mask touches.
    const unsigned char *v_base = &s_v[0][0];
    auto mid = []() __attribute__((always_inline)) {
        if (GROUPS == 2) phase_barrier();
    };
#define KVC_TURN(MASKED, PH, VLIM, LIMIT)                                                                      \
    {                                                                                                          \
        KVC_TURN_BEGIN(PH);                                                                                    \
        pipeline_turn<MASKED>(st, x, ka_lo, va0, k_lane + ((ph + 1) & 3) * kStageBytes,                        \
                              k_lane + ((ph + 2) & 3) * kStageBytes, v_base + ph * kStageBytes,                \
                              v_base + ((ph + 1) & 3) * kStageBytes, voff, qb, p.scale_log2e, VLIM, LIMIT,     \
                              half, c, turn_k, turn_v, mid, turn_lookup);                                      \
        KVC_TURN_END();                                                                                        \
        ++s;                                                                                                   \
    }
    const int plain_turns = min(max(free_steps - 1, 0), wg_steps);
    while (s + 4 <= plain_turns) {
        KVC_TURN(false, 0, kStepTokens, kStepTokens)
        KVC_TURN(false, 1, kStepTokens, kStepTokens)
        KVC_TURN(false, 2, kStepTokens, kStepTokens)
        KVC_TURN(false, 3, kStepTokens, kStepTokens)
    }
    while (s < plain_turns) KVC_TURN(false, s & 3, kStepTokens, kStepTokens)
    // steps past the last token that any row of this wavefront sees carry no weight for it: it
    // only loads and synchronises during the workgroup's remaining turns
    const int live_turns = min(wg_steps, (wave_vis + kStepTokens - 1) / kStepTokens);
    while (s < live_turns) KVC_TURN(true, s & 3, wave_vis - s * kStepTokens, my_pos + 1 - (s + 1) * kStepTokens)
    for (; s < wg_steps; ++s) {
        KVC_TURN_BEGIN(s & 3);
        if (GROUPS == 2) phase_barrier();
        turn_lookup();
        turn_k();
        turn_v();
        KVC_TURN_END();
    }
#undef KVC_TURN
#undef KVC_TURN_BEGIN
#undef KVC_TURN_END
    if (GROUPS == 2 && group == 0) phase_barrier();
    wait_loads_but<0>();  // nothing may still be landing in LDS when the workgroup's LDS is handed on

    // lane (half, c) holds O[query row i0 + r][my_head][32*b + 8*a + 4*half .. +3] in acc[b][4a .. 4a+3]
    const float inv = 1.0f / sum_over_halves(st.lsum);
    if (r < nrows) {
        uint16_t *dst = out + (size_t(qs + i0 + r) * p.num_q_heads + my_head) * D + 4 * half;
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                uint2 w;
                w.x = pack_bf16(st.acc[b][4 * a] * inv, st.acc[b][4 * a + 1] * inv);
                w.y = pack_bf16(st.acc[b][4 * a + 2] * inv, st.acc[b][4 * a + 3] * inv);
                *reinterpret_cast<uint2 *>(dst + 32 * b + 8 * a) = w;
            }
    }
}

}  // namespace

// Needs a positive scale (the max is taken over raw scores).  heads_per_chunk = 2: two heads of a
// KV head per wavefront (even group sizes); 1: one head, twice the query rows.
hipError_t launch_prefill_mfma32(const void *q, const void *k_cache, const void *v_cache,
                                 const int32_t *block_tables, const int32_t *context_lens,
                                 const int32_t *q_start, void *out, const PrefillParams &p,
                                 hipStream_t stream) {
    const auto *qq = static_cast<const uint16_t *>(q);
    const auto *kk = static_cast<const uint16_t *>(k_cache);
    const auto *vv = static_cast<const uint16_t *>(v_cache);
    auto *oo = static_cast<uint16_t *>(out);
    const int heads = p.heads_per_chunk;
    const int rows64 = 2 / heads;  // 64-row units in the query rows of four wavefronts
    // Two groups per workgroup pay off (by a few percent) for long recomputations with workgroups
    // enough to keep every compute unit busy for several rounds; up to about 2048 query rows per
    // sequence the finer grain of four-wavefront workgroups wins, whatever the batch (measured).
    const auto tiles_of = [&](int groups) { return (p.max_query_tiles + rows64 * groups - 1) / (rows64 * groups); };
    const int64_t wide_grid = int64_t(p.num_q_heads / heads) * p.num_seqs * tiles_of(2);
    const bool wide = wide_grid >= 2 * 256 && p.max_query_tiles >= 48;
    const bool small = p.block_size < kTileTokens;
    const int query_tiles = tiles_of(wide ? 2 : 1);  // max_query_tiles counts 64-row tiles
    // A grid that fits the device at once (two workgroups of four wavefronts per compute unit)
    // gets the second half of its query tiles in rising order (a few percent on one short request).
    const int64_t grid = int64_t(p.num_q_heads / heads) * p.num_seqs * query_tiles;
    const int fold_at = (!wide && grid <= 2 * 256) ? (query_tiles + 1) / 2 : query_tiles;
    const dim3 g(unsigned(int64_t(p.num_q_heads / heads) * p.num_seqs * query_tiles)), b(wide ? 512 : 256);
#define KVC_LAUNCH(SMALL, GROUPS, HEADS)                                                                        \
    pa_prefill_mfma32_kernel<SMALL, GROUPS, HEADS><<<g, b, 0, stream>>>(qq, kk, vv, block_tables, context_lens, \
                                                                         q_start, oo, p, query_tiles, fold_at)
#define KVC_LAUNCH_HEADS(SMALL, GROUPS)           \
    do {                                          \
        if (heads == 2) KVC_LAUNCH(SMALL, GROUPS, 2); \
        else KVC_LAUNCH(SMALL, GROUPS, 1);        \
    } while (0)
    if (wide && small) KVC_LAUNCH_HEADS(true, 2);
    else if (wide) KVC_LAUNCH_HEADS(false, 2);
    else if (small) KVC_LAUNCH_HEADS(true, 1);
    else KVC_LAUNCH_HEADS(false, 1);
#undef KVC_LAUNCH_HEADS
#undef KVC_LAUNCH
    return hipGetLastError();
}

}  // namespace kvc
