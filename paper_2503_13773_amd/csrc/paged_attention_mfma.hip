// Split-K partial kernel of paged decode attention on the matrix cores with FIXED-LENGTH
// partitions (gfx950, bf16, head_dim 128, block_size a multiple of 16, up to 16 query heads
// per KV head).
//
// One workgroup = one (sequence, KV head, partition of the context); all query heads that
// share the KV head ride along as the 16 columns of an MFMA tile, so K and V are read from
// HBM exactly once per KV head (grouped-query heads form a real dense tile: 16 tokens x
// 128 dims x G heads).  The four wavefronts take 16-token tiles round-robin, each with its
// own online softmax; they are merged through LDS at the end.  The per-tile arithmetic is
// in pa_mfma_tile.h.
//
// K reaches the MFMA operand layout either straight from HBM (KLDS = false) or by fully
// coalesced 1 KiB loads, a 16-byte XOR-swizzled write to LDS and a conflict-free 16-byte
// read back (KLDS = true).
#include <math.h>

#include "kvc_internal.h"
#include "pa_mfma_tile.h"

namespace kvc {

namespace {

using namespace mfma;

template <int GP, bool KLDS>
__global__ __launch_bounds__(kThreads, 3) void pa_partial_mfma_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k_cache,
    const uint16_t *__restrict__ v_cache, const int32_t *__restrict__ block_tables,
    const int32_t *__restrict__ context_lens, uint16_t *__restrict__ out, Workspace ws,
    AttnParams p, int tiles_per_block_log2) {
    // LDS: per-wavefront K staging (4 KiB each, KLDS only), reused after a barrier for the
    // cross-wavefront merge: acc [4][GP][128] fp32, then m [4][16], l [4][16].
    constexpr int kAccFloats = kWaves * GP * D;
    constexpr int kMergeBytes = (kAccFloats + 2 * kWaves * 16) * 4;
    constexpr int kStageBytes = KLDS ? kWaves * kTileElems * 2 : 0;
    constexpr int kSmemBytes = kMergeBytes > kStageBytes ? kMergeBytes : kStageBytes;
    __shared__ __attribute__((aligned(16))) unsigned char smem[kSmemBytes];

    // blockIdx.x = kv_head + num_kv_heads * (seq + num_seqs * partition).  Workgroups go
    // round-robin over the 8 XCDs, so with 8 KV heads every XCD's L2 serves one KV head:
    // blocks shared between sequences (a common prefix) are fetched into one L2 only.
    const int item = blockIdx.x;
    const int kvh = item % p.num_kv_heads;
    const int seq = (item / p.num_kv_heads) % p.num_seqs;
    const int part = item / (p.num_kv_heads * p.num_seqs);
    const int G = p.group;
    const int head0 = kvh * G;
    const int ctx = min(context_lens[seq], p.max_context_len);
    const int tid = threadIdx.x;

    if (ctx <= 0) {  // empty context: zeros, written by partition 0
        if (part == 0)
            for (int i = tid; i < G * D; i += kThreads)
                out[(size_t(seq) * p.num_q_heads + head0) * D + i] = 0;
        return;
    }
    const int tok0 = part * p.partition_tokens;
    if (tok0 >= ctx) return;
    const int tok1 = min(ctx, tok0 + p.partition_tokens);

    const int wave = tid >> 6, lane = tid & 63;
    const int quad = lane >> 4, r = lane & 15;

    const int ntile = (tok1 - tok0 + kTileTokens - 1) >> 4;
    const int tile0 = tok0 >> 4;
    const int my_n = wave < ntile ? (ntile - wave + kWaves - 1) / kWaves : 0;  // <= 64

    // physical block of my i-th tile sits in lane i
    const int32_t *table = block_tables + size_t(seq) * p.max_blocks_per_seq;
    int my_blk = 0;
    if (lane < my_n) my_blk = table[(tile0 + wave + kWaves * lane) >> tiles_per_block_log2];

    bf16x8 qb[4];
    load_q_operand(qb, q + (size_t(seq) * p.num_q_heads + head0 + (r < G ? r : 0)) * D, quad, r < G);

    HeadState st;
    st.reset();

    const size_t head_elems = size_t(p.block_size) * D;
    const size_t block_elems = head_elems * p.num_kv_heads;
    const int sub_mask = (1 << tiles_per_block_log2) - 1;
    unsigned char *stage = smem + wave * (kTileElems * 2);

    auto issue = [&](uint4(&kr)[4], uint4(&vr)[4], int it) __attribute__((always_inline)) {
        const int blk = __builtin_amdgcn_readlane(my_blk, it);
        const int gt = tile0 + wave + kWaves * it;
        const size_t base = size_t(blk) * block_elems + kvh * head_elems + size_t(gt & sub_mask) * kTileElems;
        const uint16_t *kp = k_cache + base;
        const uint16_t *vp = v_cache + base;
        if (KLDS) {
#pragma unroll
            for (int i = 0; i < 4; ++i) kr[i] = load16_stream(kp + i * 512 + lane * 8);
#pragma unroll
            for (int i = 0; i < 4; ++i) vr[i] = load16_stream(vp + (4 * quad + i) * D + 8 * r);
        } else {
            issue_tile_direct(kr, vr, kp, vp, quad, r);
        }
    };

    auto compute = [&](uint4(&kr)[4], uint4(&vr)[4], int it) __attribute__((always_inline)) {
        const int gt = tile0 + wave + kWaves * it;
        bf16x8 ka[4];
        if (KLDS) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {  // loaded: token 4i + quad, 16-byte chunk r
                const int t = 4 * i + quad;
                *reinterpret_cast<uint4 *>(stage + t * 256 + ((r ^ t) & 15) * 16) = kr[i];
            }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int j = 0; j < 4; ++j) {  // wanted: token r, chunk 4j + quad
                const int c = 4 * j + quad;
                ka[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(stage + r * 256 + ((c ^ r) & 15) * 16));
            }
            __builtin_amdgcn_wave_barrier();
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) ka[j] = __builtin_bit_cast(bf16x8, kr[j]);
        }
        compute_tile(st, ka, vr, qb, p.scale_log2e, tok1 - gt * kTileTokens, quad);
    };

    // Two register sets, software-pipelined; the steady-state loop is branch-free so that the
    // compiler's wait counts keep the 8 newest loads in flight, the 1- or 2-tile tail is peeled.
    uint4 kA[4], vA[4], kB[4], vB[4];
    if (my_n > 0) {
        issue(kA, vA, 0);
        int it = 0;
        for (; it + 2 < my_n; it += 2) {
            issue(kB, vB, it + 1);
            compute(kA, vA, it);
            issue(kA, vA, it + 2);
            compute(kB, vB, it + 1);
        }
        if (it + 1 < my_n) {
            issue(kB, vB, it + 1);
            compute(kA, vA, it);
            compute(kB, vB, it + 1);
        } else {
            compute(kA, vA, it);
        }
    }

    st.finish();

    float *sm_acc = reinterpret_cast<float *>(smem);  // [kWaves][GP][D]
    float *sm_m = sm_acc + kAccFloats;                // [kWaves][16]
    float *sm_l = sm_m + kWaves * 16;                 // [kWaves][16]
    if (KLDS) __syncthreads();  // staging areas are about to be overwritten
    if (r < G) {
        float *dst = sm_acc + (size_t(wave) * GP + r) * D + 32 * quad;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            *reinterpret_cast<float4 *>(dst + 8 * i) = float4{st.acc[0][i], st.acc[1][i], st.acc[2][i], st.acc[3][i]};
            *reinterpret_cast<float4 *>(dst + 8 * i + 4) = float4{st.acc[4][i], st.acc[5][i], st.acc[6][i], st.acc[7][i]};
        }
        if (quad == 0) {
            sm_m[wave * 16 + r] = st.m;
            sm_l[wave * 16 + r] = st.l;
        }
    }
    __syncthreads();

    const bool single = ctx <= p.partition_tokens;
    for (int i = tid; i < G * D; i += kThreads) {
        const int g = i >> 7, d = i & (D - 1);
        float M = sm_m[g];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) M = fmaxf(M, sm_m[w * 16 + g]);
        float L = 0.f, A = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float wgt = __builtin_amdgcn_exp2f(sm_m[w * 16 + g] - M);  // idle wavefront: exp2(-inf) = 0
            L = fmaf(wgt, sm_l[w * 16 + g], L);
            A = fmaf(wgt, sm_acc[(size_t(w) * GP + g) * D + d], A);
        }
        const size_t row = size_t(seq) * p.num_q_heads + head0 + g;
        if (single) {
            out[row * D + d] = f32_to_bf16_rne(A / L);
        } else {
            const size_t slot = row * p.max_partitions + part;
            ws.acc[slot * D + d] = A;
            if (d == 0) {
                ws.ml[slot * 2] = M;
                ws.ml[slot * 2 + 1] = L;
            }
        }
    }
}

template <int GP>
void launch_gp(bool klds, const void *q, const void *k, const void *v, const int32_t *bt,
               const int32_t *cl, void *out, Workspace ws, const AttnParams &p, int tpb_log2,
               int grid, hipStream_t stream) {
    const auto *qq = static_cast<const uint16_t *>(q);
    const auto *kk = static_cast<const uint16_t *>(k);
    const auto *vv = static_cast<const uint16_t *>(v);
    auto *oo = static_cast<uint16_t *>(out);
    if (klds)
        pa_partial_mfma_kernel<GP, true><<<dim3(grid), dim3(kThreads), 0, stream>>>(qq, kk, vv, bt, cl, oo, ws, p, tpb_log2);
    else
        pa_partial_mfma_kernel<GP, false><<<dim3(grid), dim3(kThreads), 0, stream>>>(qq, kk, vv, bt, cl, oo, ws, p, tpb_log2);
}

}  // namespace

hipError_t launch_partial_mfma(const void *q, const void *k_cache, const void *v_cache,
                               const int32_t *block_tables, const int32_t *context_lens, void *out,
                               Workspace ws, const AttnParams &p, int grid, hipStream_t stream) {
    int tpb_log2 = 0;
    while ((16 << tpb_log2) < p.block_size) ++tpb_log2;
    const bool klds = p.k_via_lds != 0;
    if (p.group <= 4) launch_gp<4>(klds, q, k_cache, v_cache, block_tables, context_lens, out, ws, p, tpb_log2, grid, stream);
    else if (p.group <= 8) launch_gp<8>(klds, q, k_cache, v_cache, block_tables, context_lens, out, ws, p, tpb_log2, grid, stream);
    else launch_gp<16>(klds, q, k_cache, v_cache, block_tables, context_lens, out, ws, p, tpb_log2, grid, stream);
    return hipGetLastError();
}

}  // namespace kvc
