// Causal attention of many query positions per sequence over the block-allocated KV cache on
// the matrix cores (gfx950, bf16, head_dim 128, block_size a multiple of 16): the recomputation
// path of a preempted request (prefill re-run over prompt + generated tokens, quadratic in the
// sequence length: paper Section 2.5 and 3.5) and chunked prefill.
//
// Bound: MFMA (4 * D * Hq * sum over query rows of (position + 1) flops), not HBM: every K/V
// tile is used by 16 query positions x the query heads that share the KV head.
//
// One workgroup = (sequence, chunk of NG query heads sharing one KV head, 64 consecutive query
// rows); each of its 4 wavefronts owns 16 query rows and walks the K/V tiles from token 0 to
// its last visible token with the same two-register-set software pipeline as the decode
// kernels.  Per tile a wavefront computes, for every one of its NG heads, S = K . Q^T with the
// 16 query rows as the 16 columns of the MFMA tile, an online softmax per column, and
// O^T += V^T . P^T (per-tile code in pa_mfma_tile.h); the K operand and the register
// transpose of V are shared by the NG heads.  The causal mask only bites in the one or two
// tiles on the diagonal; it is a per-lane row limit.  Token 0 is visible to every query row and
// tiles are walked in order, so every column has a finite running max after the first tile.
// Workgroups with the most tiles (the last query rows) are dispatched first.
//
// The block ids of the sequence are staged in LDS once per workgroup (contexts up to 32768
// tokens).
#include <math.h>

#include "kvc_internal.h"
#include "pa_mfma_tile.h"

namespace kvc {

namespace {

using namespace mfma;

constexpr int kMaxPrefillTiles = 2048;  // 32768 tokens

template <int NG>
__global__ __launch_bounds__(kThreads, NG <= 2 ? 2 : 1) void pa_prefill_mfma_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k_cache,
    const uint16_t *__restrict__ v_cache, const int32_t *__restrict__ block_tables,
    const int32_t *__restrict__ context_lens, const int32_t *__restrict__ q_start,
    uint16_t *__restrict__ out, PrefillParams p) {
    __shared__ int s_blk[kMaxPrefillTiles];

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
    if (qtile * 64 >= Qn || Qn > S) return;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int quad = lane >> 4, r = lane & 15;

    // stage the block ids of every tile this workgroup can touch
    const int last_pos = S - Qn + min(Qn, qtile * 64 + 64) - 1;
    const int wg_tiles = min((last_pos >> 4) + 1, kMaxPrefillTiles);
    const int32_t *table = block_tables + size_t(n) * p.max_blocks_per_seq;
    for (int t = tid; t < wg_tiles; t += kThreads) s_blk[t] = table[t >> p.tiles_per_block_log2];
    __syncthreads();

    const int i0 = qtile * 64 + 16 * wave;  // first query row of this wavefront
    if (i0 >= Qn) return;
    const int ncols = min(16, Qn - i0);
    const int col = min(r, ncols - 1);      // lanes past the last query row shadow it
    const int p0 = S - Qn + i0;             // position of column 0
    const int my_pos = p0 + col;
    const int nt = min(((p0 + ncols - 1) >> 4) + 1, wg_tiles);  // tiles 0 .. nt-1

    bf16x8 qb[NG][4];
#pragma unroll
    for (int g = 0; g < NG; ++g)
        load_q_operand(qb[g], q + (size_t(qs + i0 + col) * p.num_q_heads + head0 + g) * D, quad, true);

    HeadState st[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) st[g].reset();

    const size_t head_elems = size_t(p.block_size) * D;
    const size_t block_elems = head_elems * p.num_kv_heads;
    const int sub_mask = (1 << p.tiles_per_block_log2) - 1;

    auto issue = [&](uint4(&kr)[4], uint4(&vr)[4], int kt) __attribute__((always_inline)) {
        const int blk = __builtin_amdgcn_readfirstlane(s_blk[kt]);
        const size_t base = size_t(blk) * block_elems + size_t(kvh) * head_elems + size_t(kt & sub_mask) * kTileElems;
        // K/V tiles are re-read by the other wavefronts and head chunks: plain (cached) loads
#pragma unroll
        for (int j = 0; j < 4; ++j) kr[j] = *reinterpret_cast<const uint4 *>(k_cache + base + r * D + 32 * j + 8 * quad);
#pragma unroll
        for (int i = 0; i < 4; ++i) vr[i] = *reinterpret_cast<const uint4 *>(v_cache + base + (4 * quad + i) * D + 8 * r);
    };
    auto compute = [&](uint4(&kr)[4], uint4(&vr)[4], int kt) __attribute__((always_inline)) {
        bf16x8 ka[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) ka[j] = __builtin_bit_cast(bf16x8, kr[j]);
        compute_tile_groups<NG>(st, ka, vr, qb, p.scale_log2e, S - kt * kTileTokens,
                                my_pos + 1 - kt * kTileTokens, quad);
    };

    uint4 kA[4], vA[4], kB[4], vB[4];
    issue(kA, vA, 0);
    int kt = 0;
    for (; kt + 2 < nt; kt += 2) {
        issue(kB, vB, kt + 1);
        compute(kA, vA, kt);
        issue(kA, vA, kt + 2);
        compute(kB, vB, kt + 1);
    }
    if (kt + 1 < nt) {
        issue(kB, vB, kt + 1);
        compute(kA, vA, kt);
        compute(kB, vB, kt + 1);
    } else {
        compute(kA, vA, kt);
    }

    // lane (quad, r < ncols) holds O[query row i0 + r][head0 + g][32*quad .. +31]
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        st[g].finish();
        if (r < ncols) {
            const float inv = 1.0f / st[g].l;
            uint16_t *dst = out + (size_t(qs + i0 + r) * p.num_q_heads + head0 + g) * D + 32 * quad;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                uint4 w;
                w.x = pack_bf16(st[g].acc[0][i] * inv, st[g].acc[1][i] * inv);
                w.y = pack_bf16(st[g].acc[2][i] * inv, st[g].acc[3][i] * inv);
                w.z = pack_bf16(st[g].acc[4][i] * inv, st[g].acc[5][i] * inv);
                w.w = pack_bf16(st[g].acc[6][i] * inv, st[g].acc[7][i] * inv);
                *reinterpret_cast<uint4 *>(dst + 8 * i) = w;
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
    const unsigned grid = unsigned(int64_t(p.num_q_heads / ng) * p.num_seqs * p.max_query_tiles);
    const dim3 g(grid), b(kThreads);
    if (ng == 4) pa_prefill_mfma_kernel<4><<<g, b, 0, stream>>>(qq, kk, vv, block_tables, context_lens, q_start, oo, p);
    else if (ng == 2) pa_prefill_mfma_kernel<2><<<g, b, 0, stream>>>(qq, kk, vv, block_tables, context_lens, q_start, oo, p);
    else pa_prefill_mfma_kernel<1><<<g, b, 0, stream>>>(qq, kk, vv, block_tables, context_lens, q_start, oo, p);
    return hipGetLastError();
}

}  // namespace kvc
