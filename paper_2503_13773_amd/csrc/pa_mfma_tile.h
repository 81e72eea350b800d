// One 16-token tile of decode attention on the gfx950 matrix cores, shared by the MFMA
// partial kernels (bf16, head_dim 128).  Lane = 16*quad + r throughout.
//
//   S[token][head]  = K[16 x 128] . Q^T[128 x 16]       4 x v_mfma_f32_16x16x32_bf16
//       A operand: lane holds K[token r][32j + 8*quad .. +7]; B operand: the same dims of
//       Q[head r] (zero for r >= group size).
//   softmax over the C layout: lane holds S[token 4*quad + i][head r], i < 4.  The max over
//       the tile's tokens is 3 in-lane max + 2 cross-quad shuffles; exp2 with
//       scale*log2(e) folded into the scores.
//   O^T[dim][head] += V^T[128 x 16] . P^T[16 x 16]       8 x v_mfma_f32_16x16x16_bf16
//       B operand P^T is exactly the C layout of S (tokens 4*quad + i, head r): no data
//       movement.  A operand needs 4 tokens of one dim per lane: V is loaded row-wise (lane
//       reads dims 8r..8r+7 of tokens 4*quad + i, so 16 lanes read one full 256-byte row)
//       and the 4x8 patch is transposed in registers with 16 v_perm_b32.  MFMA number e
//       then yields dims {8*row + e}: the lane ends up with O[head r][32*quad .. +31],
//       element 8i + e in acc[e][i].
//   Everything attached to a head (max, sum, rescale factor, accumulator) lives in the
//   lanes with that r, so the online-softmax rescale needs no cross-lane traffic.
//
// Softmax weights are rounded to bf16 for the P.V product and the normaliser sums the
// *rounded* weights, so the weights that multiply V still sum to the normaliser.  Rows
// past the context in a ragged tile get score -inf and their V data is zeroed, so NaN
// or Inf stored there cannot reach the output.
#pragma once

#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

namespace kvc {
namespace mfma {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int D = 128;
constexpr int kTileTokens = 16;
constexpr int kTileElems = kTileTokens * D;  // 2048 bf16 = 4 KiB

__device__ inline uint16_t f32_to_bf16_rne(float x) {
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return uint16_t((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return uint16_t(u >> 16);
}

// two fp32 -> packed bf16 pair (round to nearest even), low half = a
__device__ inline uint32_t pack_bf16(float a, float b) {
    const floatx2 f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

// Online-softmax state of the (up to 16) heads of one KV head, as held by one wavefront.
struct HeadState {
    floatx4 acc[8];
    float m;  // running max of the scaled scores (base-2 units) of head r
    float l;  // running sum of weights; partial over this lane's tokens until finish()

    __device__ inline void reset() {
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = floatx4{0.f, 0.f, 0.f, 0.f};
        m = -INFINITY;
        l = 0.f;
    }
    // sum l over the 4 quads (the max is already common to them)
    __device__ inline void finish() {
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
    }
};

// Q as the B operand of S = K.Q^T: lane (quad, r) holds Q[head r][32j + 8*quad .. +7].
// `qrow` points at Q[head r of this KV head's group]; lanes with active == false get zeros.
__device__ inline void load_q_operand(bf16x8 (&qb)[4], const uint16_t *qrow, int quad, bool active) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        uint4 w = {0u, 0u, 0u, 0u};
        if (active) w = *reinterpret_cast<const uint4 *>(qrow + 32 * j + 8 * quad);
        qb[j] = __builtin_bit_cast(bf16x8, w);
    }
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// 16-byte load of KV data.  K and V are streamed once per step, so the load carries the
// non-temporal hint (no reuse expected in L2 / the memory-side cache).
__device__ inline uint4 load16_stream(const uint16_t *p) {
    return __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p)));
}

// Issue the 8 x 16-byte loads of one tile: K straight into the A-operand layout (16 rows x
// 64 bytes per instruction), V row-wise (4 full rows per instruction).
__device__ inline void issue_tile_direct(uint4 (&kr)[4], uint4 (&vr)[4], const uint16_t *kp,
                                         const uint16_t *vp, int quad, int r) {
#pragma unroll
    for (int j = 0; j < 4; ++j) kr[j] = load16_stream(kp + r * D + 32 * j + 8 * quad);
#pragma unroll
    for (int i = 0; i < 4; ++i) vr[i] = load16_stream(vp + (4 * quad + i) * D + 8 * r);
}

// One tile: scores, online softmax update, P.V accumulation.  `valid` = tokens of the tile
// that lie inside the context (16 for a full tile, wavefront-uniform).
__device__ inline void compute_tile(HeadState &st, const bf16x8 (&ka)[4], uint4 (&vr)[4],
                                    const bf16x8 (&qb)[4], float scale_log2e, int valid, int quad) {
    floatx4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 4; ++j) s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[j], qb[j], s, 0, 0, 0);

    float sv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) sv[i] = s[i] * scale_log2e;
    if (valid < kTileTokens) {  // ragged tile
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (4 * quad + i >= valid) {
                sv[i] = -INFINITY;
                vr[i] = uint4{0u, 0u, 0u, 0u};
            }
        }
    }
    float mx = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(st.m, mx);  // finite: every tile has at least one valid token
    const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);
    st.m = m_new;
    float pf[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) pf[i] = __builtin_amdgcn_exp2f(sv[i] - m_new);
    const uint32_t p01 = pack_bf16(pf[0], pf[1]);
    const uint32_t p23 = pack_bf16(pf[2], pf[3]);
    const float psum = (__uint_as_float(p01 << 16) + __uint_as_float(p01 & 0xffff0000u)) +
                       (__uint_as_float(p23 << 16) + __uint_as_float(p23 & 0xffff0000u));
    st.l = fmaf(st.l, alpha, psum);
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) st.acc[e] *= alpha;
    }
    const uint2 pw = {p01, p23};
    const shortx4 pb = __builtin_bit_cast(shortx4, pw);

    const uint32_t v0[4] = {vr[0].x, vr[0].y, vr[0].z, vr[0].w};
    const uint32_t v1[4] = {vr[1].x, vr[1].y, vr[1].z, vr[1].w};
    const uint32_t v2[4] = {vr[2].x, vr[2].y, vr[2].z, vr[2].w};
    const uint32_t v3[4] = {vr[3].x, vr[3].y, vr[3].z, vr[3].w};
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        // dword w of a row holds dims 8r+2w (low half) and 8r+2w+1 (high half)
        const uint2 lo = {__builtin_amdgcn_perm(v1[w], v0[w], 0x05040100u),
                          __builtin_amdgcn_perm(v3[w], v2[w], 0x05040100u)};
        const uint2 hi = {__builtin_amdgcn_perm(v1[w], v0[w], 0x07060302u),
                          __builtin_amdgcn_perm(v3[w], v2[w], 0x07060302u)};
        st.acc[2 * w] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(shortx4, lo), pb, st.acc[2 * w], 0, 0, 0);
        st.acc[2 * w + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(shortx4, hi), pb, st.acc[2 * w + 1], 0, 0, 0);
    }
}

// Several 16-column groups against the same K/V tile (prefill: the groups are the query heads
// that share the KV head, their 16 columns are 16 query positions).  The K operand and the
// register transpose of V are shared by the groups; each group keeps its own softmax state.
// `valid` = tokens of the tile inside the context (wavefront-uniform, zeroes V rows past it);
// `limit` = tokens of the tile visible to this lane's column (causal mask; may be <= 0, the
// column must already hold a finite running max then).
template <int NG>
__device__ inline void compute_tile_groups(HeadState (&st)[NG], const bf16x8 (&ka)[4], uint4 (&vr)[4],
                                           const bf16x8 (&qb)[NG][4], float scale_log2e, int valid,
                                           int limit, int quad) {
    if (valid < kTileTokens) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (4 * quad + i >= valid) vr[i] = uint4{0u, 0u, 0u, 0u};
    }
    shortx4 pb[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        floatx4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j) s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[j], qb[g][j], s, 0, 0, 0);
        float sv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) sv[i] = (4 * quad + i < limit) ? s[i] * scale_log2e : -INFINITY;
        float mx = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(st[g].m, mx);
        const float alpha = __builtin_amdgcn_exp2f(st[g].m - m_new);
        st[g].m = m_new;
        float pf[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) pf[i] = __builtin_amdgcn_exp2f(sv[i] - m_new);
        const uint32_t p01 = pack_bf16(pf[0], pf[1]);
        const uint32_t p23 = pack_bf16(pf[2], pf[3]);
        const float psum = (__uint_as_float(p01 << 16) + __uint_as_float(p01 & 0xffff0000u)) +
                           (__uint_as_float(p23 << 16) + __uint_as_float(p23 & 0xffff0000u));
        st[g].l = fmaf(st[g].l, alpha, psum);
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) st[g].acc[e] *= alpha;
        }
        const uint2 pw = {p01, p23};
        pb[g] = __builtin_bit_cast(shortx4, pw);
    }
    const uint32_t v0[4] = {vr[0].x, vr[0].y, vr[0].z, vr[0].w};
    const uint32_t v1[4] = {vr[1].x, vr[1].y, vr[1].z, vr[1].w};
    const uint32_t v2[4] = {vr[2].x, vr[2].y, vr[2].z, vr[2].w};
    const uint32_t v3[4] = {vr[3].x, vr[3].y, vr[3].z, vr[3].w};
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const uint2 lo = {__builtin_amdgcn_perm(v1[w], v0[w], 0x05040100u),
                          __builtin_amdgcn_perm(v3[w], v2[w], 0x05040100u)};
        const uint2 hi = {__builtin_amdgcn_perm(v1[w], v0[w], 0x07060302u),
                          __builtin_amdgcn_perm(v3[w], v2[w], 0x07060302u)};
        const shortx4 alo = __builtin_bit_cast(shortx4, lo), ahi = __builtin_bit_cast(shortx4, hi);
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            st[g].acc[2 * w] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(alo, pb[g], st[g].acc[2 * w], 0, 0, 0);
            st[g].acc[2 * w + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ahi, pb[g], st[g].acc[2 * w + 1], 0, 0, 0);
        }
    }
}

}  // namespace mfma
}  // namespace kvc
