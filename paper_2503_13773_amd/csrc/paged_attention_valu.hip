// Split-K partial kernel of paged decode attention on the vector ALUs (gfx950).
//
// Computes, for one (sequence, chunk of query heads sharing a KV head, partition of the
// context), the un-normalised softmax-weighted sum of V rows together with the running
// max and sum, reading K and V through the block table (block-allocated KV cache:
// paper Section 1 and 3.3.1).  It serves fp32 tensors, head_dim 64 and any
// power-of-two block size; bf16 / head_dim 128 shapes normally take the MFMA kernel.
//
// Mapping: a token row of K or V is D*sizeof(T) bytes = LR lanes x 16 bytes, so one
// wavefront load covers TPL = 64/LR tokens, fully coalesced.  Each group of LR lanes
// keeps its own online-softmax state over the tokens it sees (no cross-lane traffic in
// the loop beyond the LR-lane dot-product reduction); the TPL groups, then the four
// wavefronts, are merged with the log-sum-exp rule at the end.  Scores and softmax are
// in natural-log units, accumulation in fp32.
//
// PREFILL variant (causal attention of several query positions per sequence, the recompute
// path of Section 2.5 / 3.5, for the shapes the MFMA prefill kernel does not take): a
// "sequence" of the grid is one query row; the row finds its sequence n by a search over
// q_start, attends to the first S_n - Qn + i + 1 tokens of n's block list in one partition and
// writes its normalised output directly.
#include <math.h>

#include "kvc_internal.h"

namespace kvc {

namespace {

template <typename T>
struct Elem;

template <>
struct Elem<float> {
    static constexpr int kPerLane = 4;  // elements in 16 bytes
    __device__ static void load16(const float *p, float (&x)[4]) {
        const float4 v = *reinterpret_cast<const float4 *>(p);
        x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
    }
    __device__ static float exp_(float x) { return expf(x); }
    __device__ static float to_out(float x) { return x; }
};

template <>
struct Elem<uint16_t> {  // bfloat16 bit patterns
    static constexpr int kPerLane = 8;
    __device__ static void load16(const uint16_t *p, float (&x)[8]) {
        const uint4 v = *reinterpret_cast<const uint4 *>(p);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = __uint_as_float(w[i] << 16);
            x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    __device__ static float exp_(float x) { return __expf(x); }
    __device__ static uint16_t to_out(float x) {  // round to nearest even
        uint32_t u = __float_as_uint(x);
        if ((u & 0x7fffffffu) > 0x7f800000u) return uint16_t((u >> 16) | 0x40u);
        u += 0x7fffu + ((u >> 16) & 1u);
        return uint16_t(u >> 16);
    }
};

constexpr int kUnroll = 4;  // tokens per lane group per loop trip (8 x 16-byte loads in flight)

template <typename T, int D, int GC, bool PREFILL>
__global__ __launch_bounds__(kThreads) void pa_partial_valu_kernel(
    const T *__restrict__ q, const T *__restrict__ k_cache, const T *__restrict__ v_cache,
    const int32_t *__restrict__ block_tables, const int32_t *__restrict__ context_lens,
    const int32_t *__restrict__ q_start, int num_tables, int max_query_len,
    T *__restrict__ out, Workspace ws, AttnParams p) {
    using E = Elem<T>;
    constexpr int EPL = E::kPerLane;
    constexpr int LR = D / EPL;    // lanes per token row
    constexpr int TPL = 64 / LR;   // tokens per wavefront load
    static_assert(LR >= 1 && LR <= 64 && (LR & (LR - 1)) == 0, "row must be 16..1024 bytes");

    // blockIdx.x = head_chunk + chunks * (seq + num_seqs * partition): the partition index
    // varies slowest, so the (always busy) first partitions are dispatched first.
    const int chunks = p.num_q_heads / GC;
    const int item = blockIdx.x;
    const int hc = item % chunks;
    const int seq = (item / chunks) % p.num_seqs;
    const int part = item / (chunks * p.num_seqs);
    const int head0 = hc * GC;
    const int kvh = head0 / p.group;
    const int tid = threadIdx.x;
    int ctx, tseq = seq;  // context length of this item, and the sequence whose table it walks
    if (PREFILL) {
        // seq is a row of q: largest n with q_start[n] <= row (sequences without rows are skipped)
        int lo = 0, hi = num_tables;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (q_start[mid] <= seq) lo = mid; else hi = mid;
        }
        tseq = lo;
        const int i = seq - q_start[lo], Qn = q_start[lo + 1] - q_start[lo], S = context_lens[lo];
        if (Qn > S || i >= max_query_len) return;
        ctx = S - Qn + i + 1;
    } else {
        ctx = min(context_lens[seq], p.max_context_len);
    }

    if (ctx <= 0) {  // empty context: a row of zeros, written by partition 0
        if (part == 0)
            for (int i = tid; i < GC * D; i += kThreads)
                out[(size_t(seq) * p.num_q_heads + head0) * D + i] = E::to_out(0.f);
        return;
    }
    const int tok0 = part * p.partition_tokens;
    if (tok0 >= ctx) return;
    const int tok1 = min(ctx, tok0 + p.partition_tokens);

    const int wave = tid >> 6, lane = tid & 63;
    const int tg = lane / LR, c = lane % LR;

    float qf[GC][EPL];
#pragma unroll
    for (int g = 0; g < GC; ++g)
        E::load16(q + (size_t(seq) * p.num_q_heads + head0 + g) * D + c * EPL, qf[g]);

    float m[GC], l[GC], acc[GC][EPL];
#pragma unroll
    for (int g = 0; g < GC; ++g) {
        m[g] = -INFINITY;
        l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
    }

    const int32_t *table = block_tables + size_t(tseq) * p.max_blocks_per_seq;
    const size_t head_stride = size_t(p.block_size) * D;               // elements per (block, kv head)
    const size_t block_stride = head_stride * p.num_kv_heads;
    constexpr int CH = TPL * kUnroll;                                   // tokens per wavefront per trip

    for (int base = tok0 + wave * CH; base < tok1; base += kWaves * CH) {
        float kf[kUnroll][EPL], vf[kUnroll][EPL];
        bool valid[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int t = base + u * TPL + tg;
            valid[u] = t < tok1;
            const int tc = valid[u] ? t : tok1 - 1;  // clamp: never touch a table entry or slot past the context
            const int blk = table[tc >> p.block_size_log2];
            const int slot = tc & (p.block_size - 1);
            const size_t off = size_t(blk) * block_stride + kvh * head_stride + size_t(slot) * D + c * EPL;
            E::load16(k_cache + off, kf[u]);
            E::load16(v_cache + off, vf[u]);
        }
#pragma unroll
        for (int g = 0; g < GC; ++g) {
            float s[kUnroll];
            float mx = -INFINITY;
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                float d = 0.f;
#pragma unroll
                for (int e = 0; e < EPL; ++e) d = fmaf(qf[g][e], kf[u][e], d);
#pragma unroll
                for (int off = 1; off < LR; off <<= 1) d += __shfl_xor(d, off);
                s[u] = valid[u] ? d * p.scale : -INFINITY;
                mx = fmaxf(mx, s[u]);
            }
            const float m_new = fmaxf(m[g], mx);
            const float m_ref = m_new == -INFINITY ? 0.f : m_new;  // group has seen no token yet
            const float alpha = E::exp_(m[g] - m_ref);
            float psum = 0.f, pv[EPL];
#pragma unroll
            for (int e = 0; e < EPL; ++e) pv[e] = 0.f;
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const float pu = E::exp_(s[u] - m_ref);
                psum += pu;
#pragma unroll
                for (int e = 0; e < EPL; ++e) pv[e] = fmaf(pu, vf[u][e], pv[e]);
            }
            l[g] = fmaf(l[g], alpha, psum);
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(acc[g][e], alpha, pv[e]);
            m[g] = m_new;
        }
    }

    // merge the TPL lane groups of this wavefront (log-sum-exp rule)
#pragma unroll
    for (int off = LR; off < 64; off <<= 1) {
#pragma unroll
        for (int g = 0; g < GC; ++g) {
            const float m_o = __shfl_xor(m[g], off);
            const float l_o = __shfl_xor(l[g], off);
            const float M = fmaxf(m[g], m_o);
            const float M_ref = M == -INFINITY ? 0.f : M;
            const float a = E::exp_(m[g] - M_ref), b = E::exp_(m_o - M_ref);
            l[g] = l[g] * a + l_o * b;
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                const float acc_o = __shfl_xor(acc[g][e], off);
                acc[g][e] = acc[g][e] * a + acc_o * b;
            }
            m[g] = M;
        }
    }

    // merge the four wavefronts through LDS
    __shared__ float sm_m[kWaves][GC], sm_l[kWaves][GC];
    __shared__ float sm_acc[kWaves][GC][D];
    if (tg == 0) {
#pragma unroll
        for (int g = 0; g < GC; ++g) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) sm_acc[wave][g][c * EPL + e] = acc[g][e];
        }
        if (c == 0) {
#pragma unroll
            for (int g = 0; g < GC; ++g) {
                sm_m[wave][g] = m[g];
                sm_l[wave][g] = l[g];
            }
        }
    }
    __syncthreads();

    const bool single = ctx <= p.partition_tokens;  // the whole context sat in this partition
    for (int i = tid; i < GC * D; i += kThreads) {
        const int g = i / D, d = i % D;
        float M = sm_m[0][g];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) M = fmaxf(M, sm_m[w][g]);
        float L = 0.f, A = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float wgt = E::exp_(sm_m[w][g] - M);  // M is finite: wavefront 0 always has a token
            L = fmaf(wgt, sm_l[w][g], L);
            A = fmaf(wgt, sm_acc[w][g][d], A);
        }
        const size_t row = size_t(seq) * p.num_q_heads + head0 + g;
        if (single) {
            out[row * D + d] = E::to_out(A / L);
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

template <typename T, int D, bool PREFILL>
hipError_t launch_for_chunk(int gc, const void *q, const void *k, const void *v, const int32_t *bt,
                            const int32_t *cl, const int32_t *qs, int num_tables, int max_query_len,
                            void *out, Workspace ws, const AttnParams &p, int grid, hipStream_t stream) {
#define KVC_LAUNCH_VALU(GC)                                                                       \
    pa_partial_valu_kernel<T, D, GC, PREFILL><<<dim3(grid), dim3(kThreads), 0, stream>>>(         \
        static_cast<const T *>(q), static_cast<const T *>(k), static_cast<const T *>(v), bt, cl, \
        qs, num_tables, max_query_len, static_cast<T *>(out), ws, p)
    switch (gc) {
        case 8: KVC_LAUNCH_VALU(8); break;
        case 4: KVC_LAUNCH_VALU(4); break;
        case 2: KVC_LAUNCH_VALU(2); break;
        default: KVC_LAUNCH_VALU(1); break;
    }
#undef KVC_LAUNCH_VALU
    return hipGetLastError();
}

template <bool PREFILL>
hipError_t launch_for_type(const void *q, const void *k_cache, const void *v_cache,
                           const int32_t *block_tables, const int32_t *context_lens,
                           const int32_t *q_start, int num_tables, int max_query_len, void *out,
                           Workspace ws, const AttnParams &p, int dtype, int head_dim, int grid,
                           hipStream_t stream) {
    const int gc = valu_head_chunk(p.group);
    if (dtype == KVC_F32) {
        if (head_dim == 64)
            return launch_for_chunk<float, 64, PREFILL>(gc, q, k_cache, v_cache, block_tables, context_lens, q_start,
                                                        num_tables, max_query_len, out, ws, p, grid, stream);
        return launch_for_chunk<float, 128, PREFILL>(gc, q, k_cache, v_cache, block_tables, context_lens, q_start,
                                                     num_tables, max_query_len, out, ws, p, grid, stream);
    }
    if (head_dim == 64)
        return launch_for_chunk<uint16_t, 64, PREFILL>(gc, q, k_cache, v_cache, block_tables, context_lens, q_start,
                                                       num_tables, max_query_len, out, ws, p, grid, stream);
    return launch_for_chunk<uint16_t, 128, PREFILL>(gc, q, k_cache, v_cache, block_tables, context_lens, q_start,
                                                    num_tables, max_query_len, out, ws, p, grid, stream);
}

}  // namespace

hipError_t launch_partial_valu(const void *q, const void *k_cache, const void *v_cache,
                               const int32_t *block_tables, const int32_t *context_lens, void *out,
                               Workspace ws, const AttnParams &p, int dtype, int head_dim,
                               int grid, hipStream_t stream) {
    return launch_for_type<false>(q, k_cache, v_cache, block_tables, context_lens, nullptr, 0, 0, out, ws, p,
                                  dtype, head_dim, grid, stream);
}

// p.num_seqs = rows of q, p.partition_tokens covers any context (one partition, no workspace).
hipError_t launch_prefill_valu(const void *q, const void *k_cache, const void *v_cache,
                               const int32_t *block_tables, const int32_t *context_lens,
                               const int32_t *q_start, int num_tables, int max_query_len, void *out,
                               const AttnParams &p, int dtype, int head_dim, int grid,
                               hipStream_t stream) {
    return launch_for_type<true>(q, k_cache, v_cache, block_tables, context_lens, q_start, num_tables,
                                 max_query_len, out, Workspace{nullptr, nullptr, nullptr}, p, dtype, head_dim,
                                 grid, stream);
}

}  // namespace kvc
