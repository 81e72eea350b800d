// Second pass of split-K paged decode attention (gfx950): combine the per-partition
// (max, sum, un-normalised accumulator) triples of every (sequence, query head) whose
// context was split, normalise and cast.
//
//   M = max_p m_p;  out = sum_p w_p acc_p / sum_p w_p l_p,  w_p = exp(m_p - M)
//
// (exp is base 2 when the partial kernel worked in base-2 units.)  One wavefront per
// (sequence, head).  Lane i first fetches (m, l) of partial i, so all weights of up to 64
// partials come from one load and one wavefront max/sum; that load is issued speculatively
// together with the loads of the context length and the partial count, so the kernel is two
// memory round trips deep.  The accumulator rows are then streamed with the weight broadcast
// from its lane, lanes striding over head_dim (coalesced 256/512-byte reads, 8 rows in flight).
//
// The number of partials of a row is ceil(context_len / partition_tokens); rows finished by
// the partial kernel (one partial, or an empty context) are skipped.  The balanced kernel
// merges inside its own launch and does not use this one.
#include <math.h>

#include "kvc_internal.h"

namespace kvc {

namespace {

__device__ inline uint16_t f32_to_bf16_rne(float x) {
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return uint16_t((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return uint16_t(u >> 16);
}
__device__ inline void store_out(float *o, float x) { *o = x; }
__device__ inline void store_out(uint16_t *o, float x) { *o = f32_to_bf16_rne(x); }

template <typename T, int D, bool BASE2>
__global__ __launch_bounds__(kThreads) void pa_merge_kernel(const int32_t *__restrict__ context_lens,
                                                            T *__restrict__ out, Workspace ws,
                                                            AttnParams p) {
    constexpr int DPL = D / 64;  // dims per lane
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row = blockIdx.x * kWaves + wave;  // seq * num_q_heads + head
    if (row >= p.num_seqs * p.num_q_heads) return;
    const int seq = row / p.num_q_heads;
    const int head = row - seq * p.num_q_heads;
    const float *ml = ws.ml + size_t(row) * p.max_partitions * 2;
    const float *acc = ws.acc + size_t(row) * p.max_partitions * D + lane * DPL;

    // Two independent loads go out together: the context length and (speculatively, whatever
    // the slots hold) the (max, sum) pairs of the first 64 slots.
    const int ctx = min(context_lens[seq], p.max_context_len);
    float2 ml0 = float2{-INFINITY, 0.f};
    if (lane < p.max_partitions) ml0 = *reinterpret_cast<const float2 *>(ml + 2 * lane);
    int nparts = (ctx + p.partition_tokens - 1) / p.partition_tokens;  // <= 1: finished already, or empty
    if (nparts <= 1) return;
    nparts = min(nparts, p.max_partitions);

    float M = lane < nparts ? ml0.x : -INFINITY;
    for (int i = lane + 64; i < nparts; i += 64) M = fmaxf(M, ml[2 * i]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));

    float L = 0.f, a[DPL];
#pragma unroll
    for (int j = 0; j < DPL; ++j) a[j] = 0.f;
    for (int c0 = 0; c0 < nparts; c0 += 64) {
        const int i = c0 + lane;
        float w = 0.f;
        if (i < nparts) {
            const float2 v = c0 == 0 ? ml0 : *reinterpret_cast<const float2 *>(ml + 2 * i);
            const float x = v.x - M;
            w = BASE2 ? __builtin_amdgcn_exp2f(x) : expf(x);
            L = fmaf(w, v.y, L);
        }
        const int nt = min(64, nparts - c0);
        int t = 0;
        for (; t + 8 <= nt; t += 8) {  // 8 accumulator rows in flight
            float x[8][DPL];
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int j = 0; j < DPL; ++j) x[u][j] = acc[size_t(c0 + t + u) * D + j];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float wt = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w), t + u));
#pragma unroll
                for (int j = 0; j < DPL; ++j) a[j] = fmaf(wt, x[u][j], a[j]);
            }
        }
        for (; t < nt; ++t) {
            const float wt = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w), t));
#pragma unroll
            for (int j = 0; j < DPL; ++j) a[j] = fmaf(wt, acc[size_t(c0 + t) * D + j], a[j]);
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) L += __shfl_xor(L, off);
#pragma unroll
    for (int j = 0; j < DPL; ++j) store_out(out + size_t(row) * D + lane * DPL + j, a[j] / L);
}

template <typename T, int D>
void launch(bool base2, const int32_t *cl, void *out, Workspace ws, const AttnParams &p, int grid,
            hipStream_t stream) {
    T *o = static_cast<T *>(out);
    const dim3 g(grid), b(kThreads);
    if (base2)
        pa_merge_kernel<T, D, true><<<g, b, 0, stream>>>(cl, o, ws, p);
    else
        pa_merge_kernel<T, D, false><<<g, b, 0, stream>>>(cl, o, ws, p);
}

__global__ void workspace_init_kernel(int32_t *header) {
    header[blockIdx.x * blockDim.x + threadIdx.x] = 0;
}

}  // namespace

hipError_t launch_merge(const int32_t *context_lens, void *out, Workspace ws, const AttnParams &p,
                        int dtype, int head_dim, bool base2, int grid, hipStream_t stream) {
    if (dtype == KVC_F32) {
        if (head_dim == 64) launch<float, 64>(base2, context_lens, out, ws, p, grid, stream);
        else launch<float, 128>(base2, context_lens, out, ws, p, grid, stream);
    } else {
        if (head_dim == 64) launch<uint16_t, 64>(base2, context_lens, out, ws, p, grid, stream);
        else launch<uint16_t, 128>(base2, context_lens, out, ws, p, grid, stream);
    }
    return hipGetLastError();
}

hipError_t launch_workspace_init(void *workspace, hipStream_t stream) {
    constexpr int kWords = int(kWorkspaceHeaderBytes / sizeof(int32_t));
    workspace_init_kernel<<<dim3(kWords / kThreads), dim3(kThreads), 0, stream>>>(static_cast<int32_t *>(workspace));
    return hipGetLastError();
}

}  // namespace kvc
