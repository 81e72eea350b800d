// Second pass of split-K paged decode attention (gfx950): combine the per-partition
// (max, sum, un-normalised accumulator) triples of every (sequence, query head) whose
// context spans more than one partition, normalise and cast.
//
//   M = max_p m_p;  out = sum_p w_p acc_p / sum_p w_p l_p,  w_p = exp(m_p - M)
//
// (exp is base 2 when the partial kernel worked in base-2 units.)  One wavefront per
// (sequence, head); lanes stride over head_dim, so every workspace row is read with
// coalesced 256/512-byte accesses.  Rows finished by the partial kernel (one partition)
// and empty contexts are skipped.
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
    const int ctx = context_lens[seq];
    if (ctx <= p.partition_tokens) return;  // finished by the partial kernel (or empty)
    const int nparts = min((ctx + p.partition_tokens - 1) / p.partition_tokens, p.max_partitions);

    const float *ml = ws.ml + size_t(row) * p.max_partitions * 2;
    const float *acc = ws.acc + size_t(row) * p.max_partitions * D;

    float M = -INFINITY;
    for (int i = lane; i < nparts; i += 64) M = fmaxf(M, ml[2 * i]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));

    float L = 0.f, a[DPL];
#pragma unroll
    for (int j = 0; j < DPL; ++j) a[j] = 0.f;
    for (int i = 0; i < nparts; ++i) {
        const float x = ml[2 * i] - M;
        const float w = BASE2 ? __builtin_amdgcn_exp2f(x) : expf(x);
        L = fmaf(w, ml[2 * i + 1], L);
#pragma unroll
        for (int j = 0; j < DPL; ++j) a[j] = fmaf(w, acc[size_t(i) * D + lane * DPL + j], a[j]);
    }
#pragma unroll
    for (int j = 0; j < DPL; ++j) store_out(out + size_t(row) * D + lane * DPL + j, a[j] / L);
}

template <typename T, int D>
void launch(bool base2, const int32_t *cl, void *out, Workspace ws, const AttnParams &p, int grid,
            hipStream_t stream) {
    if (base2)
        pa_merge_kernel<T, D, true><<<dim3(grid), dim3(kThreads), 0, stream>>>(cl, static_cast<T *>(out), ws, p);
    else
        pa_merge_kernel<T, D, false><<<dim3(grid), dim3(kThreads), 0, stream>>>(cl, static_cast<T *>(out), ws, p);
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

}  // namespace kvc
