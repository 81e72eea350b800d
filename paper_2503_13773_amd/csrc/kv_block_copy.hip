// kv_block_copy: bit-exact block gather/scatter between KV pools (gfx950).
//
// The data movement behind swapping a preempted request's KV out and back in
// (paper Section 2.5 and 3.5: cost linear in the sequence length) and behind
// relocating blocks when allocated-but-unused KV cache is reused (Section 3.3.1).
//
// Pure HBM streaming: a workgroup is one wavefront that moves one contiguous 1 KiB
// slab of one (pair, plane) block, a 16-byte non-temporal load and store per lane.
// Many small workgroups beat fewer, larger ones here (measured on the cfg3b swap-out,
// 51 MB each way: 18.5 us against 19.0 us with 256 lanes x 16 bytes, 19.7 us with 256
// lanes x 64 bytes, 31.5 us with one workgroup per 32 KiB block, 20.5 us and more for
// grid-stride loops with the next load in flight): the device keeps more independent
// wavefronts in flight and the tail of the grid is finer.  The (src, dst) pair is read
// once per workgroup through the scalar path (its index is workgroup-uniform).
#include "kvc_internal.h"

namespace kvc {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));  // one 16-byte word

constexpr int kCopyThreads = 64;                      // one wavefront per workgroup
constexpr int kRounds = 1;                            // 16-byte words per lane
constexpr int64_t kSlabBytes = kCopySlabBytes;          // 1 KiB per workgroup
static_assert(kSlabBytes == int64_t(kCopyThreads) * 16 * kRounds, "slab = lanes x 16 bytes x rounds");

struct CopyParams {
    const uint8_t *src;
    uint8_t *dst;
    int64_t block_bytes;
    int64_t src_plane_stride;
    int64_t dst_plane_stride;
    int64_t num_pairs;
    int32_t slabs_per_block;
};

__global__ __launch_bounds__(kCopyThreads) void kv_block_copy_kernel(CopyParams p,
                                                                 const int64_t *__restrict__ mapping) {
    // grid.x = slab + slabs_per_block * pair, grid.y = plane
    const int64_t wg = blockIdx.x;
    const int slab = int(wg % p.slabs_per_block);
    const int64_t pair = wg / p.slabs_per_block;
    if (pair >= p.num_pairs) return;
    const int64_t sblk = mapping[2 * pair];
    const int64_t dblk = mapping[2 * pair + 1];
    const uint8_t *s = p.src + blockIdx.y * p.src_plane_stride + sblk * p.block_bytes;
    uint8_t *d = p.dst + blockIdx.y * p.dst_plane_stride + dblk * p.block_bytes;

    const int64_t off0 = slab * kSlabBytes + int64_t(threadIdx.x) * 16;
    u32x4 w[kRounds];
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int64_t off = off0 + int64_t(r) * kCopyThreads * 16;
        if (off < p.block_bytes) w[r] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(s + off));
    }
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int64_t off = off0 + int64_t(r) * kCopyThreads * 16;
        if (off < p.block_bytes) __builtin_nontemporal_store(w[r], reinterpret_cast<u32x4 *>(d + off));
    }
}

}  // namespace

hipError_t launch_block_copy(const kvc_pool &src, const kvc_pool &dst, const int64_t *mapping,
                             int64_t num_pairs, hipStream_t stream) {
    CopyParams p;
    p.src = static_cast<const uint8_t *>(src.base);
    p.dst = static_cast<uint8_t *>(dst.base);
    p.block_bytes = src.block_bytes;
    p.src_plane_stride = src.num_planes > 1 ? src.plane_stride_bytes : 0;
    p.dst_plane_stride = dst.num_planes > 1 ? dst.plane_stride_bytes : 0;
    p.num_pairs = num_pairs;
    p.slabs_per_block = int32_t((src.block_bytes + kSlabBytes - 1) / kSlabBytes);
    const dim3 grid(unsigned(num_pairs * p.slabs_per_block), unsigned(src.num_planes), 1);
    kv_block_copy_kernel<<<grid, dim3(kCopyThreads), 0, stream>>>(p, mapping);
    return hipGetLastError();
}

}  // namespace kvc
