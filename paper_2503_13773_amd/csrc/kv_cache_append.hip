// kv_cache_append: scatter one new token's K and V per sequence into the block-allocated
// cache (gfx950).  The write that precedes the decode attention of every iteration: each
// running request appends one token to the next free slot of its last block (block-based
// allocation: paper Section 1; iteration structure: Section 3.1).
//
// One 16-byte word per lane for K and one for V; a (sequence, kv head) row is row_bytes / 16
// consecutive lanes, so both the reads of k_new / v_new and the writes into the cache rows
// are coalesced.  Bytes moved are tiny (num_seqs * Hkv * D * e * 2): the kernel is
// launch-latency bound.
#include "kvc_internal.h"

namespace kvc {

namespace {

__global__ __launch_bounds__(kThreads) void kv_cache_append_kernel(
    const uint4 *__restrict__ k_new, const uint4 *__restrict__ v_new, uint4 *__restrict__ k_cache,
    uint4 *__restrict__ v_cache, const int32_t *__restrict__ block_tables,
    const int32_t *__restrict__ positions, int num_seqs, int num_kv_heads, int words_per_row,
    int block_size_log2, int max_blocks_per_seq) {
    const int64_t gid = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    const int64_t total = int64_t(num_seqs) * num_kv_heads * words_per_row;
    if (gid >= total) return;
    const int w = int(gid % words_per_row);
    const int h = int((gid / words_per_row) % num_kv_heads);
    const int n = int(gid / (int64_t(words_per_row) * num_kv_heads));
    const int pos = positions[n];
    // negative: skip the sequence; past the block table's reach: nothing to write to (not an error
    // this launch can report, but never an out-of-range table read)
    if (pos < 0 || (pos >> block_size_log2) >= max_blocks_per_seq) return;
    const int blk = block_tables[int64_t(n) * max_blocks_per_seq + (pos >> block_size_log2)];
    const int slot = pos & ((1 << block_size_log2) - 1);
    // cache row index: ((blk * Hkv + h) * Bs + slot), in units of words_per_row
    const int64_t row = ((int64_t(blk) * num_kv_heads + h) << block_size_log2) + slot;
    k_cache[row * words_per_row + w] = k_new[gid];
    v_cache[row * words_per_row + w] = v_new[gid];
}

}  // namespace

hipError_t launch_cache_append(const void *k_new, const void *v_new, void *k_cache, void *v_cache,
                               const int32_t *block_tables, const int32_t *positions, int num_seqs,
                               int num_kv_heads, int row_bytes, int block_size_log2,
                               int max_blocks_per_seq, hipStream_t stream) {
    const int words = row_bytes / 16;
    const int64_t total = int64_t(num_seqs) * num_kv_heads * words;
    const unsigned grid = unsigned((total + kThreads - 1) / kThreads);
    kv_cache_append_kernel<<<dim3(grid), dim3(kThreads), 0, stream>>>(
        static_cast<const uint4 *>(k_new), static_cast<const uint4 *>(v_new),
        static_cast<uint4 *>(k_cache), static_cast<uint4 *>(v_cache), block_tables, positions,
        num_seqs, num_kv_heads, words, block_size_log2, max_blocks_per_seq);
    return hipGetLastError();
}

}  // namespace kvc
