// Internal declarations shared by the HIP translation units of libkvc_hip.so.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvc.h"

namespace kvc {

// Everything the attention kernels need besides the tensor pointers.
struct AttnParams {
    int num_seqs;
    int num_q_heads;
    int num_kv_heads;
    int group;              // num_q_heads / num_kv_heads
    int block_size;
    int block_size_log2;
    int max_blocks_per_seq;
    int partition_tokens;   // split-K partition length, multiple of 16
    int max_partitions;     // partitions per sequence the grid and workspace provide for
    int k_via_lds;          // MFMA kernel: stage K tiles through LDS (1) or load them in operand layout (0)
    int min_chunk_tiles;    // balanced kernel: smallest number of 16-token tiles a worker takes
    int max_context_len;    // context lengths are clamped to this (the bound every size is derived from)
    float scale;            // as given by the caller
    float scale_log2e;      // scale * log2(e), for the base-2 softmax of the MFMA kernel
};

// Causal multi-query (prefill / recompute) attention.
struct PrefillParams {
    int num_seqs;
    int num_q_heads;
    int num_kv_heads;
    int group;                 // num_q_heads / num_kv_heads
    int heads_per_chunk;       // query heads one wavefront carries (1 or 2; divides group)
    int block_size;
    int block_size_log2;
    int tiles_per_block_log2;  // log2(block_size / 16); 0 for block sizes below 16
    int max_blocks_per_seq;
    int max_query_tiles;       // ceil(max_query_len / 64)
    float scale_log2e;
};

// Workspace layout.  The first kWorkspaceHeaderBytes hold the arrival counters of the
// balanced kernel (int32 [workers], 0 between calls); no kernel writes anything else there.
// Fixed-partition kernels: acc [num_seqs][num_q_heads][max_partitions][head_dim] fp32, then
// ml [num_seqs][num_q_heads][max_partitions][2] fp32 (running max, running sum).
// Balanced kernel: acc [workers][2][group][head_dim] fp32, ml [workers][2][group][2] fp32
// (two partial slots per worker).  Each array starts at a 256-byte aligned offset.
struct Workspace {
    float *acc;
    float *ml;
    int32_t *cnt;
};
constexpr size_t kWorkspaceHeaderBytes = 4096;

// Placement of the balanced kernel's workers for one (block_tables, context_lens), kept in device
// memory between a build launch and the attention launches of the layers that share it:
// pref [num_seqs + 2], ctx [num_seqs], plans [workers][16], tiles [workers][stride] (all int32).
struct Schedule {
    int *pref;
    int *ctx;
    int *plans;
    int *tiles;
    int stride;  // tile-address entries a worker's share of `tiles` holds
};

constexpr int kThreads = 256;       // 4 wavefronts per workgroup, every attention kernel
constexpr int kWaves = kThreads / 64;
constexpr int kNumCUs = 256;        // MI355X
constexpr int kMaxStreamSeqs = 4096;  // batch limit of the balanced kernel (prefix sum lives in LDS)

// Launchers (defined next to their kernels).  All enqueue on `stream` and return the
// hipError_t of the launch.
hipError_t launch_partial_valu(const void *q, const void *k_cache, const void *v_cache,
                               const int32_t *block_tables, const int32_t *context_lens, void *out,
                               Workspace ws, const AttnParams &p, int dtype, int head_dim,
                               int grid, hipStream_t stream);
hipError_t launch_partial_mfma(const void *q, const void *k_cache, const void *v_cache,
                               const int32_t *block_tables, const int32_t *context_lens, void *out,
                               Workspace ws, const AttnParams &p, int grid, hipStream_t stream);
// mode 0: stateless call; 1: only build `sched` from block_tables / context_lens; 2: run from `sched`
// (block_tables / context_lens unused).
hipError_t launch_partial_mfma_stream(const void *q, const void *k_cache, const void *v_cache,
                                      const int32_t *block_tables, const int32_t *context_lens,
                                      void *out, Workspace ws, const AttnParams &p, int grid,
                                      int mode, Schedule sched, hipStream_t stream);
// base2: partials are in base-2 units.
hipError_t launch_merge(const int32_t *context_lens, void *out, Workspace ws, const AttnParams &p,
                        int dtype, int head_dim, bool base2, int grid, hipStream_t stream);
// Sets the counter header of a workspace to 0 (a fill kernel, safe under graph capture).
hipError_t launch_workspace_init(void *workspace, hipStream_t stream);
hipError_t launch_prefill_mfma(const void *q, const void *k_cache, const void *v_cache,
                               const int32_t *block_tables, const int32_t *context_lens,
                               const int32_t *q_start, void *out, const PrefillParams &p,
                               hipStream_t stream);
hipError_t launch_prefill_mfma32(const void *q, const void *k_cache, const void *v_cache,
                                 const int32_t *block_tables, const int32_t *context_lens,
                                 const int32_t *q_start, void *out, const PrefillParams &p,
                                 hipStream_t stream);
hipError_t launch_prefill_valu(const void *q, const void *k_cache, const void *v_cache,
                               const int32_t *block_tables, const int32_t *context_lens,
                               const int32_t *q_start, int num_tables, int max_query_len, void *out,
                               const AttnParams &p, int dtype, int head_dim, int grid,
                               hipStream_t stream);
hipError_t launch_cache_append(const void *k_new, const void *v_new, void *k_cache, void *v_cache,
                               const int32_t *block_tables, const int32_t *positions, int num_seqs,
                               int num_kv_heads, int row_bytes, int block_size_log2,
                               int max_blocks_per_seq, hipStream_t stream);
constexpr int64_t kCopySlabBytes = 1024;  // bytes one workgroup of the block-copy kernel moves (grid.x = pairs * slabs per block)
hipError_t launch_block_copy(const kvc_pool &src, const kvc_pool &dst, const int64_t *mapping,
                             int64_t num_pairs, hipStream_t stream);

// Largest head chunk (8, 4, 2 or 1) the VALU kernel processes per workgroup for a group size.
inline int valu_head_chunk(int group) {
    return group % 8 == 0 ? 8 : group % 4 == 0 ? 4 : group % 2 == 0 ? 2 : 1;
}

}  // namespace kvc
