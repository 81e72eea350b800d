/*
 * kvc.h - C ABI of the paged-KV decode hot path for AMD MI355X (gfx950 / CDNA4).
 *
 * The paper's method (Sections 3.2-3.5) is host-side scheduling policy over a KV
 * cache that is handed out in fixed-size token blocks (Section 1; Section 3.3.1:
 * a request's blocks may sit anywhere in the pool, even inside another
 * request's allocation).  Every iteration that policy pays for is a batched
 * decode attention that reads each running request's whole KV through its
 * block list (Section 3.3.2: iteration time grows with the tokens in the
 * batch), and every preemption by swapping (Section 2.5, Section 3.5: cost
 * linear in sequence length) or KV reuse is a copy of KV blocks.  This library
 * is those two operations and nothing else.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE memory owned by the caller unless a comment
 *     says "host".  Descriptor structs are host memory, read during the call only.
 *   - The library allocates and frees nothing and never synchronises the stream;
 *     work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and the call returns at once.  The kvc_validate_* calls are
 *     the exception: they copy index arrays to the host and block.
 *   - Return value: KVC_OK (0) or a negative kvc_status.  Host-visible arguments
 *     are checked before anything is launched; on error nothing is written.
 *   - Contents of device index arrays (block ids, context lengths, mappings) are
 *     NOT checked on the fast path; out-of-range values there are undefined
 *     behaviour.  Use kvc_validate_* when in doubt.
 *
 * Tensor layouts (row-major, last index fastest; T = float or bfloat16):
 *   q, out        T [num_seqs][num_q_heads][head_dim]
 *   k_cache       T [num_pool_blocks][num_kv_heads][block_size][head_dim]
 *   v_cache       T [num_pool_blocks][num_kv_heads][block_size][head_dim]
 *   block_tables  int32 [num_seqs][max_blocks_per_seq]
 *   context_lens  int32 [num_seqs]
 * Query head h reads KV head h / (num_q_heads / num_kv_heads).
 */
#ifndef KVC_H
#define KVC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* exported from libkvc_hip.so (the library is built with hidden default visibility) */
#define KVC_API __attribute__((visibility("default")))

typedef enum {
    KVC_OK = 0,
    KVC_ERR_NULL = -1,        /* a required pointer is NULL */
    KVC_ERR_BAD_SHAPE = -2,   /* a size is non-positive or inconsistent */
    KVC_ERR_BAD_DTYPE = -3,
    KVC_ERR_UNSUPPORTED = -4, /* valid but not implemented (e.g. head_dim 96) */
    KVC_ERR_WORKSPACE = -5,   /* workspace NULL or too small */
    KVC_ERR_ALIGN = -6,       /* pointer / stride not 16-byte aligned */
    KVC_ERR_LAUNCH = -7,      /* HIP reported an error; see kvc_last_hip_error */
    KVC_ERR_BAD_INDEX = -8,   /* kvc_validate_*: an index is out of range */
    KVC_ERR_DUPLICATE = -9,   /* kvc_validate_*: a destination block appears twice */
    KVC_ERR_OVERLAP = -10     /* kvc_validate_*: same pool, source and destination sets meet */
} kvc_status;

typedef enum { KVC_F32 = 0, KVC_BF16 = 1 } kvc_dtype;

/* Which partial kernel computes the attention (KVC_KERNEL_AUTO picks). */
typedef enum {
    KVC_KERNEL_AUTO = 0,
    KVC_KERNEL_VALU = 1, /* vector-ALU dot products; any supported shape */
    KVC_KERNEL_MFMA = 2, /* matrix-core tiles; bf16, head_dim 128, block_size % 16 == 0, group <= 16;
                            K tiles go from HBM straight into the MFMA operand layout */
    KVC_KERNEL_MFMA_LDS = 3, /* same, K tiles loaded fully coalesced and re-laid-out through LDS */
    KVC_KERNEL_MFMA_BALANCED = 4 /* matrix-core tiles, persistent grid: the batch's (sequence, kv head,
                            16-token tile) work is flattened and cut into equal per-wavefront ranges;
                            bf16, head_dim 128, block_size >= 4, group <= 16, num_seqs <= 4096 */
} kvc_kernel;

typedef struct {
    int32_t num_seqs;           /* >= 0 (0 is a no-op) */
    int32_t num_q_heads;        /* multiple of num_kv_heads */
    int32_t num_kv_heads;
    int32_t head_dim;           /* 64 or 128 */
    int32_t block_size;         /* tokens per block: a power of two, 1..256 */
    int32_t max_blocks_per_seq; /* row length of block_tables */
    int32_t num_pool_blocks;    /* blocks in k_cache / v_cache (bounds for validation) */
    int32_t dtype;              /* kvc_dtype of q, k_cache, v_cache and out */
    int32_t max_context_len;    /* host-known upper bound on context_lens; 0 means
                                   max_blocks_per_seq * block_size.  A tight bound keeps
                                   the launch grid and the workspace small. */
    int32_t partition_tokens;   /* split-K partition length in tokens (multiple of 16, at most
                                   4096); 0 lets the library choose.  With kernel ==
                                   KVC_KERNEL_MFMA_BALANCED: the smallest range a wavefront takes
                                   (multiple of 16, at most 2^20). */
    int32_t kernel;             /* kvc_kernel */
    int32_t reserved;           /* must be 0 */
} kvc_attn_desc;

/* What the library will do for a descriptor (filled by kvc_attn_plan). */
typedef struct {
    int32_t kernel;            /* the kvc_kernel that will run (never AUTO) */
    int32_t partition_tokens;
    int32_t max_partitions;    /* partitions per sequence the grid provides for (balanced kernel:
                                  partial slots per wavefront) */
    int32_t partial_grid;      /* workgroups of the partial kernel */
    int32_t merge_grid;        /* workgroups of the merge kernel (0: not launched) */
    int32_t reserved;
    uint64_t workspace_bytes;
} kvc_attn_plan_info;

KVC_API int kvc_version(void);
KVC_API const char *kvc_status_string(int status);
/* hipError_t of the last failed HIP call made by this thread inside the library (0 if none). */
KVC_API int kvc_last_hip_error(void);

/* Checks `desc` (host) and reports kernel choice, grid and workspace.  No GPU needed. */
KVC_API int kvc_attn_plan(const kvc_attn_desc *desc, kvc_attn_plan_info *plan);

/* Bytes of device workspace kvc_paged_attention_decode needs for `desc`
 * (0 when no sequence can span more than one partition, or on a bad desc).  For the balanced
 * kernel it depends on the group size only, not on the batch or the context lengths. */
KVC_API size_t kvc_paged_attention_decode_workspace_bytes(const kvc_attn_desc *desc);

/*
 * Batched single-token attention over a block-allocated KV cache:
 *   out[n][h][:] = sum_t softmax_t( scale * q[n][h] . K[n,t] ) * V[n,t],  t < context_lens[n],
 * where token t of sequence n lives in block block_tables[n][t / block_size], slot
 * t % block_size, KV head h / group.  (Decode step of an iteration-level scheduler over
 * block-based KV allocation: Section 1, Section 3.1, Section 3.3.)
 *
 *   - Table entries at index >= ceil(context_len / block_size) are never dereferenced, and
 *     pool contents at slots >= context_len in the last block never reach `out` (NaN there
 *     is fine).  One block id may appear in many rows (shared prefix).
 *   - context_lens[n] == 0 writes a row of zeros.
 *   - Accumulation is fp32; bf16 output is rounded to nearest even.
 *   - Split-K: a long context is cut into pieces whose (max, sum, accumulator) partials go
 *     through the workspace.  The balanced kernel (KVC_KERNEL_MFMA_BALANCED, what AUTO picks for
 *     bf16 / head_dim 128) is ONE launch: the last wavefront to finish a piece of a cut context
 *     merges its partials and writes the row.  The other kernels are followed by a merge launch.
 *   - `workspace`: device memory, 256-byte aligned, at least
 *     kvc_paged_attention_decode_workspace_bytes(desc); may be NULL when that is 0.  Its first
 *     4096 bytes hold arrival counters that must be 0 when a call starts:
 *     kvc_paged_attention_decode_workspace_init sets them once after allocation, every call
 *     leaves them 0 again (whatever descriptor it ran with), and no call writes anything else
 *     there.  The rest is scratch: contents before and after a call are meaningless.  Calls that
 *     share a workspace must not overlap in time (one stream, or ordered by events).
 *   - q, k_cache, v_cache, out must be 16-byte aligned.
 */
KVC_API int kvc_paged_attention_decode(const void *q, const void *k_cache, const void *v_cache,
                               const int32_t *block_tables, const int32_t *context_lens,
                               float scale, void *out, const kvc_attn_desc *desc,
                               void *workspace, size_t workspace_bytes, void *hip_stream);

/* Prepares a freshly allocated (or overwritten) workspace: sets its 4096-byte counter header
 * to 0 with a small kernel on `hip_stream` (no memset node, safe under graph capture).
 * workspace_bytes == 0 is a no-op. */
KVC_API int kvc_paged_attention_decode_workspace_init(void *workspace, size_t workspace_bytes,
                                                      void *hip_stream);

/* The launches of kvc_paged_attention_decode on their own (same arguments, same checks), for
 * callers that time or schedule them separately.  Running partial then merge on one stream
 * equals kvc_paged_attention_decode; with the balanced kernel partial is the whole call and
 * merge launches nothing. */
KVC_API int kvc_paged_attention_decode_partial(const void *q, const void *k_cache, const void *v_cache,
                                       const int32_t *block_tables, const int32_t *context_lens,
                                       float scale, void *out, const kvc_attn_desc *desc,
                                       void *workspace, size_t workspace_bytes, void *hip_stream);
KVC_API int kvc_paged_attention_decode_merge(const int32_t *context_lens, void *out,
                                     const kvc_attn_desc *desc, void *workspace,
                                     size_t workspace_bytes, void *hip_stream);

/*
 * The same attention with the placement work taken out of the call.  Within one iteration of an
 * iteration-level scheduler (Section 3.1) every layer of the model attends over the same
 * block_tables and context_lens; what the balanced kernel derives from them at the start of every
 * launch (prefix table of the batch, which tiles each wavefront takes, their pool addresses, which
 * contexts are cut where) can therefore be computed once per iteration and reused by all layers.
 *   kvc_attn_schedule_bytes   bytes of device memory a schedule for `desc` needs (0 when the
 *                             descriptor is not served by the balanced kernel, or is invalid);
 *                             a host-side bound that depends on num_seqs and max_context_len.
 *   kvc_attn_schedule_build   one short launch that fills `schedule` (256-byte aligned device
 *                             memory) from block_tables and context_lens.  The schedule stays valid
 *                             until either array changes; it may be rebuilt in place.
 *   kvc_paged_attention_decode_scheduled
 *                             kvc_paged_attention_decode with block_tables / context_lens replaced
 *                             by the schedule built from them (same desc): same kernel, same
 *                             split, bit-identical output; the first KV bytes are requested after
 *                             one memory round trip instead of three.  Workspace rules as above.
 * Errors: KVC_ERR_UNSUPPORTED when the descriptor does not use the balanced kernel,
 * KVC_ERR_WORKSPACE when `schedule` is NULL or smaller than kvc_attn_schedule_bytes.  A schedule
 * built for other arrays or another descriptor is not detected: undefined behaviour.
 */
KVC_API size_t kvc_attn_schedule_bytes(const kvc_attn_desc *desc);
KVC_API int kvc_attn_schedule_build(const int32_t *block_tables, const int32_t *context_lens,
                                    const kvc_attn_desc *desc, void *schedule, size_t schedule_bytes,
                                    void *hip_stream);
KVC_API int kvc_paged_attention_decode_scheduled(const void *q, const void *k_cache, const void *v_cache,
                                                 const void *schedule, size_t schedule_bytes, float scale,
                                                 void *out, const kvc_attn_desc *desc, void *workspace,
                                                 size_t workspace_bytes, void *hip_stream);

/*
 * kvc_paged_attention_decode for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, checks, kernels and results as kvc_paged_attention_decode, but
 * the split-K workspace is a fixed region of KVC_NOALLOC_WORKSPACE_BYTES that the library
 * holds on every GPU it is loaded on (placed with the code object, kept until the process
 * ends).  The call allocates and frees nothing.
 *   - A descriptor whose kvc_paged_attention_decode_workspace_bytes exceeds
 *     KVC_NOALLOC_WORKSPACE_BYTES is refused with KVC_ERR_WORKSPACE (nothing is launched);
 *     every descriptor the balanced kernel serves fits.
 *   - The device that owns `hip_stream` must be the current device.  The first call on a
 *     device looks up the region's address (a HIP symbol query); make that call outside a
 *     graph capture.
 *   - All calls on one GPU share the region: calls whose kernels can overlap in time (different
 *     streams, or graphs replayed concurrently) race and give undefined results.  Calls on one
 *     stream are ordered and safe.  The region starts zeroed and every call leaves its counter
 *     header zeroed, so no initialisation call is needed.
 */
#define KVC_NOALLOC_WORKSPACE_BYTES (32u << 20)
KVC_API int kvc_paged_attention_decode_noalloc(const void *q, const void *k_cache, const void *v_cache,
                                               const int32_t *block_tables, const int32_t *context_lens,
                                               float scale, void *out, const kvc_attn_desc *desc,
                                               void *hip_stream);

/* Blocking check of the device index arrays against `desc`: 0 <= context_lens[n] <=
 * min(max_context_len, max_blocks_per_seq * block_size) and every dereferenced table entry in
 * [0, num_pool_blocks).  Returns KVC_ERR_BAD_INDEX on the first violation. */
KVC_API int kvc_validate_attention_inputs(const int32_t *block_tables, const int32_t *context_lens,
                                  const kvc_attn_desc *desc, void *hip_stream);

/*
 * Causal attention of several query positions per sequence over the block-allocated cache: the
 * recomputation path of a preempted request (prefill re-run over its prompt and generated tokens;
 * Section 2.5 and 3.5: cost quadratic in the sequence length) and chunked prefill.
 *   q, out        T [total_q][num_q_heads][head_dim], the query rows of all sequences back to back
 *   q_start       int32 [num_seqs + 1] (device): sequence n owns rows q_start[n] .. q_start[n+1]-1
 *   context_lens  int32 [num_seqs] (device): tokens of sequence n present in the cache (S_n);
 *                 its Qn query rows sit at positions S_n - Qn .. S_n - 1 and row i attends to
 *                 tokens 0 .. (S_n - Qn + i).  Qn <= S_n; a sequence with Qn == 0 is skipped.
 *   total_q, max_query_len   host-known: number of rows of q, and an upper bound on Qn (sizes
 *                 the launch grid; rows of sequences with Qn > max_query_len beyond it are not
 *                 computed).
 * Every shape the descriptor allows is served: bf16 with head_dim 128 and group <= 16 runs on
 * the matrix cores (any block size): on 32x32 tiles when the scale is positive (two heads of a KV
 * head per wavefront for even group sizes, one head otherwise), on 16x16 tiles for other scales or
 * when desc->kernel is KVC_KERNEL_MFMA; everything else
 * (fp32, head_dim 64, larger groups) on the vector ALUs, one workgroup per query row and head
 * chunk.  No workspace.  desc->max_context_len and partition_tokens are ignored; desc->kernel must
 * be valid for the shape and is otherwise ignored.
 */
KVC_API int kvc_paged_attention_prefill(const void *q, const void *k_cache, const void *v_cache,
                                        const int32_t *block_tables, const int32_t *context_lens,
                                        const int32_t *q_start, float scale, void *out,
                                        const kvc_attn_desc *desc, int32_t total_q,
                                        int32_t max_query_len, void *hip_stream);

/*
 * Write one new token per sequence into the block-allocated cache (the step that precedes
 * the decode attention of an iteration: every running request produces one token whose K and V
 * land in the next free slot of its last block; Section 1, Section 3.3).
 *   k_new, v_new   T [num_seqs][num_kv_heads][head_dim]   (device, 16-byte aligned)
 *   positions      int32 [num_seqs] (device): token index to write for each sequence; the
 *                  token goes to block block_tables[n][pos / block_size], slot pos % block_size.
 *                  A negative position skips the sequence, and so does one at or past
 *                  max_blocks_per_seq * block_size (the table has no entry for it).
 * Every other byte of the caches is left untouched.  Uses desc->num_seqs, num_kv_heads,
 * head_dim, block_size, max_blocks_per_seq and dtype (the attention-only fields are ignored
 * but must be valid).  Block ids are not range-checked.
 */
KVC_API int kvc_kv_cache_append(const void *k_new, const void *v_new, void *k_cache, void *v_cache,
                                const int32_t *block_tables, const int32_t *positions,
                                const kvc_attn_desc *desc, void *hip_stream);

/*
 * A KV pool as the copy sees it: num_planes planes (K or V of one layer each) of num_blocks
 * blocks of block_bytes bytes; plane p starts at base + p * plane_stride_bytes.
 */
typedef struct {
    void *base;                 /* 16-byte aligned; device memory, or pinned host memory mapped into the
                                   device address space (hipHostMalloc): swap to / from CPU memory */
    int64_t num_blocks;
    int64_t block_bytes;        /* multiple of 16 */
    int64_t plane_stride_bytes; /* multiple of 16, >= num_blocks * block_bytes (ignored if num_planes == 1) */
    int32_t num_planes;         /* >= 1 */
    int32_t reserved;           /* must be 0 */
} kvc_pool;

/*
 * Block gather/scatter between KV pools, bit-exact: for every pair (s, d) of
 * block_mapping and every plane p, dst[p][d][:] = src[p][s][:].  This is the data
 * movement behind swapping a preempted request's KV out and back in (Section 2.5,
 * Section 3.5) and behind relocating blocks for KV reuse (Section 3.3.1).
 *
 *   - block_mapping: device int64 [num_pairs][2] = (src_block, dst_block); num_pairs may be 0.
 *   - src and dst must agree in block_bytes and num_planes; num_blocks may differ.
 *   - A source block may appear several times (fan-out).  A destination block must appear at
 *     most once, and when src and dst are the same memory the source and destination block
 *     sets must be disjoint; neither is checked here (see kvc_validate_block_mapping).
 *   - Blocks of dst that are not a destination are left untouched.
 *   - Either pool may be pinned host memory; the kernel then moves the blocks over PCIe
 *     itself (no staging copy, one launch for any number of blocks).
 */
KVC_API int kvc_kv_block_copy(const kvc_pool *src, const kvc_pool *dst, const int64_t *block_mapping,
                      int64_t num_pairs, void *hip_stream);

/* Blocking check of a device block_mapping: ids in range (KVC_ERR_BAD_INDEX), no duplicate
 * destination (KVC_ERR_DUPLICATE), and no source/destination overlap when the pools share
 * memory (KVC_ERR_OVERLAP). */
KVC_API int kvc_validate_block_mapping(const kvc_pool *src, const kvc_pool *dst,
                               const int64_t *block_mapping, int64_t num_pairs, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* KVC_H */
