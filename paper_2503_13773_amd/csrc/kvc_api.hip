// C ABI of libkvc_hip.so: argument checks, launch planning, kernel launches.
// The contract of every entry point is stated in include/kvc.h.
#include <math.h>

#include <algorithm>
#include <mutex>
#include <vector>

#include "kvc_internal.h"

// Workspace of kvc_paged_attention_decode_noalloc: one copy per GPU, placed by the loader with the
// code object and held until the process ends.  In host code the name below is only a handle
// for hipGetSymbolAddress; the address kernels can use is looked up once per device.
constexpr size_t kScratchBytes = size_t(KVC_NOALLOC_WORKSPACE_BYTES);
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

thread_local int g_last_hip_error = 0;

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up on the first call per device).
hipError_t scratch_of_current_device(void **ptr) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}

int hip_failed(hipError_t e) {
    g_last_hip_error = int(e);
    return KVC_ERR_LAUNCH;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool is_pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }
int ilog2(int x) { int l = 0; while ((1 << l) < x) ++l; return l; }
int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

constexpr int kMaxPartitionTokens = 4096;  // 4 wavefronts x 64 table entries x 16 tokens
constexpr int kMaxBalancedChunkTokens = 1 << 20;  // explicit minimum range of the balanced kernel
constexpr int64_t kMaxGrid = 0x7fffffff;

struct Plan {
    int kernel;
    int partition_tokens;
    int max_partitions;
    int64_t partial_grid;
    int64_t merge_grid;
    uint64_t acc_offset;  // offset of the accumulator array inside the workspace (after the counter header)
    uint64_t ml_offset;   // offset of the (max, sum) array
    uint64_t workspace_bytes;
    int min_chunk_tiles;
    int max_context_len;
};

bool mfma_ok(const kvc_attn_desc &d) {
    return d.dtype == KVC_BF16 && d.head_dim == 128 && d.block_size >= 16 &&
           d.num_q_heads / d.num_kv_heads <= 16;
}

// The balanced kernel keeps a prefix sum over the batch in LDS and indexes flat tiles in int32.
bool balanced_ok(const kvc_attn_desc &d, int max_ctx) {
    return d.dtype == KVC_BF16 && d.head_dim == 128 && d.block_size >= 4 &&
           d.num_q_heads / d.num_kv_heads <= 16 && d.num_seqs <= kvc::kMaxStreamSeqs &&
           int64_t(d.num_seqs) * d.num_kv_heads * (ceil_div(max_ctx, 16) + 1) < (int64_t(1) << 30) &&
           int64_t(d.num_pool_blocks) * d.num_kv_heads * std::max(1, d.block_size / 16) < (int64_t(1) << 31);
}

int make_plan(const kvc_attn_desc *d, Plan *pl) {
    if (!d) return KVC_ERR_NULL;
    if (d->num_seqs < 0 || d->num_q_heads <= 0 || d->num_kv_heads <= 0 || d->head_dim <= 0 ||
        d->block_size <= 0 || d->max_blocks_per_seq <= 0 || d->num_pool_blocks <= 0 ||
        d->max_context_len < 0 || d->partition_tokens < 0 || d->reserved != 0)
        return KVC_ERR_BAD_SHAPE;
    if (d->num_q_heads % d->num_kv_heads != 0) return KVC_ERR_BAD_SHAPE;
    if (d->dtype != KVC_F32 && d->dtype != KVC_BF16) return KVC_ERR_BAD_DTYPE;
    if (d->head_dim != 64 && d->head_dim != 128) return KVC_ERR_UNSUPPORTED;
    if (!is_pow2(d->block_size) || d->block_size > 256) return KVC_ERR_UNSUPPORTED;
    const int64_t table_tokens = int64_t(d->max_blocks_per_seq) * d->block_size;
    if (table_tokens > 0x40000000) return KVC_ERR_BAD_SHAPE;
    if (d->max_context_len > table_tokens) return KVC_ERR_BAD_SHAPE;
    const int max_ctx = d->max_context_len ? d->max_context_len : int(table_tokens);
    if (d->partition_tokens % 16 != 0) return KVC_ERR_BAD_SHAPE;
    if (d->partition_tokens > (d->kernel == KVC_KERNEL_MFMA_BALANCED ? kMaxBalancedChunkTokens : kMaxPartitionTokens))
        return KVC_ERR_BAD_SHAPE;

    int kernel = d->kernel;
    if (kernel < KVC_KERNEL_AUTO || kernel > KVC_KERNEL_MFMA_BALANCED) return KVC_ERR_BAD_SHAPE;
    if (kernel == KVC_KERNEL_AUTO)
        kernel = balanced_ok(*d, max_ctx) ? KVC_KERNEL_MFMA_BALANCED
                 : mfma_ok(*d)            ? KVC_KERNEL_MFMA
                                          : KVC_KERNEL_VALU;
    if ((kernel == KVC_KERNEL_MFMA || kernel == KVC_KERNEL_MFMA_LDS) && !mfma_ok(*d)) return KVC_ERR_UNSUPPORTED;
    if (kernel == KVC_KERNEL_MFMA_BALANCED && !balanced_ok(*d, max_ctx)) return KVC_ERR_UNSUPPORTED;

    const int64_t rows = int64_t(d->num_seqs) * d->num_q_heads;
    constexpr uint64_t kHeader = kvc::kWorkspaceHeaderBytes;
    if (kernel == KVC_KERNEL_MFMA_BALANCED) {
        // One launch: cut rows are merged by the last worker to arrive.  A wavefront never takes
        // fewer than min_chunk tiles; the workspace is two partial slots per wavefront.
        const int64_t max_tiles = ceil_div(max_ctx, 16);
        const int min_chunk = d->partition_tokens ? d->partition_tokens / 16
                                                  : int(std::max<int64_t>(4, ceil_div(max_tiles, 32)));
        const int group = d->num_q_heads / d->num_kv_heads;
        const uint64_t slots = uint64_t(kvc::kNumCUs) * kvc::kWaves * 2;
        pl->kernel = kernel;
        pl->partition_tokens = min_chunk * 16;
        pl->min_chunk_tiles = min_chunk;
        pl->max_partitions = 2;           // partial slots per worker
        pl->partial_grid = kvc::kNumCUs;  // 4 wavefronts per CU: one worker per SIMD
        pl->merge_grid = 0;
        pl->max_context_len = max_ctx;
        const uint64_t acc = slots * group * d->head_dim * sizeof(float);
        pl->acc_offset = kHeader;
        pl->ml_offset = (kHeader + acc + 255) & ~uint64_t(255);
        pl->workspace_bytes = pl->ml_offset + slots * group * 2 * sizeof(float);
        return KVC_OK;
    }

    const int group = d->num_q_heads / d->num_kv_heads;
    const int64_t base_items = kernel == KVC_KERNEL_VALU
                                   ? int64_t(d->num_seqs) * (d->num_q_heads / kvc::valu_head_chunk(group))
                                   : int64_t(d->num_seqs) * d->num_kv_heads;
    int pt = d->partition_tokens;
    if (pt == 0) {
        // Short partitions spread a skewed length mix over the 256 CUs; longer ones keep the
        // grid (mostly idle workgroups when max_context_len is loose) and the workspace small.
        if (max_ctx <= 256) {
            pt = int(ceil_div(max_ctx, 16) * 16);
        } else {
            pt = 256;
            while (pt < kMaxPartitionTokens && base_items * ceil_div(max_ctx, pt) > 16384) pt *= 2;
        }
    }
    const int64_t parts = ceil_div(max_ctx, pt);
    if (base_items * parts > kMaxGrid || rows * parts > kMaxGrid) return KVC_ERR_BAD_SHAPE;

    pl->kernel = kernel;
    pl->partition_tokens = pt;
    pl->max_partitions = int(parts);
    pl->partial_grid = base_items * parts;
    pl->merge_grid = parts > 1 ? ceil_div(rows, kvc::kWaves) : 0;
    pl->max_context_len = max_ctx;
    pl->min_chunk_tiles = 0;
    pl->acc_offset = kHeader;
    if (parts > 1) {
        const uint64_t acc = uint64_t(rows) * parts * d->head_dim * sizeof(float);
        pl->ml_offset = (kHeader + acc + 255) & ~uint64_t(255);
        pl->workspace_bytes = pl->ml_offset + uint64_t(rows) * parts * 2 * sizeof(float);
    } else {
        pl->ml_offset = 0;
        pl->workspace_bytes = 0;
    }
    return KVC_OK;
}

kvc::AttnParams make_params(const kvc_attn_desc &d, const Plan &pl, float scale) {
    kvc::AttnParams p;
    p.num_seqs = d.num_seqs;
    p.num_q_heads = d.num_q_heads;
    p.num_kv_heads = d.num_kv_heads;
    p.group = d.num_q_heads / d.num_kv_heads;
    p.block_size = d.block_size;
    p.block_size_log2 = ilog2(d.block_size);
    p.max_blocks_per_seq = d.max_blocks_per_seq;
    p.partition_tokens = pl.partition_tokens;
    p.max_partitions = pl.max_partitions;
    p.k_via_lds = pl.kernel == KVC_KERNEL_MFMA_LDS;
    p.min_chunk_tiles = pl.min_chunk_tiles;
    p.max_context_len = pl.max_context_len;
    p.scale = scale;
    p.scale_log2e = float(double(scale) * 1.4426950408889634);
    return p;
}

int check_workspace(const Plan &pl, void *workspace, size_t workspace_bytes, kvc::Workspace *ws) {
    ws->acc = nullptr;
    ws->ml = nullptr;
    ws->cnt = nullptr;
    if (pl.workspace_bytes == 0) return KVC_OK;
    if (!workspace || workspace_bytes < pl.workspace_bytes) return KVC_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return KVC_ERR_ALIGN;
    unsigned char *base = static_cast<unsigned char *>(workspace);
    ws->cnt = reinterpret_cast<int32_t *>(base);
    ws->acc = reinterpret_cast<float *>(base + pl.acc_offset);
    ws->ml = reinterpret_cast<float *>(base + pl.ml_offset);
    return KVC_OK;
}

int run_partial(const void *q, const void *k_cache, const void *v_cache, const int32_t *block_tables,
                const int32_t *context_lens, float scale, void *out, const kvc_attn_desc *desc,
                const Plan &pl, kvc::Workspace ws, hipStream_t stream) {
    const kvc::AttnParams p = make_params(*desc, pl, scale);
    hipError_t e;
    if (pl.kernel == KVC_KERNEL_VALU)
        e = kvc::launch_partial_valu(q, k_cache, v_cache, block_tables, context_lens, out, ws, p,
                                     desc->dtype, desc->head_dim, int(pl.partial_grid), stream);
    else if (pl.kernel == KVC_KERNEL_MFMA_BALANCED)
        e = kvc::launch_partial_mfma_stream(q, k_cache, v_cache, block_tables, context_lens, out,
                                            ws, p, int(pl.partial_grid), 0, kvc::Schedule{}, stream);
    else
        e = kvc::launch_partial_mfma(q, k_cache, v_cache, block_tables, context_lens, out, ws, p,
                                     int(pl.partial_grid), stream);
    return e == hipSuccess ? KVC_OK : hip_failed(e);
}

int run_merge(const int32_t *context_lens, void *out, const kvc_attn_desc *desc, const Plan &pl,
              kvc::Workspace ws, hipStream_t stream) {
    if (pl.merge_grid == 0) return KVC_OK;
    const kvc::AttnParams p = make_params(*desc, pl, 1.0f);
    const hipError_t e = kvc::launch_merge(context_lens, out, ws, p, desc->dtype, desc->head_dim,
                                           pl.kernel != KVC_KERNEL_VALU, int(pl.merge_grid), stream);
    return e == hipSuccess ? KVC_OK : hip_failed(e);
}

// Layout of a schedule buffer for a descriptor served by the balanced kernel.
struct ScheduleLayout {
    uint64_t pref_off, ctx_off, plans_off, tiles_off, bytes;
    int stride;
};

bool schedule_layout(const kvc_attn_desc &d, const Plan &pl, ScheduleLayout *L) {
    if (pl.kernel != KVC_KERNEL_MFMA_BALANCED) return false;
    const int64_t workers = int64_t(kvc::kNumCUs) * kvc::kWaves;
    const int64_t units_per_tile = d.block_size >= 16 ? 1 : 16 / d.block_size;
    // no worker takes more flat units than this, whatever the context lengths turn out to be
    const int64_t max_units = int64_t(d.num_seqs) * d.num_kv_heads * (ceil_div(pl.max_context_len, 16) + 1);
    const int64_t chunk = std::max<int64_t>(pl.min_chunk_tiles, ceil_div(max_units, workers));
    const int64_t stride = chunk * units_per_tile;
    if (stride > (int64_t(1) << 28)) return false;
    auto up = [](uint64_t x) { return (x + 255) & ~uint64_t(255); };
    L->stride = int(stride);
    L->pref_off = 0;
    L->ctx_off = up(uint64_t(d.num_seqs + 2) * 4);
    L->plans_off = L->ctx_off + up(uint64_t(d.num_seqs) * 4);
    L->tiles_off = L->plans_off + up(uint64_t(workers) * 16 * 4);
    L->bytes = L->tiles_off + up(uint64_t(workers) * uint64_t(stride) * 4);
    return true;
}

kvc::Schedule schedule_view(void *base, const ScheduleLayout &L) {
    auto *b = static_cast<unsigned char *>(base);
    kvc::Schedule s;
    s.pref = reinterpret_cast<int *>(b + L.pref_off);
    s.ctx = reinterpret_cast<int *>(b + L.ctx_off);
    s.plans = reinterpret_cast<int *>(b + L.plans_off);
    s.tiles = reinterpret_cast<int *>(b + L.tiles_off);
    s.stride = L.stride;
    return s;
}

int check_attn_args(const void *q, const void *k_cache, const void *v_cache,
                    const int32_t *block_tables, const int32_t *context_lens, float scale,
                    const void *out) {
    if (!q || !k_cache || !v_cache || !block_tables || !context_lens || !out) return KVC_ERR_NULL;
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out))
        return KVC_ERR_ALIGN;
    if (!isfinite(scale)) return KVC_ERR_BAD_SHAPE;
    return KVC_OK;
}

int check_pools(const kvc_pool *src, const kvc_pool *dst, const int64_t *mapping, int64_t num_pairs) {
    if (!src || !dst) return KVC_ERR_NULL;
    if (num_pairs < 0) return KVC_ERR_BAD_SHAPE;
    for (const kvc_pool *pl : {src, dst}) {
        if (pl->num_blocks <= 0 || pl->block_bytes <= 0 || pl->num_planes <= 0 || pl->reserved != 0)
            return KVC_ERR_BAD_SHAPE;
        if (pl->num_planes > 65535) return KVC_ERR_UNSUPPORTED;
        if (pl->block_bytes % 16 != 0) return KVC_ERR_ALIGN;
        if (pl->num_planes > 1) {
            if (pl->plane_stride_bytes % 16 != 0) return KVC_ERR_ALIGN;
            if (pl->plane_stride_bytes / pl->block_bytes < pl->num_blocks) return KVC_ERR_BAD_SHAPE;
        }
    }
    if (src->block_bytes != dst->block_bytes || src->num_planes != dst->num_planes)
        return KVC_ERR_BAD_SHAPE;
    if (num_pairs == 0) return KVC_OK;
    if (!src->base || !dst->base || !mapping) return KVC_ERR_NULL;
    if (!aligned16(src->base) || !aligned16(dst->base)) return KVC_ERR_ALIGN;
    const int64_t slabs = ceil_div(src->block_bytes, kvc::kCopySlabBytes);
    if (num_pairs > kMaxGrid / slabs) return KVC_ERR_BAD_SHAPE;
    return KVC_OK;
}

}  // namespace

extern "C" {

int kvc_version(void) { return 200; }

const char *kvc_status_string(int status) {
    switch (status) {
        case KVC_OK: return "ok";
        case KVC_ERR_NULL: return "a required pointer is NULL";
        case KVC_ERR_BAD_SHAPE: return "a size is non-positive or inconsistent";
        case KVC_ERR_BAD_DTYPE: return "unknown dtype";
        case KVC_ERR_UNSUPPORTED: return "shape or option not implemented";
        case KVC_ERR_WORKSPACE: return "workspace missing or too small";
        case KVC_ERR_ALIGN: return "pointer or stride not aligned";
        case KVC_ERR_LAUNCH: return "HIP call failed (see kvc_last_hip_error)";
        case KVC_ERR_BAD_INDEX: return "index out of range";
        case KVC_ERR_DUPLICATE: return "destination block listed twice";
        case KVC_ERR_OVERLAP: return "source and destination blocks overlap in one pool";
        default: return "unknown status";
    }
}

int kvc_last_hip_error(void) { return g_last_hip_error; }

int kvc_attn_plan(const kvc_attn_desc *desc, kvc_attn_plan_info *plan) {
    if (!plan) return KVC_ERR_NULL;
    Plan pl;
    const int rc = make_plan(desc, &pl);
    if (rc != KVC_OK) return rc;
    plan->kernel = pl.kernel;
    plan->partition_tokens = pl.partition_tokens;
    plan->max_partitions = pl.max_partitions;
    plan->partial_grid = int32_t(pl.partial_grid);
    plan->merge_grid = int32_t(pl.merge_grid);
    plan->reserved = 0;
    plan->workspace_bytes = pl.workspace_bytes;
    return KVC_OK;
}

size_t kvc_paged_attention_decode_workspace_bytes(const kvc_attn_desc *desc) {
    Plan pl;
    return make_plan(desc, &pl) == KVC_OK ? size_t(pl.workspace_bytes) : 0;
}

int kvc_paged_attention_decode_workspace_init(void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (workspace_bytes == 0) return KVC_OK;
    if (!workspace || workspace_bytes < kvc::kWorkspaceHeaderBytes) return KVC_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return KVC_ERR_ALIGN;
    const hipError_t e = kvc::launch_workspace_init(workspace, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? KVC_OK : hip_failed(e);
}

int kvc_paged_attention_decode_partial(const void *q, const void *k_cache, const void *v_cache,
                                       const int32_t *block_tables, const int32_t *context_lens,
                                       float scale, void *out, const kvc_attn_desc *desc,
                                       void *workspace, size_t workspace_bytes, void *hip_stream) {
    Plan pl;
    int rc = make_plan(desc, &pl);
    if (rc != KVC_OK) return rc;
    if (desc->num_seqs == 0) return KVC_OK;
    rc = check_attn_args(q, k_cache, v_cache, block_tables, context_lens, scale, out);
    if (rc != KVC_OK) return rc;
    kvc::Workspace ws;
    rc = check_workspace(pl, workspace, workspace_bytes, &ws);
    if (rc != KVC_OK) return rc;
    return run_partial(q, k_cache, v_cache, block_tables, context_lens, scale, out, desc, pl, ws,
                       static_cast<hipStream_t>(hip_stream));
}

int kvc_paged_attention_decode_merge(const int32_t *context_lens, void *out,
                                     const kvc_attn_desc *desc, void *workspace,
                                     size_t workspace_bytes, void *hip_stream) {
    Plan pl;
    int rc = make_plan(desc, &pl);
    if (rc != KVC_OK) return rc;
    if (desc->num_seqs == 0) return KVC_OK;
    if (!context_lens || !out) return KVC_ERR_NULL;
    if (!aligned16(out)) return KVC_ERR_ALIGN;
    kvc::Workspace ws;
    rc = check_workspace(pl, workspace, workspace_bytes, &ws);
    if (rc != KVC_OK) return rc;
    return run_merge(context_lens, out, desc, pl, ws, static_cast<hipStream_t>(hip_stream));
}

int kvc_paged_attention_decode(const void *q, const void *k_cache, const void *v_cache,
                               const int32_t *block_tables, const int32_t *context_lens,
                               float scale, void *out, const kvc_attn_desc *desc, void *workspace,
                               size_t workspace_bytes, void *hip_stream) {
    Plan pl;
    int rc = make_plan(desc, &pl);
    if (rc != KVC_OK) return rc;
    if (desc->num_seqs == 0) return KVC_OK;
    rc = check_attn_args(q, k_cache, v_cache, block_tables, context_lens, scale, out);
    if (rc != KVC_OK) return rc;
    kvc::Workspace ws;
    rc = check_workspace(pl, workspace, workspace_bytes, &ws);
    if (rc != KVC_OK) return rc;
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    rc = run_partial(q, k_cache, v_cache, block_tables, context_lens, scale, out, desc, pl, ws, stream);
    if (rc != KVC_OK) return rc;
    return run_merge(context_lens, out, desc, pl, ws, stream);
}

int kvc_paged_attention_decode_noalloc(const void *q, const void *k_cache, const void *v_cache,
                                       const int32_t *block_tables, const int32_t *context_lens,
                                       float scale, void *out, const kvc_attn_desc *desc,
                                       void *hip_stream) {
    Plan pl;
    int rc = make_plan(desc, &pl);
    if (rc != KVC_OK) return rc;
    if (pl.workspace_bytes > kScratchBytes) return KVC_ERR_WORKSPACE;
    if (desc->num_seqs == 0) return KVC_OK;
    rc = check_attn_args(q, k_cache, v_cache, block_tables, context_lens, scale, out);
    if (rc != KVC_OK) return rc;
    void *base = nullptr;
    const hipError_t e = scratch_of_current_device(&base);
    if (e != hipSuccess) return hip_failed(e);
    kvc::Workspace ws;
    rc = check_workspace(pl, base, kScratchBytes, &ws);
    if (rc != KVC_OK) return rc;
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    rc = run_partial(q, k_cache, v_cache, block_tables, context_lens, scale, out, desc, pl, ws, stream);
    if (rc != KVC_OK) return rc;
    return run_merge(context_lens, out, desc, pl, ws, stream);
}

size_t kvc_attn_schedule_bytes(const kvc_attn_desc *desc) {
    Plan pl;
    ScheduleLayout L;
    if (make_plan(desc, &pl) != KVC_OK || !schedule_layout(*desc, pl, &L)) return 0;
    return size_t(L.bytes);
}

int kvc_attn_schedule_build(const int32_t *block_tables, const int32_t *context_lens,
                            const kvc_attn_desc *desc, void *schedule, size_t schedule_bytes,
                            void *hip_stream) {
    Plan pl;
    int rc = make_plan(desc, &pl);
    if (rc != KVC_OK) return rc;
    ScheduleLayout L;
    if (!schedule_layout(*desc, pl, &L)) return KVC_ERR_UNSUPPORTED;
    if (!schedule || schedule_bytes < L.bytes) return KVC_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(schedule) & 255u) return KVC_ERR_ALIGN;
    if (desc->num_seqs == 0) return KVC_OK;
    if (!block_tables || !context_lens) return KVC_ERR_NULL;
    const kvc::AttnParams p = make_params(*desc, pl, 1.0f);
    const hipError_t e = kvc::launch_partial_mfma_stream(nullptr, nullptr, nullptr, block_tables, context_lens,
                                                         nullptr, kvc::Workspace{}, p, int(pl.partial_grid), 1,
                                                         schedule_view(schedule, L),
                                                         static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? KVC_OK : hip_failed(e);
}

int kvc_paged_attention_decode_scheduled(const void *q, const void *k_cache, const void *v_cache,
                                         const void *schedule, size_t schedule_bytes, float scale,
                                         void *out, const kvc_attn_desc *desc, void *workspace,
                                         size_t workspace_bytes, void *hip_stream) {
    Plan pl;
    int rc = make_plan(desc, &pl);
    if (rc != KVC_OK) return rc;
    ScheduleLayout L;
    if (!schedule_layout(*desc, pl, &L)) return KVC_ERR_UNSUPPORTED;
    if (!schedule || schedule_bytes < L.bytes) return KVC_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(schedule) & 255u) return KVC_ERR_ALIGN;
    if (desc->num_seqs == 0) return KVC_OK;
    if (!q || !k_cache || !v_cache || !out) return KVC_ERR_NULL;
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out)) return KVC_ERR_ALIGN;
    if (!isfinite(scale)) return KVC_ERR_BAD_SHAPE;
    kvc::Workspace ws;
    rc = check_workspace(pl, workspace, workspace_bytes, &ws);
    if (rc != KVC_OK) return rc;
    const kvc::AttnParams p = make_params(*desc, pl, scale);
    const hipError_t e = kvc::launch_partial_mfma_stream(q, k_cache, v_cache, nullptr, nullptr, out, ws, p,
                                                         int(pl.partial_grid), 2,
                                                         schedule_view(const_cast<void *>(schedule), L),
                                                         static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? KVC_OK : hip_failed(e);
}

int kvc_validate_attention_inputs(const int32_t *block_tables, const int32_t *context_lens,
                                  const kvc_attn_desc *desc, void *hip_stream) {
    Plan pl;
    const int rc = make_plan(desc, &pl);
    if (rc != KVC_OK) return rc;
    if (desc->num_seqs == 0) return KVC_OK;
    if (!block_tables || !context_lens) return KVC_ERR_NULL;
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    std::vector<int32_t> lens(desc->num_seqs);
    std::vector<int32_t> tables(size_t(desc->num_seqs) * desc->max_blocks_per_seq);
    hipError_t e = hipMemcpyAsync(lens.data(), context_lens, lens.size() * sizeof(int32_t),
                                  hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess)
        e = hipMemcpyAsync(tables.data(), block_tables, tables.size() * sizeof(int32_t),
                           hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return hip_failed(e);
    for (int n = 0; n < desc->num_seqs; ++n) {
        if (lens[n] < 0 || lens[n] > pl.max_context_len) return KVC_ERR_BAD_INDEX;
        const int nblk = int(ceil_div(lens[n], desc->block_size));
        for (int b = 0; b < nblk; ++b) {
            const int32_t id = tables[size_t(n) * desc->max_blocks_per_seq + b];
            if (id < 0 || id >= desc->num_pool_blocks) return KVC_ERR_BAD_INDEX;
        }
    }
    return KVC_OK;
}

int kvc_paged_attention_prefill(const void *q, const void *k_cache, const void *v_cache,
                                const int32_t *block_tables, const int32_t *context_lens,
                                const int32_t *q_start, float scale, void *out,
                                const kvc_attn_desc *desc, int32_t total_q, int32_t max_query_len,
                                void *hip_stream) {
    Plan pl;
    int rc = make_plan(desc, &pl);
    if (rc != KVC_OK) return rc;
    if (total_q < 0 || max_query_len < 0) return KVC_ERR_BAD_SHAPE;
    if (desc->num_seqs == 0 || total_q == 0 || max_query_len == 0) return KVC_OK;
    if (!q_start) return KVC_ERR_NULL;
    rc = check_attn_args(q, k_cache, v_cache, block_tables, context_lens, scale, out);
    if (rc != KVC_OK) return rc;
    const bool on_mfma = desc->dtype == KVC_BF16 && desc->head_dim == 128 &&
                         desc->num_q_heads / desc->num_kv_heads <= 16;
    if (!on_mfma) {
        // vector-ALU kernel, one query row per "sequence" of its grid, one partition, no workspace
        kvc::AttnParams vp = make_params(*desc, pl, scale);
        vp.num_seqs = total_q;
        vp.partition_tokens = 1 << 30;
        vp.max_partitions = 1;
        vp.max_context_len = desc->max_blocks_per_seq * desc->block_size;
        const int64_t grid = int64_t(total_q) * (desc->num_q_heads / kvc::valu_head_chunk(vp.group));
        if (grid > kMaxGrid) return KVC_ERR_BAD_SHAPE;
        const hipError_t e = kvc::launch_prefill_valu(q, k_cache, v_cache, block_tables, context_lens, q_start,
                                                      desc->num_seqs, max_query_len, out, vp, desc->dtype,
                                                      desc->head_dim, int(grid), static_cast<hipStream_t>(hip_stream));
        return e == hipSuccess ? KVC_OK : hip_failed(e);
    }
    kvc::PrefillParams p;
    p.num_seqs = desc->num_seqs;
    p.num_q_heads = desc->num_q_heads;
    p.num_kv_heads = desc->num_kv_heads;
    p.group = desc->num_q_heads / desc->num_kv_heads;
    p.heads_per_chunk = p.group % 2 == 0 ? 2 : 1;
    p.block_size = desc->block_size;
    p.block_size_log2 = ilog2(desc->block_size);
    p.tiles_per_block_log2 = desc->block_size >= 16 ? ilog2(desc->block_size / 16) : 0;
    p.max_blocks_per_seq = desc->max_blocks_per_seq;
    p.max_query_tiles = int(ceil_div(max_query_len, 64));
    p.scale_log2e = float(double(scale) * 1.4426950408889634);
    if (int64_t(p.num_q_heads / p.heads_per_chunk) * p.num_seqs * p.max_query_tiles > kMaxGrid)
        return KVC_ERR_BAD_SHAPE;
    // 32x32 tiles need a positive scale (their max is taken over raw scores); KVC_KERNEL_MFMA asks
    // for the 16x16-tile kernel whatever the shape
    const bool tiles32 = p.scale_log2e > 0.0f && desc->kernel != KVC_KERNEL_MFMA;
    const hipError_t e = tiles32 ? kvc::launch_prefill_mfma32(q, k_cache, v_cache, block_tables, context_lens, q_start,
                                                              out, p, static_cast<hipStream_t>(hip_stream))
                                 : kvc::launch_prefill_mfma(q, k_cache, v_cache, block_tables, context_lens, q_start,
                                                            out, p, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? KVC_OK : hip_failed(e);
}

int kvc_kv_cache_append(const void *k_new, const void *v_new, void *k_cache, void *v_cache,
                        const int32_t *block_tables, const int32_t *positions,
                        const kvc_attn_desc *desc, void *hip_stream) {
    Plan pl;
    const int rc = make_plan(desc, &pl);
    if (rc != KVC_OK) return rc;
    if (desc->num_seqs == 0) return KVC_OK;
    if (!k_new || !v_new || !k_cache || !v_cache || !block_tables || !positions) return KVC_ERR_NULL;
    if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) || !aligned16(v_cache))
        return KVC_ERR_ALIGN;
    const int row_bytes = desc->head_dim * (desc->dtype == KVC_F32 ? 4 : 2);
    const hipError_t e = kvc::launch_cache_append(
        k_new, v_new, k_cache, v_cache, block_tables, positions, desc->num_seqs, desc->num_kv_heads,
        row_bytes, ilog2(desc->block_size), desc->max_blocks_per_seq, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? KVC_OK : hip_failed(e);
}

int kvc_kv_block_copy(const kvc_pool *src, const kvc_pool *dst, const int64_t *block_mapping,
                      int64_t num_pairs, void *hip_stream) {
    const int rc = check_pools(src, dst, block_mapping, num_pairs);
    if (rc != KVC_OK) return rc;
    if (num_pairs == 0) return KVC_OK;
    const hipError_t e = kvc::launch_block_copy(*src, *dst, block_mapping, num_pairs,
                                                static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? KVC_OK : hip_failed(e);
}

int kvc_validate_block_mapping(const kvc_pool *src, const kvc_pool *dst,
                               const int64_t *block_mapping, int64_t num_pairs, void *hip_stream) {
    const int rc = check_pools(src, dst, block_mapping, num_pairs);
    if (rc != KVC_OK) return rc;
    if (num_pairs == 0) return KVC_OK;
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    std::vector<int64_t> map(size_t(num_pairs) * 2);
    hipError_t e = hipMemcpyAsync(map.data(), block_mapping, map.size() * sizeof(int64_t),
                                  hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return hip_failed(e);
    std::vector<int64_t> srcs(num_pairs), dsts(num_pairs);
    for (int64_t i = 0; i < num_pairs; ++i) {
        srcs[i] = map[2 * i];
        dsts[i] = map[2 * i + 1];
        if (srcs[i] < 0 || srcs[i] >= src->num_blocks || dsts[i] < 0 || dsts[i] >= dst->num_blocks)
            return KVC_ERR_BAD_INDEX;
    }
    std::sort(dsts.begin(), dsts.end());
    if (std::adjacent_find(dsts.begin(), dsts.end()) != dsts.end()) return KVC_ERR_DUPLICATE;
    // Pools that share memory: a block that is both read and written would race.
    const auto *sb = static_cast<const unsigned char *>(src->base);
    const auto *db = static_cast<const unsigned char *>(dst->base);
    const int64_t s_extent = (src->num_planes > 1 ? (src->num_planes - 1) * src->plane_stride_bytes : 0) +
                             src->num_blocks * src->block_bytes;
    const int64_t d_extent = (dst->num_planes > 1 ? (dst->num_planes - 1) * dst->plane_stride_bytes : 0) +
                             dst->num_blocks * dst->block_bytes;
    if (sb < db + d_extent && db < sb + s_extent) {
        if (sb != db) return KVC_ERR_OVERLAP;  // partially overlapping pools: no safe reading
        std::sort(srcs.begin(), srcs.end());
        for (int64_t s : srcs)
            if (std::binary_search(dsts.begin(), dsts.end(), s)) return KVC_ERR_OVERLAP;
    }
    return KVC_OK;
}

}  // extern "C"
