/*
 * CPU oracle for the paged-KV decode path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition the HIP kernels are checked against.
 * It shares no code, header, table or helper with the HIP path, and nothing in
 * the product imports it: only the tests, the smoke check and the benchmark's
 * cpu_baseline leg call it.
 *
 * What it computes
 * ----------------
 * The paper (Section 1; Section 3.3.1) hands out the KV cache in fixed-size
 * token blocks and lets a request's blocks sit anywhere in the pool; each
 * decode iteration reads a request's whole KV through its block list
 * (Section 3.3.2: iteration time grows with the number of tokens in the
 * batch), and preemption by swapping moves a request's KV values out and
 * back (Section 2.5, Section 3.5: cost linear in the sequence length).  The
 * paper gives no formula for attention: it is the textbook one, written out
 * below in fp64 with no blocking, fusion or reordering:
 *
 *   for sequence n, query head h, kv head g = h / (Hq / Hkv), L = context_lens[n]:
 *     s[t]   = scale * sum_d q[n][h][d] * K[blk(t)][g][t % Bs][d],  blk(t) = block_tables[n][t / Bs]
 *     m      = max_t s[t];   p[t] = exp(s[t] - m);   Z = sum_t p[t]
 *     out[n][h][d] = ( sum_t p[t] * V[blk(t)][g][t % Bs][d] ) / Z
 *   L == 0 gives a row of zeros (reading chosen where the definition is empty).
 *
 * Stored inputs (fp32 or bf16 bit patterns) widen to fp64 exactly, so the
 * oracle sees the same values the GPU does.
 *
 * Pins (tests/test_oracle_pins.py): brute-force dense attention on the
 * un-paged sequence, a library attention routine in fp64, hand-derived closed
 * forms under tests/golden/, placement / permutation / GQA / poison
 * invariants.  No function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F64 = 2 };

/* one stored element -> double (exact) */
static double widen(const void *base, int64_t idx, int dtype)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[idx];
    if (dtype == ORACLE_F64)
        return ((const double *)base)[idx];
    /* bf16: the 16 stored bits are the top half of an IEEE fp32 */
    uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* layout accessor: pool[block][kv_head][slot][d] */
static int64_t pool_index(int64_t block, int kv_head, int slot, int d,
                          int num_kv_heads, int block_size, int head_dim)
{
    return ((block * num_kv_heads + kv_head) * (int64_t)block_size + slot) * head_dim + d;
}

/* One (sequence, query head) row of the definition. `s` is scratch of L doubles. */
static void attention_row(const void *q, const void *k_cache, const void *v_cache,
                          const int32_t *block_tables, int L, double scale, double *out_row,
                          int dtype, int n, int h, int num_q_heads, int num_kv_heads,
                          int head_dim, int block_size, int max_blocks_per_seq, double *s)
{
    const int group = num_q_heads / num_kv_heads;
    const int g = h / group;
    const int32_t *table = block_tables + (int64_t)n * max_blocks_per_seq;
    const int64_t qbase = ((int64_t)n * num_q_heads + h) * head_dim;

    for (int d = 0; d < head_dim; ++d)
        out_row[d] = 0.0;
    if (L <= 0)
        return;

    for (int t = 0; t < L; ++t) {
        int64_t blk = table[t / block_size];
        int slot = t % block_size;
        double dot = 0.0;
        for (int d = 0; d < head_dim; ++d)
            dot += widen(q, qbase + d, dtype) *
                   widen(k_cache, pool_index(blk, g, slot, d, num_kv_heads, block_size, head_dim), dtype);
        s[t] = scale * dot;
    }
    double m = s[0];
    for (int t = 1; t < L; ++t)
        if (s[t] > m)
            m = s[t];
    double Z = 0.0;
    for (int t = 0; t < L; ++t) {
        s[t] = exp(s[t] - m); /* now p[t] */
        Z += s[t];
    }
    for (int t = 0; t < L; ++t) {
        int64_t blk = table[t / block_size];
        int slot = t % block_size;
        for (int d = 0; d < head_dim; ++d)
            out_row[d] += s[t] *
                          widen(v_cache, pool_index(blk, g, slot, d, num_kv_heads, block_size, head_dim), dtype);
    }
    for (int d = 0; d < head_dim; ++d)
        out_row[d] /= Z;
}

/*
 * out: [num_seqs][num_q_heads][head_dim] doubles.
 * rows: optional list of (sequence, query head) pairs, [n_rows][2]; when NULL
 * every row is computed, otherwise only the listed rows of `out` are written.
 * num_threads <= 1 runs serially; otherwise rows are spread over that many
 * OpenMP threads (each row is still the serial definition above).
 * Returns 0, or -1 on a bad argument / allocation failure.
 */
int oracle_paged_attention_decode(const void *q, const void *k_cache, const void *v_cache,
                                  const int32_t *block_tables, const int32_t *context_lens,
                                  double scale, double *out, int dtype, int num_seqs,
                                  int num_q_heads, int num_kv_heads, int head_dim, int block_size,
                                  int max_blocks_per_seq, const int32_t *rows, int64_t n_rows,
                                  int num_threads)
{
    if (num_kv_heads <= 0 || num_q_heads % num_kv_heads != 0 || head_dim <= 0 || block_size <= 0)
        return -1;
    const int64_t total = rows ? n_rows : (int64_t)num_seqs * num_q_heads;
    int max_len = 0;
    for (int n = 0; n < num_seqs; ++n)
        if (context_lens[n] > max_len)
            max_len = context_lens[n];
    if (max_len > (int64_t)max_blocks_per_seq * block_size)
        return -1;
    int failed = 0;
    if (num_threads < 1)
        num_threads = 1;
#ifdef _OPENMP
#pragma omp parallel num_threads(num_threads)
#endif
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)(max_len > 0 ? max_len : 1));
        if (!s) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        }
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 1)
#endif
        for (int64_t r = 0; r < total; ++r) {
            if (!s)
                continue;
            int n = rows ? rows[2 * r] : (int)(r / num_q_heads);
            int h = rows ? rows[2 * r + 1] : (int)(r % num_q_heads);
            attention_row(q, k_cache, v_cache, block_tables, context_lens[n], scale,
                          out + ((int64_t)n * num_q_heads + h) * head_dim, dtype, n, h,
                          num_q_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq, s);
        }
        free(s);
    }
    return failed ? -1 : 0;
}

int oracle_num_threads_available(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Block copy (swap-out / swap-in / reuse, Section 2.5 and Section 3.3.1): for
 * each pair (s, d) and each plane, dst[plane][d][:] = src[plane][s][:], byte for
 * byte.  A plane is K or V of one layer.  Pools: [plane][block][block_bytes] with
 * the given plane strides.  Everything else in dst is left alone.
 */
int oracle_kv_block_copy(const uint8_t *src, uint8_t *dst, int64_t block_bytes, int num_planes,
                         int64_t src_plane_stride, int64_t dst_plane_stride,
                         int64_t src_num_blocks, int64_t dst_num_blocks,
                         const int64_t *mapping, int64_t n_pairs)
{
    for (int64_t i = 0; i < n_pairs; ++i) {
        int64_t s = mapping[2 * i], d = mapping[2 * i + 1];
        if (s < 0 || s >= src_num_blocks || d < 0 || d >= dst_num_blocks)
            return -1;
    }
    for (int p = 0; p < num_planes; ++p)
        for (int64_t i = 0; i < n_pairs; ++i)
            memcpy(dst + p * dst_plane_stride + mapping[2 * i + 1] * block_bytes,
                   src + p * src_plane_stride + mapping[2 * i] * block_bytes, (size_t)block_bytes);
    return 0;
}

/*
 * Append one token per sequence (the cache write before each decode step; Section 1 and 3.1):
 * for every sequence n with positions[n] >= 0 and every kv head h,
 *   cache[block_tables[n][pos / Bs]][h][pos % Bs][:] = new[n][h][:]   (bytewise, K and V).
 * row_bytes = head_dim * element size.  Returns -1 if a block id or position is out of range.
 */
int oracle_kv_cache_append(const uint8_t *k_new, const uint8_t *v_new, uint8_t *k_cache,
                           uint8_t *v_cache, const int32_t *block_tables, const int32_t *positions,
                           int num_seqs, int num_kv_heads, int64_t row_bytes, int block_size,
                           int max_blocks_per_seq, int64_t num_pool_blocks)
{
    for (int n = 0; n < num_seqs; ++n) {
        int pos = positions[n];
        if (pos < 0)
            continue;
        if (pos / block_size >= max_blocks_per_seq)
            return -1;
        int64_t blk = block_tables[(int64_t)n * max_blocks_per_seq + pos / block_size];
        if (blk < 0 || blk >= num_pool_blocks)
            return -1;
    }
    for (int n = 0; n < num_seqs; ++n) {
        int pos = positions[n];
        if (pos < 0)
            continue;
        int64_t blk = block_tables[(int64_t)n * max_blocks_per_seq + pos / block_size];
        int slot = pos % block_size;
        for (int h = 0; h < num_kv_heads; ++h) {
            int64_t dst = (((blk * num_kv_heads + h) * block_size) + slot) * row_bytes;
            int64_t src = ((int64_t)n * num_kv_heads + h) * row_bytes;
            memcpy(k_cache + dst, k_new + src, (size_t)row_bytes);
            memcpy(v_cache + dst, v_new + src, (size_t)row_bytes);
        }
    }
    return 0;
}

/*
 * Causal attention of several query positions per sequence over the block-allocated cache:
 * the recomputation path of a preempted request re-runs prefill over its prompt and generated
 * tokens (Section 2.5 and 3.5: cost quadratic in the sequence length), and chunked prefill
 * attends a chunk of new positions to everything before it.
 *
 * Sequence n has S = context_lens[n] tokens in the cache and Qn = q_start[n+1] - q_start[n]
 * query rows; query row i sits at position pos = S - Qn + i and attends to tokens 0 .. pos:
 *   s[t] = scale * q . K[t],  p = softmax over t <= pos,  out = sum_t p[t] V[t]      (fp64)
 * With Qn == 1 this is the decode definition above.  Returns -1 on inconsistent arguments
 * (Qn > S, negative sizes).
 * q, out: [total_q][num_q_heads][head_dim] (out in doubles).
 */
int oracle_paged_attention_prefill(const void *q, const void *k_cache, const void *v_cache,
                                   const int32_t *block_tables, const int32_t *context_lens,
                                   const int32_t *q_start, double scale, double *out, int dtype,
                                   int num_seqs, int num_q_heads, int num_kv_heads, int head_dim,
                                   int block_size, int max_blocks_per_seq, int num_threads)
{
    if (num_kv_heads <= 0 || num_q_heads % num_kv_heads != 0 || head_dim <= 0 || block_size <= 0)
        return -1;
    int max_len = 1;
    for (int n = 0; n < num_seqs; ++n) {
        int S = context_lens[n], Qn = q_start[n + 1] - q_start[n];
        if (S < 0 || Qn < 0 || Qn > S || S > (int64_t)max_blocks_per_seq * block_size)
            return -1;
        if (S > max_len)
            max_len = S;
    }
    const int group = num_q_heads / num_kv_heads;
    int failed = 0;
    if (num_threads < 1)
        num_threads = 1;
#ifdef _OPENMP
#pragma omp parallel num_threads(num_threads)
#endif
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)max_len);
        if (!s) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        }
        for (int n = 0; n < num_seqs && s; ++n) {
            const int S = context_lens[n], Qn = q_start[n + 1] - q_start[n];
            const int32_t *table = block_tables + (int64_t)n * max_blocks_per_seq;
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 1) nowait
#endif
            for (int64_t r = 0; r < (int64_t)Qn * num_q_heads; ++r) {
                const int i = (int)(r / num_q_heads), h = (int)(r % num_q_heads), g = h / group;
                const int pos = S - Qn + i;
                const int64_t qbase = (((int64_t)q_start[n] + i) * num_q_heads + h) * head_dim;
                double *o = out + qbase;
                for (int t = 0; t <= pos; ++t) {
                    int64_t blk = table[t / block_size];
                    double dot = 0.0;
                    for (int d = 0; d < head_dim; ++d)
                        dot += widen(q, qbase + d, dtype) *
                               widen(k_cache, pool_index(blk, g, t % block_size, d, num_kv_heads, block_size, head_dim), dtype);
                    s[t] = scale * dot;
                }
                double m = s[0];
                for (int t = 1; t <= pos; ++t)
                    if (s[t] > m)
                        m = s[t];
                double Z = 0.0;
                for (int t = 0; t <= pos; ++t) {
                    s[t] = exp(s[t] - m);
                    Z += s[t];
                }
                for (int d = 0; d < head_dim; ++d)
                    o[d] = 0.0;
                for (int t = 0; t <= pos; ++t) {
                    int64_t blk = table[t / block_size];
                    for (int d = 0; d < head_dim; ++d)
                        o[d] += s[t] * widen(v_cache, pool_index(blk, g, t % block_size, d, num_kv_heads, block_size, head_dim), dtype);
                }
                for (int d = 0; d < head_dim; ++d)
                    o[d] /= Z;
            }
        }
        free(s);
    }
    return failed ? -1 : 0;
}
