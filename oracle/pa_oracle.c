/*
 * CPU oracle for paged single-query attention and the two cache-maintenance
 * operations around it.  TEST INFRASTRUCTURE ONLY: tests, the smoke check and
 * the benchmark's CPU-baseline leg call this; the GPU library never does, and
 * this file shares no code, header or table with it.
 *
 * What it computes follows the paper's definitions, written out plainly in
 * fp64 with no blocking or reordering:
 *
 *   - Sec. 2.1, Eq. "attention-layer" (the per-token form):
 *       a_t = exp(q.k_t/sqrt(d)) / sum_u exp(q.k_u/sqrt(d)),  o = sum_t a_t v_t
 *     for the n = context_len tokens of a sequence, the query token included.
 *   - Sec. 4.1: the block-wise restatement of the same formula.  The keys and
 *     values of token t live in logical block t / B at offset t % B, and the
 *     block table maps that logical block to a physical block (Sec. 4.2).  The
 *     oracle walks the table, gathers the sequence's K and V into contiguous
 *     fp64 arrays and then applies the per-token formula, which is what the
 *     block-wise form equals in exact arithmetic.
 *   - Sec. 4.3 / 5.1(1): new K/V vectors are stored at the slot their block
 *     table position names (slot = physical_block * B + offset).
 *   - Sec. 4.4 / 5.1(3): copy-on-write copies a whole physical block.
 *   - Sec. 4.5 (swapping): whole blocks move between a GPU pool and a CPU pool.
 *
 * Cache layout (the paper leaves it open, Sec. 5.1(1)); element (block pb,
 * head h, offset off, dim d) of a cache array sits at index
 *       ((pb * H + h) * B + off) * D + d
 * i.e. an array [NB][H][B][D]; K and V use the same layout.
 *
 * Readings taken where the paper is silent: indices are 0-based; the scale
 * is an argument (the paper fixes 1/sqrt(d)), received as fp32 and widened;
 * stored fp16/bf16/fp32 bit patterns are decoded exactly to fp64 first;
 * context_len = 0 yields a zero row; a negative slot means "skip this token".
 *
 * The split-context functions follow the partition/merge definition that is
 * not in the paper (it comes with the benchmark spec): attention restricted
 * to tokens [p*PS, (p+1)*PS) gives (m_p, l_p, o_p); the merge is
 *   M = max_p m_p,  out = sum_p e^{m_p-M} l_p o_p / sum_p e^{m_p-M} l_p.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_F16 = 1, ORACLE_BF16 = 2 };

static int elem_bytes(int dtype) { return dtype == ORACLE_F32 ? 4 : 2; }

/* IEEE binary16 -> double, by fields. */
static double half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);               /* subnormal: f * 2^-10 * 2^-14 */
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)f / 1024.0, e - 15);
    return sign ? -v : v;
}

/* bfloat16 is the upper half of an IEEE binary32. */
static double bf16_bits_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

static double load_elem(const void *base, int64_t idx, int dtype)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[idx];
    if (dtype == ORACLE_F16)
        return half_bits_to_double(((const uint16_t *)base)[idx]);
    return bf16_bits_to_double(((const uint16_t *)base)[idx]);
}

static int64_t cache_index(int64_t pb, int h, int off, int d, int H, int B, int D)
{
    return ((pb * H + h) * B + off) * (int64_t)D + d;
}

/*
 * Gather tokens [t0, t1) of sequence s, head h into contiguous Kc, Vc
 * ([t1-t0][D], fp64) by walking the block table.
 */
static void gather_kv(double *Kc, double *Vc, const void *k_cache, const void *v_cache,
                      const int32_t *table_row, int t0, int t1, int h, int H, int D, int B, int dtype)
{
    for (int t = t0; t < t1; ++t) {
        int64_t pb = table_row[t / B];
        int off = t % B;
        for (int d = 0; d < D; ++d) {
            int64_t idx = cache_index(pb, h, off, d, H, B, D);
            Kc[(int64_t)(t - t0) * D + d] = load_elem(k_cache, idx, dtype);
            Vc[(int64_t)(t - t0) * D + d] = load_elem(v_cache, idx, dtype);
        }
    }
}

/*
 * Attention of one query over n contiguous tokens.  Writes o[D] = softmax-
 * weighted mean of V, and (optionally) the maximum logit m and the sum
 * l = sum_t exp(x_t - m).  n must be >= 1.
 */
static void attend(double *o, double *m_out, double *l_out, const double *qd, const double *Kc,
                   const double *Vc, int n, int D, double scale)
{
    double *x = (double *)malloc(sizeof(double) * (size_t)n);
    double m = -INFINITY;
    for (int t = 0; t < n; ++t) {
        double dot = 0.0;
        for (int d = 0; d < D; ++d)
            dot += qd[d] * Kc[(int64_t)t * D + d];
        x[t] = scale * dot;
        if (x[t] > m)
            m = x[t];
    }
    double l = 0.0;
    for (int d = 0; d < D; ++d)
        o[d] = 0.0;
    for (int t = 0; t < n; ++t) {
        double w = exp(x[t] - m);
        l += w;
        for (int d = 0; d < D; ++d)
            o[d] += w * Vc[(int64_t)t * D + d];
    }
    for (int d = 0; d < D; ++d)
        o[d] /= l;
    if (m_out)
        *m_out = m;
    if (l_out)
        *l_out = l;
    free(x);
}

/*
 * One output row: query row `qrow` of q ([rows][H][D]), head h, attending to the
 * first n tokens of sequence s.
 */
static void decode_row(double *o, const void *q, int64_t qrow, const void *k_cache,
                       const void *v_cache, const int32_t *block_tables,
                       int32_t max_blocks_per_seq, int n, int s, int h, int H, int D, int B,
                       int dtype, float scale, int partition_size)
{
    if (n <= 0) {
        for (int d = 0; d < D; ++d)
            o[d] = 0.0;
        return;
    }
    const int32_t *row = block_tables + (int64_t)s * max_blocks_per_seq;
    double *qd = (double *)malloc(sizeof(double) * (size_t)D);
    for (int d = 0; d < D; ++d)
        qd[d] = load_elem(q, (qrow * H + h) * D + d, dtype);
    double *Kc = (double *)malloc(sizeof(double) * (size_t)n * D);
    double *Vc = (double *)malloc(sizeof(double) * (size_t)n * D);
    gather_kv(Kc, Vc, k_cache, v_cache, row, 0, n, h, H, D, B, dtype);
    if (partition_size <= 0) {
        attend(o, NULL, NULL, qd, Kc, Vc, n, D, (double)scale);
    } else {
        int P = (n + partition_size - 1) / partition_size;
        double *op = (double *)malloc(sizeof(double) * (size_t)P * D);
        double *mp = (double *)malloc(sizeof(double) * (size_t)P);
        double *lp = (double *)malloc(sizeof(double) * (size_t)P);
        double M = -INFINITY;
        for (int p = 0; p < P; ++p) {
            int t0 = p * partition_size;
            int t1 = t0 + partition_size < n ? t0 + partition_size : n;
            attend(op + (int64_t)p * D, mp + p, lp + p, qd, Kc + (int64_t)t0 * D,
                   Vc + (int64_t)t0 * D, t1 - t0, D, (double)scale);
            if (mp[p] > M)
                M = mp[p];
        }
        double denom = 0.0;
        for (int d = 0; d < D; ++d)
            o[d] = 0.0;
        for (int p = 0; p < P; ++p) {
            double w = exp(mp[p] - M) * lp[p];
            denom += w;
            for (int d = 0; d < D; ++d)
                o[d] += w * op[(int64_t)p * D + d];
        }
        for (int d = 0; d < D; ++d)
            o[d] /= denom;
        free(op);
        free(mp);
        free(lp);
    }
    free(qd);
    free(Kc);
    free(Vc);
}

/*
 * out[r][D] (fp64) for the (sequence, head) pairs listed in rows[r][2]; with
 * rows == NULL, num_rows must be S*H and row r is (r / H, r % H).
 * partition_size <= 0: plain definition; > 0: split-context definition.
 * threads <= 0: all cores OpenMP offers.  Returns the thread count used.
 */
int pa_oracle_decode(double *out, const void *q, const void *k_cache, const void *v_cache,
                     const int32_t *block_tables, int32_t max_blocks_per_seq,
                     const int32_t *context_lens, int32_t num_seqs, int32_t num_heads,
                     int32_t head_dim, int32_t block_size, int32_t dtype, float scale,
                     int32_t partition_size, const int32_t *rows, int64_t num_rows, int32_t threads)
{
    int used = 1;
    (void)num_seqs;
#ifdef _OPENMP
    if (threads <= 0)
        threads = omp_get_max_threads();
    used = threads;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
#endif
    for (int64_t r = 0; r < num_rows; ++r) {
        int s = rows ? rows[2 * r] : (int)(r / num_heads);
        int h = rows ? rows[2 * r + 1] : (int)(r % num_heads);
        decode_row(out + r * head_dim, q, s, k_cache, v_cache, block_tables, max_blocks_per_seq,
                   context_lens[s], s, h, num_heads, head_dim, block_size, dtype, scale,
                   partition_size);
    }
    return used;
}

/*
 * Several query tokens per sequence: the prompt phase restricted to the part of
 * a prompt that follows an already cached prefix (Sec. 4.4, shared prefix).
 * Sequence s has q_len = q_start[s+1] - q_start[s] query rows, its last q_len
 * tokens; the query at position i (0-based in the whole sequence) attends to
 * positions 0..i, which is Eq. "attention-layer" of Sec. 2.1 with its own i.
 * out is [q_start[S]][H][D] in fp64.
 */
int pa_oracle_decode_multi(double *out, const void *q, const void *k_cache, const void *v_cache,
                           const int32_t *block_tables, int32_t max_blocks_per_seq,
                           const int32_t *context_lens, const int32_t *q_start, int32_t num_seqs,
                           int32_t num_heads, int32_t head_dim, int32_t block_size, int32_t dtype,
                           float scale, int32_t threads)
{
    int used = 1;
    int64_t total = (int64_t)q_start[num_seqs] * num_heads;
#ifdef _OPENMP
    if (threads <= 0)
        threads = omp_get_max_threads();
    used = threads;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
#endif
    for (int64_t r = 0; r < total; ++r) {
        int64_t row = r / num_heads;
        int h = (int)(r % num_heads);
        int s = 0;
        while (q_start[s + 1] <= row)
            ++s;
        int q_len = q_start[s + 1] - q_start[s];
        int pos = context_lens[s] - q_len + (int)(row - q_start[s]);   /* the query's own position */
        decode_row(out + r * head_dim, q, row, k_cache, v_cache, block_tables, max_blocks_per_seq,
                   pos + 1, s, h, num_heads, head_dim, block_size, dtype, scale, 0);
    }
    return used;
}

/*
 * For each token t in order with slot = slot_mapping[t] >= 0: copy the bit
 * patterns of k[t][h][:] and v[t][h][:] to block slot / B, offset slot % B.
 */
void pa_oracle_reshape_and_cache(const void *k, const void *v, void *k_cache, void *v_cache,
                                 const int64_t *slot_mapping, int32_t num_tokens,
                                 int32_t num_heads, int32_t head_dim, int32_t block_size,
                                 int32_t dtype)
{
    int E = elem_bytes(dtype);
    for (int t = 0; t < num_tokens; ++t) {
        int64_t slot = slot_mapping[t];
        if (slot < 0)
            continue;
        int64_t pb = slot / block_size;
        int off = (int)(slot % block_size);
        for (int h = 0; h < num_heads; ++h) {
            int64_t src = ((int64_t)t * num_heads + h) * head_dim;
            int64_t dst = cache_index(pb, h, off, 0, num_heads, block_size, head_dim);
            memcpy((char *)k_cache + dst * E, (const char *)k + src * E, (size_t)head_dim * E);
            memcpy((char *)v_cache + dst * E, (const char *)v + src * E, (size_t)head_dim * E);
        }
    }
}

/*
 * For each layer and each pair (src, dst) in order: copy the whole physical
 * block (all heads, all B slots, filled or not) in the K and the V cache.
 */
void pa_oracle_copy_blocks(void *const *k_caches, void *const *v_caches, int32_t num_layers,
                           const int64_t *src_dst_pairs, int32_t num_pairs, int32_t num_heads,
                           int32_t head_dim, int32_t block_size, int32_t dtype)
{
    size_t block_bytes = (size_t)num_heads * block_size * head_dim * elem_bytes(dtype);
    for (int l = 0; l < num_layers; ++l) {
        for (int i = 0; i < num_pairs; ++i) {
            int64_t src = src_dst_pairs[2 * i], dst = src_dst_pairs[2 * i + 1];
            memmove((char *)k_caches[l] + dst * block_bytes,
                    (const char *)k_caches[l] + src * block_bytes, block_bytes);
            memmove((char *)v_caches[l] + dst * block_bytes,
                    (const char *)v_caches[l] + src * block_bytes, block_bytes);
        }
    }
}

/*
 * Swapping (Sec. 4.5): evicted blocks are copied to another pool (CPU memory)
 * and later copied back.  For each layer and each pair (src, dst) in order:
 * the whole block src of the source pool is copied to block dst of the
 * destination pool, for K and for V.
 */
void pa_oracle_swap_blocks(void *const *src_k, void *const *src_v, void *const *dst_k,
                           void *const *dst_v, int32_t num_layers, const int64_t *src_dst_pairs,
                           int32_t num_pairs, int32_t num_heads, int32_t head_dim,
                           int32_t block_size, int32_t dtype)
{
    size_t block_bytes = (size_t)num_heads * block_size * head_dim * elem_bytes(dtype);
    for (int l = 0; l < num_layers; ++l) {
        for (int i = 0; i < num_pairs; ++i) {
            int64_t src = src_dst_pairs[2 * i], dst = src_dst_pairs[2 * i + 1];
            memcpy((char *)dst_k[l] + dst * block_bytes, (const char *)src_k[l] + src * block_bytes,
                   block_bytes);
            memcpy((char *)dst_v[l] + dst * block_bytes, (const char *)src_v[l] + src * block_bytes,
                   block_bytes);
        }
    }
}

int pa_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
