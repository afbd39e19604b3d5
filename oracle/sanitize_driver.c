/*
 * Sanitizer driver for the CPU oracle (test infrastructure only).
 *
 * Builds one tiny seeded paged workload in exactly-sized heap arrays and calls
 * every entry point of pa_oracle.c once, so that a build with
 * -fsanitize=address,undefined reports any out-of-bounds index, misaligned
 * access or undefined arithmetic in the oracle's own code.  Prints a checksum
 * of the fp64 outputs and "ok"; the test only needs the clean exit.
 *
 * Layout and calls follow the oracle's own header comments: caches are
 * [NB][H][B][D] (Sec. 4.1/4.2 of arxiv 2309.06180: fixed-size blocks reached
 * through a per-sequence block table).
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int pa_oracle_decode(double *out, const void *q, const void *k_cache, const void *v_cache,
                     const int32_t *block_tables, int32_t max_blocks_per_seq,
                     const int32_t *context_lens, int32_t num_seqs, int32_t num_heads,
                     int32_t head_dim, int32_t block_size, int32_t dtype, float scale,
                     int32_t partition_size, const int32_t *rows, int64_t num_rows, int32_t threads);
int pa_oracle_decode_multi(double *out, const void *q, const void *k_cache, const void *v_cache,
                           const int32_t *block_tables, int32_t max_blocks_per_seq,
                           const int32_t *context_lens, const int32_t *q_start, int32_t num_seqs,
                           int32_t num_heads, int32_t head_dim, int32_t block_size, int32_t dtype,
                           float scale, int32_t threads);
void pa_oracle_reshape_and_cache(const void *k, const void *v, void *k_cache, void *v_cache,
                                 const int64_t *slot_mapping, int32_t num_tokens,
                                 int32_t num_heads, int32_t head_dim, int32_t block_size,
                                 int32_t dtype);
void pa_oracle_copy_blocks(void *const *k_caches, void *const *v_caches, int32_t num_layers,
                           const int64_t *src_dst_pairs, int32_t num_pairs, int32_t num_heads,
                           int32_t head_dim, int32_t block_size, int32_t dtype);
void pa_oracle_swap_blocks(void *const *src_k, void *const *src_v, void *const *dst_k,
                           void *const *dst_v, int32_t num_layers, const int64_t *src_dst_pairs,
                           int32_t num_pairs, int32_t num_heads, int32_t head_dim,
                           int32_t block_size, int32_t dtype);

static uint32_t rng_state = 12345u;
static uint32_t next_u32(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return rng_state >> 8;
}

/* a small finite value in the storage type `dtype` (0 f32, 1 f16, 2 bf16) */
static void put_value(void *base, size_t i, int dtype)
{
    int v = (int)(next_u32() % 17u) - 8;              /* -8 .. 8, exact in every type */
    if (dtype == 0) {
        ((float *)base)[i] = (float)v * 0.25f;
    } else if (dtype == 2) {
        float f = (float)v * 0.25f;
        uint32_t u;
        memcpy(&u, &f, 4);
        ((uint16_t *)base)[i] = (uint16_t)(u >> 16);  /* few mantissa bits: exact */
    } else {
        /* fp16 bit pattern of v/4 for |v| <= 8, built by hand */
        static const uint16_t mag[9] = {0x0000, 0x3400, 0x3800, 0x3A00, 0x3C00, 0x3D00, 0x3E00, 0x3F00, 0x4000};
        uint16_t h = mag[v < 0 ? -v : v];
        ((uint16_t *)base)[i] = (uint16_t)(h | (v < 0 ? 0x8000u : 0u));
    }
}

static double run(int dtype)
{
    enum { S = 3, H = 2, D = 8, B = 4, NB = 12, MB = 4, L = 2, T = 3 };
    const int E = dtype == 0 ? 4 : 2;
    const int32_t lens[S] = {13, 1, 6};              /* 4, 1 and 2 blocks: 7 of the 12 blocks in use */
    const int32_t tables[S][MB] = {{7, 1, 3, 10}, {5, -1, -1, -1}, {0, 9, -1, 99}};
    const size_t cache_elems = (size_t)NB * H * B * D;
    void *kc[L], *vc[L], *kh[L], *vh[L];
    for (int l = 0; l < L; ++l) {
        kc[l] = malloc(cache_elems * E);
        vc[l] = malloc(cache_elems * E);
        kh[l] = malloc(cache_elems * E);
        vh[l] = malloc(cache_elems * E);
        for (size_t i = 0; i < cache_elems; ++i) {
            put_value(kc[l], i, dtype);
            put_value(vc[l], i, dtype);
        }
        memset(kh[l], 0, cache_elems * E);
        memset(vh[l], 0, cache_elems * E);
    }
    int32_t *bt = malloc(sizeof(tables));
    memcpy(bt, tables, sizeof(tables));
    int32_t *cl = malloc(sizeof(lens));
    memcpy(cl, lens, sizeof(lens));

    /* copy-on-write pair list with a fan-out, then new tokens into the last slots in use */
    int64_t *pairs = malloc(2 * 2 * sizeof(int64_t));
    pairs[0] = 3; pairs[1] = 2; pairs[2] = 3; pairs[3] = 4;
    pa_oracle_copy_blocks(kc, vc, L, pairs, 2, H, D, B, dtype);

    void *kn = malloc((size_t)T * H * D * E), *vn = malloc((size_t)T * H * D * E);
    for (size_t i = 0; i < (size_t)T * H * D; ++i) {
        put_value(kn, i, dtype);
        put_value(vn, i, dtype);
    }
    int64_t *slots = malloc(T * sizeof(int64_t));
    slots[0] = 10 * B + 0;   /* token 12 of sequence 0: block 10, offset 0 */
    slots[1] = -1;           /* padding */
    slots[2] = 9 * B + 1;    /* token 5 of sequence 2: block 9, offset 1 */
    pa_oracle_reshape_and_cache(kn, vn, kc[0], vc[0], slots, T, H, D, B, dtype);

    /* swap two blocks out to the other pool and one back */
    int64_t *sw = malloc(2 * 2 * sizeof(int64_t));
    sw[0] = 7; sw[1] = 0; sw[2] = 11; sw[3] = 11;
    pa_oracle_swap_blocks(kc, vc, kh, vh, L, sw, 2, H, D, B, dtype);
    sw[0] = 0; sw[1] = 6;
    pa_oracle_swap_blocks(kh, vh, kc, vc, L, sw, 1, H, D, B, dtype);

    void *q = malloc((size_t)S * H * D * E);
    for (size_t i = 0; i < (size_t)S * H * D; ++i)
        put_value(q, i, dtype);
    double *out = malloc((size_t)S * H * D * sizeof(double));
    double sum = 0.0;
    for (int ps = 0; ps <= 8; ps += 4) {             /* plain definition, then 4- and 8-token ranges */
        pa_oracle_decode(out, q, kc[0], vc[0], bt, MB, cl, S, H, D, B, dtype, 0.35f, ps, NULL,
                         (int64_t)S * H, 1);
        for (int i = 0; i < S * H * D; ++i)
            sum += out[i];
    }
    int32_t rows[2][2] = {{2, 1}, {0, 0}};
    int32_t *rw = malloc(sizeof(rows));
    memcpy(rw, rows, sizeof(rows));
    pa_oracle_decode(out, q, kc[0], vc[0], bt, MB, cl, S, H, D, B, dtype, 0.35f, 0, rw, 2, 2);
    sum += out[0] + out[2 * D - 1];

    /* several queries per sequence: 3, 1 and 2 of the last tokens */
    const int32_t qs[S + 1] = {0, 3, 4, 6};
    int32_t *q_start = malloc(sizeof(qs));
    memcpy(q_start, qs, sizeof(qs));
    void *qm = malloc((size_t)6 * H * D * E);
    for (size_t i = 0; i < (size_t)6 * H * D; ++i)
        put_value(qm, i, dtype);
    double *outm = malloc((size_t)6 * H * D * sizeof(double));
    pa_oracle_decode_multi(outm, qm, kc[0], vc[0], bt, MB, cl, q_start, S, H, D, B, dtype, 0.35f, 1);
    for (int i = 0; i < 6 * H * D; ++i)
        sum += outm[i];

    for (int l = 0; l < L; ++l) {
        free(kc[l]); free(vc[l]); free(kh[l]); free(vh[l]);
    }
    free(bt); free(cl); free(pairs); free(kn); free(vn); free(slots); free(sw); free(q); free(out);
    free(rw); free(q_start); free(qm); free(outm);
    return sum;
}

int main(void)
{
    double total = 0.0;
    for (int dtype = 0; dtype < 3; ++dtype)
        total += run(dtype);
    if (total != total) {
        printf("checksum is NaN\n");
        return 1;
    }
    printf("checksum %.12f\nok\n", total);
    return 0;
}
