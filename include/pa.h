/*
 * pa.h - C ABI of libpa: paged single-query attention for AMD MI355X (gfx950).
 *
 * The library implements the decode-step hot path of PagedAttention
 * (arxiv 2309.06180): attention of one query token per sequence over a KV
 * cache kept in fixed-size physical blocks that each sequence reaches through
 * a block table (Sec. 4.1, 4.2), the store of new K/V vectors into those
 * blocks (Sec. 4.3, 5.1 (1)) and the batched copy-on-write block copy
 * (Sec. 4.4, 5.1 (3)).
 *
 * Conventions shared by all calls
 * -------------------------------
 * Shapes: S sequences, H heads, D head dimension, B tokens per block, NB
 * physical blocks in the pool, T new tokens, MB block-table row stride.
 *
 * Cache layout: a K (or V) cache of one layer is an array [NB][H][B][D] of
 * `dtype` elements; element (block pb, head h, offset off, dim d) is at index
 * ((pb*H + h)*B + off)*D + d.  K and V use the same layout.  Token t of a
 * sequence lives in the sequence's logical block t / B at offset t % B; its
 * slot number is physical_block*B + offset.
 *
 * Memory: every data pointer is DEVICE memory owned by the caller, 16-byte
 * aligned, unless a parameter says "host".  The library allocates and frees
 * nothing the caller can see, never synchronises, and enqueues all work on
 * `stream` (a hipStream_t passed as void*; NULL is the default stream).
 *
 * Errors: host-checkable conditions are reported synchronously through
 * pa_status and nothing is launched.  Contents of index arrays live on the
 * device and are NOT checked by the compute calls: a block id outside
 * [0, NB), a context length above max_context_len or above MB*B, a slot at or
 * above NB*B, duplicate slots, or a copy destination that is also a source or
 * appears twice are undefined behaviour.  pa_debug_validate checks them.
 *
 * Supported: dtype f16/bf16/f32; head_dim D in {64, 128}; block_size B in
 * {8, 16, 32, 64, 128}; multi-head attention with as many KV heads as query
 * heads (the paper's models).  pa_decode_multi: f16/bf16, D = 128, B >= 16.
 */
#ifndef PA_H
#define PA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PA_OK = 0,
    PA_ERR_NULL = 1,        /* a required pointer is NULL                         */
    PA_ERR_SHAPE = 2,       /* a size is negative, zero where it may not be, or inconsistent */
    PA_ERR_UNSUPPORTED = 3, /* (dtype, head_dim, block_size) outside the supported set */
    PA_ERR_ALIGN = 4,       /* a data pointer is not 16-byte aligned              */
    PA_ERR_WORKSPACE = 5,   /* workspace missing or too small                     */
    PA_ERR_HIP = 6,         /* the HIP runtime refused a launch or a copy         */
    PA_ERR_INVALID = 7,     /* pa_debug_validate found a bad index                */
    PA_ERR_LIMIT = 8        /* pa_decode_static: the shape needs more than PA_STATIC_SCRATCH_BYTES */
} pa_status;

typedef enum { PA_F32 = 0, PA_F16 = 1, PA_BF16 = 2 } pa_dtype;

/* partition_size value that lets the library choose the split (needs a workspace). */
#define PA_PARTITION_AUTO (-1)

/*
 * pa_decode - single-query attention over the paged cache.
 *
 * For every sequence s and head h, with n = context_lens[s]:
 *     x_t   = scale * sum_d q[s][h][d] * K[t][h][d]              t = 0..n-1
 *     out[s][h][:] = sum_t softmax(x)_t * V[t][h][:]
 * where K[t], V[t] are read from physical block block_tables[s][t / B] at
 * offset t % B.  This is Eq. (4) of Sec. 4.1, equal to the per-token attention
 * of Sec. 2.1; the query token is token n-1, so its K/V must already be in
 * the cache (call pa_reshape_and_cache first, Sec. 4.3).  Arithmetic is fp32;
 * the result is rounded to `dtype` once (nearest even).  n = 0 gives a zero
 * row.  Table entries at or beyond ceil(n / B) and cache slots at or beyond n
 * are never used (they may hold anything, NaN included).
 *
 *   out              [S][H][D] dtype, written
 *   q                [S][H][D] dtype
 *   k_cache, v_cache [NB][H][B][D] dtype
 *   block_tables     [S][max_blocks_per_seq] int32
 *   context_lens     [S] int32, each <= max_context_len <= max_blocks_per_seq*B
 *   max_context_len  host-known upper bound on context_lens[]
 *   partition_size   0: one pass per (sequence, head).
 *                    > 0, multiple of B: split-context - every (sequence, head)
 *                    is cut into ranges of partition_size tokens processed
 *                    independently (max logit, exp-sum and unnormalised partial
 *                    sums kept in fp32 in the workspace), then a second
 *                    kernel merges them with the log-sum-exp rule.
 *                    PA_PARTITION_AUTO: the library picks a partition size
 *                    from the shape; falls back to one pass when workspace is
 *                    NULL.
 *   workspace        device scratch of at least pa_decode_workspace_bytes(...)
 *                    bytes when a split is used; contents undefined after.
 *
 * Returns PA_OK without launching when S == 0.
 */
pa_status pa_decode(void *out, const void *q, const void *k_cache, const void *v_cache,
                    const int32_t *block_tables, int32_t max_blocks_per_seq,
                    const int32_t *context_lens, int32_t num_seqs, int32_t num_heads,
                    int32_t head_dim, int32_t block_size, int64_t num_blocks, pa_dtype dtype,
                    float scale, int32_t max_context_len, int32_t partition_size,
                    void *workspace, size_t workspace_bytes, void *stream);

/* Bytes of workspace pa_decode needs for this shape and partition_size (0 for one pass). */
size_t pa_decode_workspace_bytes(int32_t num_seqs, int32_t num_heads, int32_t head_dim,
                                 int32_t block_size, int32_t max_context_len,
                                 int32_t partition_size);

/*
 * pa_decode_static - pa_decode for callers that cannot allocate or pass device
 * scratch memory: code under HIP graph capture, tight serving loops, harnesses
 * that forbid allocation.  Same arguments and result as pa_decode without the
 * workspace: the split-context partials (max logit, exp-sum, partial sums) go
 * to an array of PA_STATIC_SCRATCH_BYTES bytes that is part of the library's
 * device image; each GPU the library runs on holds one until the process
 * ends.  The call allocates and frees nothing.  A (shape, partition_size) for
 * which pa_decode_workspace_bytes(...) exceeds PA_STATIC_SCRATCH_BYTES is
 * refused with PA_ERR_LIMIT and nothing is launched.  partition_size = 0 uses
 * no scratch at all.  All calls on one GPU share that GPU's array: calls that
 * may overlap on one GPU (different streams, different threads) race on it
 * and must be ordered by the caller.  Nothing in the array has to start at
 * zero and nothing is kept between calls.
 */
#define PA_STATIC_SCRATCH_BYTES (16u << 20)
pa_status pa_decode_static(void *out, const void *q, const void *k_cache, const void *v_cache,
                           const int32_t *block_tables, int32_t max_blocks_per_seq,
                           const int32_t *context_lens, int32_t num_seqs, int32_t num_heads,
                           int32_t head_dim, int32_t block_size, int64_t num_blocks, pa_dtype dtype,
                           float scale, int32_t max_context_len, int32_t partition_size,
                           void *stream);

/*
 * pa_decode_shared - pa_decode for batches whose sequences share physical
 * blocks (Sec. 4.4: samples of one prompt, beams of one search and requests
 * behind one prefix map their common logical blocks to the same physical
 * blocks).  Same arguments, same result as pa_decode; the difference is
 * traffic.  On the device, the library compares the block tables of
 * consecutive sequences and ties a sequence to its predecessor when the
 * leading full blocks they have in common are worth it: at least 32 tokens and
 * at least one eighth of the shorter of the two contexts.  Chains of tied
 * sequences are cut into groups of at most 16.  For every group it lists each
 * physical block that a member maps, once, with the set of members that map
 * it; one workgroup per (group, head) then applies every listed K/V tile to
 * the queries of all members that map it, on the matrix cores (the members
 * are the 16 query columns of the tiles), and writes the members' output
 * rows.  A block is therefore read from memory once per group instead of once
 * per reader.  Sequences outside any group go through pa_decode's one-pass
 * kernel in the same launch.
 *
 * When it pays: the decode launch reads the distinct bytes of a batch at about
 * 0.80 of the HBM peak (0.86 for pa_decode on batches without sharing), so it
 * wins as soon as a noticeable part of the logical bytes is shared: 1.2x at
 * the parallel-sampling configuration (a third shared), 1.9x with beams of
 * six, 3.4x when 256 requests share a 1024-token prefix.  With nothing shared
 * no group forms and the decode launch costs what pa_decode costs; the plan
 * adds 10-20 us per call, which pa_shared_plan / pa_decode_shared_planned
 * spread over the layers of a step.  A prefix of a few dozen tokens under
 * long private contexts is not worth a group by the rule above, and a short
 * prefix that every sequence shares (80 tokens) is served as fast out of the
 * caches by pa_decode.
 *
 * Callers should place sequences that were forked from one another next to
 * each other in the batch; any order is correct, only sharing between
 * neighbours is exploited.  `workspace` must hold
 * pa_decode_shared_workspace_bytes(...) bytes.  Two kernels are enqueued on
 * `stream`.  2-byte types at head_dim 128 with block_size >= 16 and at most
 * 16384 sequences; other shapes run pa_decode's one-pass kernel (same result,
 * no saving).
 */
pa_status pa_decode_shared(void *out, const void *q, const void *k_cache, const void *v_cache,
                           const int32_t *block_tables, int32_t max_blocks_per_seq,
                           const int32_t *context_lens, int32_t num_seqs, int32_t num_heads,
                           int32_t head_dim, int32_t block_size, int64_t num_blocks,
                           pa_dtype dtype, float scale, int32_t max_context_len, void *workspace,
                           size_t workspace_bytes, void *stream);

size_t pa_decode_shared_workspace_bytes(int32_t num_seqs, int32_t num_heads, int32_t head_dim,
                                        int32_t max_blocks_per_seq);

/*
 * pa_shared_plan / pa_decode_shared_planned - pa_decode_shared in two steps.
 * Every layer of a model uses the same block tables (Sec. 4.1, one table per
 * sequence for all layers), so the grouping and the tile lists need building
 * once per decoding step, not once per layer: pa_shared_plan enqueues the
 * planning kernel and leaves the plan in `workspace`
 * (pa_decode_shared_workspace_bytes(...) bytes, caller-owned);
 * pa_decode_shared_planned enqueues only the decode launch and reads the plan.
 * The plan is valid for exactly the block_tables, context_lens, num_seqs,
 * max_blocks_per_seq and block_size it was built from, for as long as the
 * caller leaves those arrays and the plan untouched; any change to them needs
 * a new plan (a stale plan gives wrong results or out-of-range reads, unchecked).
 * Plan and decode must be ordered on the device: same stream, or an event.
 * pa_decode_shared(...) is pa_shared_plan(...) followed by
 * pa_decode_shared_planned(...) on the same workspace.  For shapes that
 * pa_decode_shared passes to pa_decode, the plan is empty and never read.
 *
 * Layout of a plan, for inspection (S = num_seqs, MB = max_blocks_per_seq;
 * int32 words): six arrays of S words - in_group[s] (1 if s belongs to a
 * group), group_size[s] (members of the group that starts at s, else 0),
 * tile_count[s] (entries on that group's tile list; defined only where a group
 * starts), adj[s] (leading full blocks s shares with s-1), single_list[]
 * (sequences outside any group, ascending), group_list[] (first sequences of
 * the groups, ascending) - then group_count and single_count at words 6S and
 * 6S+1; from the next multiple of four words at or after 6S+4, S work items of
 * four words (kind: 2 group / 1 single sequence / 0 nothing, first sequence,
 * members, tile-list entries): groups first, then singles, then nothing.  At
 * the next 16-byte boundary the tile array begins: S*MB entries of four words;
 * the list of the group that starts at s begins at entry s*MB and holds
 * (physical block, member set in bits 0..15 | "some member sees only part of
 * it" in bit 16, logical block index, tokens seen by the longest member of the
 * set), ordered by logical block index.
 */
pa_status pa_shared_plan(const int32_t *block_tables, int32_t max_blocks_per_seq,
                         const int32_t *context_lens, int32_t num_seqs, int32_t num_heads,
                         int32_t head_dim, int32_t block_size, int64_t num_blocks, pa_dtype dtype,
                         int32_t max_context_len, void *workspace, size_t workspace_bytes,
                         void *stream);

pa_status pa_decode_shared_planned(void *out, const void *q, const void *k_cache,
                                   const void *v_cache, const int32_t *block_tables,
                                   int32_t max_blocks_per_seq, const int32_t *context_lens,
                                   int32_t num_seqs, int32_t num_heads, int32_t head_dim,
                                   int32_t block_size, int64_t num_blocks, pa_dtype dtype,
                                   float scale, int32_t max_context_len, const void *plan,
                                   size_t plan_bytes, void *stream);

/*
 * pa_decode_multi - several query tokens per sequence over the paged cache:
 * the case where only the tail of a prompt has to be computed because its
 * prefix is already cached (Sec. 4.4, "Shared prefix"), or a few draft tokens
 * to be checked at once.  Sequence s contributes q_len_s = q_start[s+1] -
 * q_start[s] query rows, the last q_len_s tokens of its context (their K/V
 * must already be in the cache, as for pa_decode).  Query i of them, at
 * position n_s - q_len_s + i, attends to tokens 0 .. n_s - q_len_s + i
 * (causal), by the same formula as pa_decode; q_len_s = 1 is pa_decode.
 * Runs on the matrix cores.  With max_q_len <= 16 one workgroup per (sequence,
 * head) serves all of a sequence's queries and K/V is read once; beyond that
 * one workgroup serves 64 queries (max_q_len <= 64) or 128, and K/V is read
 * once per workgroup (from the caches, mostly, after the first time).
 *
 *   out, q        [q_start[S]][H][D] dtype, rows of sequence s at q_start[s] ..
 *   q_start       device [S+1] int32, non-decreasing, q_start[0] = 0
 *   max_q_len     host-known upper bound on q_len_s; q_len_s <= context_lens[s]
 * Supported: f16 / bf16, head_dim 128, block_size a multiple of 16.
 */
pa_status pa_decode_multi(void *out, const void *q, const void *k_cache, const void *v_cache,
                          const int32_t *block_tables, int32_t max_blocks_per_seq,
                          const int32_t *context_lens, const int32_t *q_start, int32_t num_seqs,
                          int32_t max_q_len, int32_t num_heads, int32_t head_dim,
                          int32_t block_size, int64_t num_blocks, pa_dtype dtype, float scale,
                          int32_t max_context_len, void *stream);

/*
 * pa_reshape_and_cache - store new K/V vectors into the paged cache
 * (Sec. 4.3: the KV of the tokens of this iteration is saved into the
 * physical blocks; Sec. 5.1 (1): reshape and block write fused in one launch).
 *
 * For every token t with slot = slot_mapping[t] >= 0 and every head h:
 *     k_cache[slot / B][h][slot % B][:] = k[t][h][:]     (same for v)
 * Bit patterns are copied unchanged.  Negative slots are skipped.
 *
 *   k, v          [T][H][D] dtype
 *   slot_mapping  [T] int64
 * Returns PA_OK without launching when T == 0.
 */
pa_status pa_reshape_and_cache(const void *k, const void *v, void *k_cache, void *v_cache,
                               const int64_t *slot_mapping, int32_t num_tokens,
                               int32_t num_heads, int32_t head_dim, int32_t block_size,
                               int64_t num_blocks, pa_dtype dtype, void *stream);

/*
 * pa_copy_blocks - copy-on-write block copies, all pairs and all layers in
 * one launch (Sec. 4.4: a shared block that is about to be written is copied
 * to a fresh block; Sec. 5.1 (3): the copies are batched into one kernel).
 *
 * For every layer l and pair i: k_caches[l][dst_i] = k_caches[l][src_i] and the
 * same for v - the whole block, all heads, all B slots.
 *
 *   k_caches, v_caches  HOST arrays of num_layers device pointers, each a
 *                       [NB][H][B][D] cache; read during the call only
 *   src_dst_pairs       device [num_pairs][2] int64, (src, dst) block ids
 * Returns PA_OK without launching when num_pairs == 0.
 */
pa_status pa_copy_blocks(void *const *k_caches, void *const *v_caches, int32_t num_layers,
                         const int64_t *src_dst_pairs, int32_t num_pairs, int32_t num_heads,
                         int32_t head_dim, int32_t block_size, int64_t num_blocks,
                         pa_dtype dtype, void *stream);

/*
 * pa_swap_blocks - block copies between two sets of caches in one launch:
 * swapping evicted blocks out to CPU memory and back (Sec. 4.5, "Swapping":
 * evicted blocks are copied to CPU RAM, managed by a CPU block allocator, and
 * brought back when the sequence is rescheduled).  For every layer l and pair
 * i: dst_k_caches[l][dst_i] = src_k_caches[l][src_i], and the same for v.
 *
 * Either side may be device memory or PINNED host memory that the device can
 * address (hipHostMalloc / a torch tensor with pin_memory=True): the kernel
 * reads and writes it directly, so one launch moves all blocks of all layers
 * instead of one small transfer per block.  The caller synchronises `stream`
 * before the CPU touches host-side blocks.
 *
 *   src_*_caches, dst_*_caches  HOST arrays of num_layers pointers to
 *                       [src_num_blocks][H][B][D] / [dst_num_blocks][H][B][D] caches
 *   src_dst_pairs       device [num_pairs][2] int64: (block id in src, block id in dst);
 *                       destinations are distinct
 */
pa_status pa_swap_blocks(void *const *src_k_caches, void *const *src_v_caches,
                         void *const *dst_k_caches, void *const *dst_v_caches, int32_t num_layers,
                         const int64_t *src_dst_pairs, int32_t num_pairs, int32_t num_heads,
                         int32_t head_dim, int32_t block_size, int64_t src_num_blocks,
                         int64_t dst_num_blocks, pa_dtype dtype, void *stream);

/*
 * pa_debug_validate - check the device index arrays of a decode step against
 * the undefined-behaviour list above.  Copies them to the host, synchronises
 * the stream, and returns PA_ERR_INVALID on the first violation.  Any of
 * block_tables/context_lens, slot_mapping, src_dst_pairs may be NULL to skip
 * that check.  For tests and bring-up, not for the serving loop.
 */
pa_status pa_debug_validate(const int32_t *block_tables, int32_t max_blocks_per_seq,
                            const int32_t *context_lens, int32_t num_seqs,
                            int32_t max_context_len, const int64_t *slot_mapping,
                            int32_t num_tokens, const int64_t *src_dst_pairs, int32_t num_pairs,
                            int32_t block_size, int64_t num_blocks, void *stream);

/*
 * pa_stream_read - bandwidth probe: reads `bytes` bytes (multiple of 16) at
 * `src` once with non-temporal 16-byte loads, one contiguous 256 KiB tile per
 * workgroup, and (practically) never writes; `sink` must hold at least
 * 4*65536 bytes.  Gives the streaming-read ceiling of the device that roofline
 * fractions are put beside.
 */
pa_status pa_stream_read(const void *src, size_t bytes, void *sink, void *stream);

const char *pa_status_string(pa_status status);
int pa_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PA_H */
