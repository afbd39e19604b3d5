// libpa - paged single-query attention for gfx950 (MI355X).
//
// Three operations of PagedAttention's decode step (arxiv 2309.06180):
//   pa_decode            Sec. 4.1, Eq. (4): attention of one query per sequence
//                        over K/V blocks reached through a block table
//   pa_reshape_and_cache Sec. 4.3 / 5.1 (1): store new K/V vectors at their slots
//   pa_copy_blocks       Sec. 4.4 / 5.1 (3): batched copy-on-write block copies
//
// Cache layout [NB][H][B][D]: the K (or V) vectors of one (block, head) are
// B*D*E contiguous bytes, a token row is D*E bytes.  Every wavefront load is
// 64 lanes x 16 bytes = 1 KiB of consecutive addresses.
//
// The decode path is a batch of matrix-vector products (one flop per byte of
// KV at 2-byte elements), bound by HBM bandwidth, so there is no MFMA here:
// the design goal is bytes in flight per compute unit and few VALU
// instructions per byte.
#include <hip/hip_runtime.h>

#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <type_traits>

#include "pa.h"

namespace {

constexpr int kWave = 64;
#ifndef PA_CHUNKS_PER_TRIP
#define PA_CHUNKS_PER_TRIP 2
#endif
// chunks requested together per trip of the steady-state loop
constexpr int kChunksPerTrip = PA_CHUNKS_PER_TRIP;
constexpr int kChunksPerTripDevice = PA_CHUNKS_PER_TRIP;
constexpr int kGroupMax = 4;       // query slots of the VALU shared-prefix kernel
constexpr int kGroupMaxMfma = 8;   // query slots used of the 16 rows of the MFMA shared-prefix kernel
constexpr float kLog2e = 1.4426950408889634f;
// running-maximum start value: finite, so that (m - m) is 0 and never NaN
constexpr float kNegBig = -3.0e38f;

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float as_f32(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __builtin_bit_cast(uint32_t, f); }

// ---- cross-lane sums ------------------------------------------------------
// DPP controls: quad_perm [1,0,3,2] = 0xB1, quad_perm [2,3,0,1] = 0x4E,
// row_half_mirror = 0x141, row_mirror = 0x140.  Applied in this order they
// form a butterfly over 4, 8 and 16 consecutive lanes; every lane ends with
// the same bits because each step adds the same two partial sums.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x)
{
    int y = __builtin_amdgcn_update_dpp(0, (int)as_u32(x), CTRL, 0xf, 0xf, true);
    return x + as_f32((uint32_t)y);
}

template <int LANES>
__device__ __forceinline__ float group_sum(float x)
{
    static_assert(LANES == 8 || LANES == 16 || LANES == 32, "lanes per token row");
    x = dpp_add<0xB1>(x);
    x = dpp_add<0x4E>(x);
    x = dpp_add<0x141>(x);
    if (LANES >= 16) x = dpp_add<0x140>(x);
    if (LANES >= 32) x += __shfl_xor(x, 16);
    return x;
}

// ---- element types -------------------------------------------------------
// A lane always holds one 16-byte fragment of a token row: 8 two-byte
// elements or 4 floats.
template <int DT> struct Traits;

template <> struct Traits<PA_F32> {
    static constexpr int E = 4, EPL = 4;
    static constexpr bool FENCE_AXPY = false;
    static __device__ __forceinline__ float dot(const uint4 &k, const uint4 &q, float acc)
    {
        acc = __builtin_fmaf(as_f32(k.x), as_f32(q.x), acc);
        acc = __builtin_fmaf(as_f32(k.y), as_f32(q.y), acc);
        acc = __builtin_fmaf(as_f32(k.z), as_f32(q.z), acc);
        acc = __builtin_fmaf(as_f32(k.w), as_f32(q.w), acc);
        return acc;
    }
    static __device__ __forceinline__ void axpy(float (&acc)[4], float p, const uint4 &v)
    {
        acc[0] = __builtin_fmaf(p, as_f32(v.x), acc[0]);
        acc[1] = __builtin_fmaf(p, as_f32(v.y), acc[1]);
        acc[2] = __builtin_fmaf(p, as_f32(v.z), acc[2]);
        acc[3] = __builtin_fmaf(p, as_f32(v.w), acc[3]);
    }
    static __device__ __forceinline__ uint4 pack(const float (&x)[4])
    {
        return make_uint4(as_u32(x[0]), as_u32(x[1]), as_u32(x[2]), as_u32(x[3]));
    }
};

template <> struct Traits<PA_F16> {
    static constexpr int E = 2, EPL = 8;
    static constexpr bool FENCE_AXPY = false;
    static __device__ __forceinline__ float dot(const uint4 &k, const uint4 &q, float acc)
    {
        // products of two halves are exact in fp32; accumulation is fp32
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, k.x), __builtin_bit_cast(half2_t, q.x), acc, false);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, k.y), __builtin_bit_cast(half2_t, q.y), acc, false);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, k.z), __builtin_bit_cast(half2_t, q.z), acc, false);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, k.w), __builtin_bit_cast(half2_t, q.w), acc, false);
        return acc;
    }
    static __device__ __forceinline__ void axpy2(float &a0, float &a1, float p, uint32_t v)
    {
        half2_t h = __builtin_bit_cast(half2_t, v);
        a0 = __builtin_fmaf(p, (float)h.x, a0);
        a1 = __builtin_fmaf(p, (float)h.y, a1);
    }
    static __device__ __forceinline__ void axpy(float (&acc)[8], float p, const uint4 &v)
    {
        axpy2(acc[0], acc[1], p, v.x);
        axpy2(acc[2], acc[3], p, v.y);
        axpy2(acc[4], acc[5], p, v.z);
        axpy2(acc[6], acc[7], p, v.w);
    }
    static __device__ __forceinline__ uint32_t pack2(float a, float b)
    {
        half2_t h;
        h.x = (_Float16)a;   // round to nearest even
        h.y = (_Float16)b;
        return __builtin_bit_cast(uint32_t, h);
    }
    static __device__ __forceinline__ uint4 pack(const float (&x)[8])
    {
        return make_uint4(pack2(x[0], x[1]), pack2(x[2], x[3]), pack2(x[4], x[5]), pack2(x[6], x[7]));
    }
};

template <> struct Traits<PA_BF16> {
    static constexpr int E = 2, EPL = 8;
    static constexpr bool FENCE_AXPY = true;
    static __device__ __forceinline__ float dot(const uint4 &k, const uint4 &q, float acc)
    {
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.x), __builtin_bit_cast(bf16x2_t, q.x), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.y), __builtin_bit_cast(bf16x2_t, q.y), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.z), __builtin_bit_cast(bf16x2_t, q.z), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.w), __builtin_bit_cast(bf16x2_t, q.w), acc, false);
        return acc;
    }
    static __device__ __forceinline__ void axpy2(float &a0, float &a1, float p, uint32_t v)
    {
        // a bfloat16 is the upper half of a float
        a0 = __builtin_fmaf(p, as_f32(v << 16), a0);
        a1 = __builtin_fmaf(p, as_f32(v & 0xffff0000u), a1);
    }
    static __device__ __forceinline__ void axpy(float (&acc)[8], float p, const uint4 &v)
    {
        axpy2(acc[0], acc[1], p, v.x);
        axpy2(acc[2], acc[3], p, v.y);
        axpy2(acc[4], acc[5], p, v.z);
        axpy2(acc[6], acc[7], p, v.w);
    }
    static __device__ __forceinline__ uint32_t rne(float f)
    {
        uint32_t u = as_u32(f);
        if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;   // NaN stays NaN
        return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    }
    static __device__ __forceinline__ uint4 pack(const float (&x)[8])
    {
        return make_uint4(rne(x[0]) | (rne(x[1]) << 16), rne(x[2]) | (rne(x[3]) << 16),
                          rne(x[4]) | (rne(x[5]) << 16), rne(x[6]) | (rne(x[7]) << 16));
    }
};

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// 16-byte load with the non-temporal hint: K/V bytes are used exactly once per
// call, and streaming them past the caches measurably raises the HBM rate.
__device__ __forceinline__ uint4 load16_stream(const char *p)
{
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// Streaming copies: data that passes through once is loaded and stored with
// the non-temporal hint (measured 6.4 TB/s of read+write traffic for block
// copies against 5.7 TB/s with plain accesses).
__device__ __forceinline__ u32x4_t load_frag_stream(const uint4 *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
}
__device__ __forceinline__ void store_frag_stream(uint4 *p, u32x4_t v)
{
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t *>(p));
}

// ---- decode ----------------------------------------------------------------
// One workgroup of W wavefronts serves one work item: a (sequence, head) over
// its whole context, over one fixed-size partition of it, or over the suffix
// that follows a shared prefix; or a (group of sequences, head) over the
// prefix of physical blocks the group has in common.
//
// Lane roles: a token row is LPT = D*E/16 lanes wide, so one 1 KiB wavefront
// load covers TPL = 64/LPT consecutive tokens; lane = g*LPT + c holds
// dimensions [c*EPL, (c+1)*EPL) of token (base + g).  Work advances in chunks
// of LPC loads (CT = LPC*TPL tokens, at most one block); wave w takes chunks
// w, w+W, ...; U chunks (2*U*LPC KiB of K and V) are requested together
// before any of them is used.
//
// Each group g of lanes runs its own online softmax over the tokens it sees
// (running maximum m, sum l, weighted V sum acc, all fp32, exponents in base
// 2 with log2(e) folded into the scale).  Groups and waves are merged once at
// the end with the log-sum-exp rule, so the inner loop has no cross-group
// traffic.  Summation order depends only on logical token positions, so the
// result does not change with the physical placement of blocks.
//
// In the shared-prefix mode the workgroup holds the queries of up to G
// sequences and applies every K/V fragment it loads to all of them, so blocks
// that several sequences map (parallel sampling, beam search: Sec. 4.4) are
// read from memory once per group instead of once per sequence.
enum DecodeMode {
    MODE_SINGLE = 0,   // whole context, writes the output row
    MODE_PART = 1,     // tokens [part*PS, (part+1)*PS), writes partial `part` of max_parts
    MODE_SUFFIX = 2,   // tokens [range_begin[s], n), writes partial 1 of 2
    MODE_PREFIX = 3    // tokens [0, prefix) of a group, writes partial 0 of 2 for every member
};

struct DecodeParams {
    void *out;
    const void *q;
    const char *k_cache, *v_cache;
    const int32_t *block_tables;
    const int32_t *context_lens;
    const int32_t *ginfo;   // group table built by find_groups_kernel (shared-prefix path)
    const int32_t *q_start; // multi-query path: first query row of every sequence, [S+1]
    float *ws_acc, *ws_ml;
    int32_t max_blocks, S, H;
    int32_t partition_size, max_parts;
    int32_t prefix_blocks;   // fused shared-prefix launch: workgroups [0, prefix_blocks) are prefix items
    int32_t q_blocks;        // multi-query path: blocks of 16 queries per sequence in the grid
    float scale_log2;
};

// Layout of the group table, three arrays of S entries: range_begin[s] (tokens
// of s covered by its group's shared prefix), group_size[s] (members of the
// group that starts at sequence s, 0 if none starts there) and
// group_prefix_tokens[s] (tokens all members of that group have in common).
__device__ __host__ __forceinline__ int ginfo_range_begin(int S, int s) { (void)S; return s; }
__device__ __host__ __forceinline__ int ginfo_group_size(int S, int s) { return S + s; }
__device__ __host__ __forceinline__ int ginfo_group_prefix(int S, int s) { return 2 * S + s; }
__device__ __host__ __forceinline__ int ginfo_adj(int S, int s) { return 3 * S + s; }
// compact list of the first sequences of groups with two or more members, and its length
__device__ __host__ __forceinline__ int ginfo_shared_list(int S, int i) { return 4 * S + i; }
__device__ __host__ __forceinline__ int ginfo_shared_count(int S) { return 5 * S; }
__device__ __host__ __forceinline__ size_t ginfo_words(int S) { return 5 * (size_t)S + 4; }

// A sixteen-wave workgroup is kept alone on its compute unit (at most 7 waves
// per SIMD, so a second one does not fit): measured on batches of mixed
// lengths, two resident workgroups each run at half speed and stretch the end
// of the launch by more than their overlap gains.
#define PA_OCC_ATTR __attribute__((amdgpu_waves_per_eu(W == 16 ? 4 : 1, W == 16 ? 7 : 8)))
#define PA_OCC_ATTR_FUSED __attribute__((amdgpu_waves_per_eu(WS == 16 ? 4 : 1, WS == 16 ? 7 : 8)))
template <int DT, int D, int B, int W, int U, int MODE, int G>
__device__ __forceinline__ void decode_body(const DecodeParams &P, const int block_index)
{
    using Tr = Traits<DT>;
    constexpr int E = Tr::E, EPL = Tr::EPL;
    constexpr int ROW_BYTES = D * E;
    constexpr int LPT = ROW_BYTES / 16;
    constexpr int TPL = kWave / LPT;
    constexpr int LPC = (B / TPL) < 4 ? (B / TPL) : 4;
    constexpr int CT = LPC * TPL;
    constexpr int64_t TILE_BYTES = (int64_t)B * ROW_BYTES;
    static_assert(LPT >= 8 && LPT <= 32 && B % TPL == 0 && B % CT == 0 && LPC >= 1, "shape");
    static_assert(G == 1 || MODE == MODE_PREFIX, "several queries only in the shared-prefix mode");

    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int g = lane / LPT;
    const int c = lane % LPT;
    const uint32_t lane16 = (uint32_t)lane * 16u;
    const int H = P.H;

    int item = block_index;
    const int h = item % H;
    item /= H;

    // s: the sequence whose block table is walked; members: query slots in use
    int s, part = 0, parts_stride = 1, t_begin = 0, t_end, members = 1;
    if (MODE == MODE_PREFIX) {
        if (item >= P.ginfo[ginfo_shared_count(P.S)]) return;
        s = P.ginfo[ginfo_shared_list(P.S, item)];   // a group is named by its first sequence
        members = P.ginfo[ginfo_group_size(P.S, s)];
        t_end = P.ginfo[ginfo_group_prefix(P.S, s)];
        parts_stride = 2;
        if (members < 2) return;
    } else if (MODE == MODE_SUFFIX) {
        s = item;
        t_begin = P.ginfo[ginfo_range_begin(P.S, s)];
        t_end = P.context_lens[s];
        part = 1;
        parts_stride = 2;
    } else if (MODE == MODE_PART) {
        part = item % P.max_parts;
        s = item / P.max_parts;
        parts_stride = P.max_parts;
        const int n = P.context_lens[s];
        t_begin = part * P.partition_size;
        t_end = t_begin + P.partition_size < n ? t_begin + P.partition_size : n;
    } else {
        s = item;
        t_end = P.context_lens[s];
    }
    if (t_begin >= t_end) {
        if (MODE == MODE_SINGLE && w == 0 && g == 0) {
            // empty context: zero row
            reinterpret_cast<uint4 *>(P.out)[((int64_t)s * H + h) * LPT + c] = make_uint4(0, 0, 0, 0);
        }
        return;
    }

    // members of a group are consecutive sequences s, s+1, ...
    uint4 qf[G];
#pragma unroll
    for (int j = 0; j < G; ++j) {
        const int sj = j < members ? s + j : s;
        qf[j] = reinterpret_cast<const uint4 *>(P.q)[((int64_t)sj * H + h) * LPT + c];
    }
    const int32_t *__restrict__ table = P.block_tables + (int64_t)s * P.max_blocks;
    const int nchunks = (t_end - t_begin + CT - 1) / CT;

    float m[G], l[G], acc[G][EPL];
#pragma unroll
    for (int j = 0; j < G; ++j) {
        m[j] = kNegBig;
        l[j] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[j][e] = 0.f;
    }

    struct Chunk {
        uint4 k[LPC], v[LPC];
    };

    auto block_of = [&](int ci) -> int {
        // ci is wave-uniform: this is a scalar load
        return table[(t_begin + ci * CT) / B];
    };
    auto issue = [&](Chunk &ck, int ci, int pb) {
        const int t0 = t_begin + ci * CT;
        const int64_t off = ((int64_t)pb * H + h) * TILE_BYTES + (int64_t)(t0 % B) * ROW_BYTES;
        const char *kp = P.k_cache + off + lane16;
        const char *vp = P.v_cache + off + lane16;
#pragma unroll
        for (int i = 0; i < LPC; ++i) ck.k[i] = load16_stream(kp + i * 1024);
#pragma unroll
        for (int i = 0; i < LPC; ++i) ck.v[i] = load16_stream(vp + i * 1024);
    };
    // MASK is set only for a chunk that may reach past t_end (the last one)
    auto consume = [&](Chunk &ck, int ci, auto mask_tag) {
        constexpr bool MASK = decltype(mask_tag)::value;
        const int t0 = t_begin + ci * CT;
        if (MASK) {
            // slots at or past t_end hold no token and may contain anything, NaN
            // included - select them away, never multiply
#pragma unroll
            for (int i = 0; i < LPC; ++i) {
                const bool dead = t0 + i * TPL + g >= t_end;
                ck.v[i].x = dead ? 0u : ck.v[i].x;
                ck.v[i].y = dead ? 0u : ck.v[i].y;
                ck.v[i].z = dead ? 0u : ck.v[i].z;
                ck.v[i].w = dead ? 0u : ck.v[i].w;
            }
        }
#pragma unroll
        for (int j = 0; j < G; ++j) {
            if (G > 1 && j >= members) break;
            float x[LPC];
#pragma unroll
            for (int i = 0; i < LPC; ++i) x[i] = group_sum<LPT>(Tr::dot(ck.k[i], qf[j], 0.f)) * P.scale_log2;
            if (MASK) {
#pragma unroll
                for (int i = 0; i < LPC; ++i) x[i] = (t0 + i * TPL + g >= t_end) ? -INFINITY : x[i];
            }
            float m_new = m[j];
#pragma unroll
            for (int i = 0; i < LPC; ++i) m_new = fmaxf(m_new, x[i]);
            const float alpha = __builtin_amdgcn_exp2f(m[j] - m_new);
            float p[LPC], psum = 0.f;
#pragma unroll
            for (int i = 0; i < LPC; ++i) {
                p[i] = __builtin_amdgcn_exp2f(x[i] - m_new);
                psum += p[i];
            }
            l[j] = l[j] * alpha + psum;
            m[j] = m_new;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[j][e] *= alpha;
#pragma unroll
            for (int i = 0; i < LPC; ++i) {
                Tr::axpy(acc[j], p[i], ck.v[i]);
                // bf16 widening is two VALU ops per pair; without a fence the
                // scheduler widens every fragment first and doubles the live registers
                if (Tr::FENCE_AXPY) __builtin_amdgcn_sched_barrier(0);
            }
            // one member at a time: interleaving their arithmetic multiplies the live registers
            if (G > 1) __builtin_amdgcn_sched_barrier(0);
        }
    };
    const std::false_type full{};
    const std::true_type masked{};

    // Steady state: U chunks per trip, all loads issued up front, then consumed
    // in order, in one straight-line block (nothing loaded is carried across the
    // back edge, so the compiler waits exactly for the fragment it needs next).
    // Chunks before the last one of the range are full; the remainder loop takes
    // one chunk at a time with masking.  Latency is hidden by the other waves
    // resident on the SIMD.
    {
        int ci = w;
        for (; ci + (U - 1) * W <= nchunks - 2; ci += U * W) {
            Chunk ck[U];
            int pb[U];
#pragma unroll
            for (int u = 0; u < U; ++u) pb[u] = block_of(ci + u * W);
#pragma unroll
            for (int u = 0; u < U; ++u) issue(ck[u], ci + u * W, pb[u]);
#pragma unroll
            for (int u = 0; u < U; ++u) consume(ck[u], ci + u * W, full);
        }
        for (; ci < nchunks; ci += W) {
            Chunk ck;
            issue(ck, ci, block_of(ci));
            consume(ck, ci, masked);
        }
    }

    // merge the TPL token groups of this wave (lanes with equal c)
#pragma unroll
    for (int j = 0; j < G; ++j) {
        float M = m[j];
#pragma unroll
        for (int d = LPT; d < kWave; d <<= 1) M = fmaxf(M, __shfl_xor(M, d));
        const float f = __builtin_amdgcn_exp2f(m[j] - M);
        l[j] *= f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[j][e] *= f;
#pragma unroll
        for (int d = LPT; d < kWave; d <<= 1) {
            l[j] += __shfl_xor(l[j], d);
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[j][e] += __shfl_xor(acc[j][e], d);
        }
        m[j] = M;
    }

    // merge the W waves of the workgroup through LDS
    if (W > 1) {
        __shared__ float sm_acc[W][G][D];
        __shared__ float sm_m[W][G], sm_l[W][G];
        if (g == 0) {
#pragma unroll
            for (int j = 0; j < G; ++j) {
#pragma unroll
                for (int e = 0; e < EPL; ++e) sm_acc[w][j][c * EPL + e] = acc[j][e];
                if (c == 0) {
                    sm_m[w][j] = m[j];
                    sm_l[w][j] = l[j];
                }
            }
        }
        __syncthreads();
        if (w != 0) return;
#pragma unroll
        for (int j = 0; j < G; ++j) {
            float M = sm_m[0][j];
#pragma unroll
            for (int i = 1; i < W; ++i) M = fmaxf(M, sm_m[i][j]);
            l[j] = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[j][e] = 0.f;
            // (not fully unrolled: sixteen waves' worth of LDS reads hoisted at once would spill)
#pragma unroll 2
            for (int i = 0; i < W; ++i) {
                const float f = __builtin_amdgcn_exp2f(sm_m[i][j] - M);
                l[j] = __builtin_fmaf(sm_l[i][j], f, l[j]);
#pragma unroll
                for (int e = 0; e < EPL; ++e)
                    acc[j][e] = __builtin_fmaf(sm_acc[i][j][c * EPL + e], f, acc[j][e]);
            }
            m[j] = M;
        }
    }
    if (g != 0) return;

    if (MODE == MODE_SINGLE) {
        const float inv = 1.0f / l[0];
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[0][e] *= inv;
        reinterpret_cast<uint4 *>(P.out)[((int64_t)s * H + h) * LPT + c] = Tr::pack(acc[0]);
    } else {
        // unnormalised partials: the reduce kernel divides once
#pragma unroll
        for (int j = 0; j < G; ++j) {
            if (j >= members) break;
            const int64_t slot = ((int64_t)(s + j) * H + h) * parts_stride + part;
            float *dst = P.ws_acc + slot * D + c * EPL;
#pragma unroll
            for (int e = 0; e < EPL; e += 4)
                *reinterpret_cast<float4 *>(dst + e) =
                    make_float4(acc[j][e], acc[j][e + 1], acc[j][e + 2], acc[j][e + 3]);
            if (c == 0) *reinterpret_cast<float2 *>(P.ws_ml + slot * 2) = make_float2(m[j], l[j]);
        }
    }
}

template <int DT, int D, int B, int W, int U, int MODE, int G>
__global__ __launch_bounds__(W *kWave) PA_OCC_ATTR void pa_decode_kernel(const DecodeParams P)
{
    decode_body<DT, D, B, W, U, MODE, G>(P, (int)blockIdx.x);
}

// ---- shared-prefix decode on the matrix cores --------------------------------
// A group's common prefix is a small dense contraction: up to 16 queries against
// 16-token K/V tiles.  One workgroup per (group, head); wave w takes tiles
// w, w+W, ...  Per tile:
//   S^T = K Q^T   8 x v_mfma_f32_16x16x16 (f16 or bf16 operands, fp32 result):
//                 A rows are tokens, B columns are queries.  Lane l supplies
//                 row l%16; each of its four 16-byte loads feeds two MFMAs,
//                 with the same (arbitrary but consistent) assignment of head
//                 dimensions to contraction slots on the Q side.
//   softmax       the result leaves lane l with query l%16 and four tokens;
//                 the running maximum is kept per query (two cross-lane maxima
//                 per tile), exp2 in fp32, rescaling of the output only when
//                 some maximum moved.
//   O += P V      32 x v_mfma_f32_16x16x4_f32: A = P in fp32 straight from the
//                 softmax registers, B = the V fragments of the ordinary
//                 coalesced load widened to fp32 (lane l: token l/16 + 4v,
//                 dims 8*(l%16)+e; output column l%16 of MFMA e is dim
//                 8*(l%16)+e).  fp32 operands keep P exact; the fp32 matrix
//                 rate is still about three times what the HBM stream needs.
// K rows are loaded in the order token(i) = i/4 + 4*(i%4) so that result
// register v of lane l belongs to token l/16 + 4v, the token of V fragment v
// in that lane: P never moves between lanes.
// Outputs: the same unnormalised partials as MODE_PREFIX (partial 0 of 2).
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));

template <int DT>
__device__ __forceinline__ float4_t mfma_qk(uint32_t a0, uint32_t a1, uint32_t b0, uint32_t b1, float4_t c)
{
    const uint2 a = make_uint2(a0, a1), b = make_uint2(b0, b1);
    if (DT == PA_F16)
        return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(half4_t, a),
                                                     __builtin_bit_cast(half4_t, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(short4_t, a),
                                                         __builtin_bit_cast(short4_t, b), c, 0, 0, 0);
}

template <int DT>
__device__ __forceinline__ void widen8(float (&f)[8], const uint4 &v)
{
    const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (DT == PA_F16) {
            const half2_t h = __builtin_bit_cast(half2_t, u[i]);
            f[2 * i] = (float)h.x;
            f[2 * i + 1] = (float)h.y;
        } else {
            f[2 * i] = as_f32(u[i] << 16);
            f[2 * i + 1] = as_f32(u[i] & 0xffff0000u);
        }
    }
}

// MULTI = false: a group's shared prefix (GQ = 8 query slots, partial results).
// MULTI = true:  the last q_len tokens of ONE sequence as queries over its whole
//                context, 16 per workgroup, with the causal rule that query i of the
//                q_len new tokens sees tokens 0 .. n - q_len + i; writes output rows.
template <int DT, int B, int W, int GQ, bool MULTI>
__device__ __forceinline__ void prefix_mfma_body(const DecodeParams &P, const int block_index)
{
    using Tr = Traits<DT>;
    constexpr int D = 128, ROW_BYTES = 256;
    constexpr int64_t TILE_BYTES = (int64_t)B * ROW_BYTES;
    static_assert(DT != PA_F32 && B % 16 == 0, "two-byte elements, whole 16-token tiles per block");
    static_assert(GQ <= 16, "one MFMA row per query");

    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int r = lane / 16;
    const int c = lane % 16;
    const int H = P.H;
    const int h = block_index % H;
    const int rest = block_index / H;

    // s: sequence whose table is walked; query c of this item is row q_row0 + c*q_row_step
    // of P.q; tokens [0, t_hi) are visited; token t counts for query c iff t <= limit
    int s, members, t_hi, t_lo, limit;
    int64_t q_row0, q_row_step;
    if (MULTI) {
        const int qb = rest % P.q_blocks;
        s = rest / P.q_blocks;
        const int n = P.context_lens[s];
        const int qs = P.q_start[s];
        const int qlen = P.q_start[s + 1] - qs;
        const int q0 = qb * 16;
        if (q0 >= qlen || n <= 0) return;
        members = qlen - q0 < 16 ? qlen - q0 : 16;
        t_lo = n - qlen + q0 + 1;            // tokens the first query of the item sees
        t_hi = t_lo + members - 1;           // tokens the last one sees
        if (t_hi > n) t_hi = n;
        limit = c < members ? t_lo - 1 + c : -1;
        q_row0 = qs + q0;
        q_row_step = 1;
    } else {
        if (rest >= P.ginfo[ginfo_shared_count(P.S)]) return;
        s = P.ginfo[ginfo_shared_list(P.S, rest)];   // a group is named by its first sequence
        members = P.ginfo[ginfo_group_size(P.S, s)];
        t_hi = P.ginfo[ginfo_group_prefix(P.S, s)];
        if (members < 2 || t_hi <= 0) return;
        if (members > GQ) members = GQ;
        t_lo = t_hi;                          // every member sees every token of the prefix
        limit = 0x7fffffff;
        q_row0 = s;
        q_row_step = 1;
    }
    const int ntiles = (t_hi + 15) / 16;

    // Q^T as the B operand: lane l holds, for query l%16, the same byte ranges of the
    // query row that it will hold of each K row
    uint4 qf[4];
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) {
        qf[cc] = make_uint4(0, 0, 0, 0);
        if (c < members)
            qf[cc] = *reinterpret_cast<const uint4 *>(static_cast<const char *>(P.q) +
                                                      ((q_row0 + c * q_row_step) * H + h) * ROW_BYTES +
                                                      64 * cc + 16 * r);
    }
    float4_t O[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) O[e] = float4_t{0.f, 0.f, 0.f, 0.f};
    float m = kNegBig, lsum = 0.f;

    const int32_t *__restrict__ table = P.block_tables + (int64_t)s * P.max_blocks;
    const uint32_t k_lane_off = (uint32_t)((c / 4 + 4 * (c % 4)) * ROW_BYTES + 16 * r);
    const uint32_t v_lane_off = (uint32_t)lane * 16u;

    for (int ti = w; ti < ntiles; ti += W) {
        const int t0 = ti * 16;
        const int pb = table[t0 / B];
        const int64_t base = ((int64_t)pb * H + h) * TILE_BYTES + (int64_t)(t0 % B) * ROW_BYTES;
        uint4 kf[4], vf[4];
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) kf[cc] = load16_stream(P.k_cache + base + k_lane_off + 64 * cc);
#pragma unroll
        for (int v = 0; v < 4; ++v) vf[v] = load16_stream(P.v_cache + base + v_lane_off + 1024 * v);

        float4_t S = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
            S = mfma_qk<DT>(kf[cc].x, kf[cc].y, qf[cc].x, qf[cc].y, S);
            S = mfma_qk<DT>(kf[cc].z, kf[cc].w, qf[cc].z, qf[cc].w, S);
        }
        float x[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) x[v] = S[v] * P.scale_log2;
        if (MULTI && t0 + 16 > t_lo) {
            // the tile reaches past what the first query sees: apply the causal rule per
            // (query, token), and clear V rows no query of the item sees (they may lie
            // past the context and hold anything) - by select, never by multiplying
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int tok = t0 + r + 4 * v;
                x[v] = tok <= limit ? x[v] : -INFINITY;
                const bool unseen = tok >= t_hi;
                vf[v].x = unseen ? 0u : vf[v].x;
                vf[v].y = unseen ? 0u : vf[v].y;
                vf[v].z = unseen ? 0u : vf[v].z;
                vf[v].w = unseen ? 0u : vf[v].w;
            }
        }
        float tmax = fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3]));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float m_new = fmaxf(m, tmax);
        if (__any(m_new > m)) {
            const float alpha = __builtin_amdgcn_exp2f(m - m_new);
            lsum *= alpha;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float a = __shfl(alpha, 4 * r + v);   // output row 4r+v is query 4r+v
#pragma unroll
                for (int e = 0; e < 8; ++e) O[e][v] *= a;
            }
            m = m_new;
        }
        float p[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            p[v] = __builtin_amdgcn_exp2f(x[v] - m);
            lsum += p[v];
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float vv[8];
            widen8<DT>(vv, vf[v]);
#pragma unroll
            for (int e = 0; e < 8; ++e) O[e] = __builtin_amdgcn_mfma_f32_16x16x4f32(p[v], vv[e], O[e], 0, 0, 0);
        }
    }
    lsum += __shfl_xor(lsum, 16);
    lsum += __shfl_xor(lsum, 32);

    // merge the waves: per query, its 128 accumulators sit in the 16 lanes r = query/4
    __shared__ float sm_acc[W][GQ][D];
    __shared__ float sm_m[W][GQ], sm_l[W][GQ];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int qi = 4 * r + v;
        if (qi < members) {
#pragma unroll
            for (int e = 0; e < 8; ++e) sm_acc[w][qi][8 * c + e] = O[e][v];
        }
    }
    if (r == 0 && c < members) {
        sm_m[w][c] = m;
        sm_l[w][c] = lsum;
    }
    __syncthreads();
    if (w != 0 || r != 0) return;
    for (int j = 0; j < members; ++j) {
        float M = sm_m[0][j];
#pragma unroll
        for (int i = 1; i < W; ++i) M = fmaxf(M, sm_m[i][j]);
        float l = 0.f, acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll 2
        for (int i = 0; i < W; ++i) {
            const float f = __builtin_amdgcn_exp2f(sm_m[i][j] - M);
            l = __builtin_fmaf(sm_l[i][j], f, l);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = __builtin_fmaf(sm_acc[i][j][8 * c + e], f, acc[e]);
        }
        if (MULTI) {
            const float inv = 1.0f / l;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] *= inv;
            reinterpret_cast<uint4 *>(P.out)[((q_row0 + j) * H + h) * 16 + c] = Tr::pack(acc);
        } else {
            const int64_t slot = ((int64_t)(s + j) * H + h) * 2;
            float *dst = P.ws_acc + slot * D + 8 * c;
            *reinterpret_cast<float4 *>(dst) = make_float4(acc[0], acc[1], acc[2], acc[3]);
            *reinterpret_cast<float4 *>(dst + 4) = make_float4(acc[4], acc[5], acc[6], acc[7]);
            if (c == 0) *reinterpret_cast<float2 *>(P.ws_ml + slot * 2) = make_float2(M, l);
        }
    }
}

// Several query tokens per sequence (the tail of a prompt over an already cached
// prefix, Sec. 4.4 "shared prefix"; or draft tokens to verify): grid =
// (sequence, block of 16 queries, head).
template <int DT, int B, int W>
__global__ __launch_bounds__(W *kWave) void pa_decode_multi_kernel(const DecodeParams P)
{
    prefix_mfma_body<DT, B, W, 16, true>(P, (int)blockIdx.x);
}

// Shared prefixes and private suffixes in one launch.  The first
// P.prefix_blocks workgroups are shared-prefix items (group, head), the rest
// are suffix items (sequence, head); the short prefix items start first and the
// long suffix items fill the machine around them.
template <int DT, int B, int WS, int WP>
__global__ __launch_bounds__(WS *kWave) PA_OCC_ATTR_FUSED void pa_shared_fused_kernel(const DecodeParams P)
{
    static_assert(WP == WS, "every wave of the workgroup takes part in either kind of item");
    if ((int)blockIdx.x < P.prefix_blocks) {
        prefix_mfma_body<DT, B, WP, kGroupMaxMfma, false>(P, (int)blockIdx.x);
    } else {
        decode_body<DT, 128, B, WS, kChunksPerTripDevice, MODE_SUFFIX, 1>(P, (int)blockIdx.x - P.prefix_blocks);
    }
}

// Merge of partials: out = sum_p 2^(m_p-M) a_p / sum_p 2^(m_p-M) l_p with a_p the
// unnormalised partial sums.  One wavefront per (sequence, head); lane c
// handles the same 16-byte output fragment as in the decode kernel.  With
// fixed partitions the first ceil(n/PS) partials exist; on the shared-prefix
// path partial 0 (prefix) exists when range_begin[s] > 0 and partial 1
// (suffix) when range_begin[s] < n.
template <int DT, int D, bool SHARED>
__global__ __launch_bounds__(kWave) void pa_reduce_kernel(const DecodeParams P)
{
    using Tr = Traits<DT>;
    constexpr int EPL = Tr::EPL;
    constexpr int LPT = D * Tr::E / 16;
    const int c = threadIdx.x;
    if (c >= LPT) return;
    const int H = P.H;
    const int h = blockIdx.x % H;
    const int s = blockIdx.x / H;
    const int n = P.context_lens[s];
    int first = 0, last, stride;
    if (SHARED) {
        const int rb = P.ginfo[ginfo_range_begin(P.S, s)];
        stride = 2;
        first = rb > 0 ? 0 : 1;
        last = n > rb ? 2 : 1;
    } else {
        stride = P.max_parts;
        last = (n + P.partition_size - 1) / P.partition_size;
        if (last > stride) last = stride;
    }
    const int64_t base = ((int64_t)s * H + h) * stride;
    float acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
    if (n > 0 && first < last) {
        float M = kNegBig;
        for (int p = first; p < last; ++p) M = fmaxf(M, P.ws_ml[(base + p) * 2]);
        float l = 0.f;
        for (int p = first; p < last; ++p) {
            const float2 ml = *reinterpret_cast<const float2 *>(P.ws_ml + (base + p) * 2);
            const float f = __builtin_amdgcn_exp2f(ml.x - M);
            l = __builtin_fmaf(ml.y, f, l);
            const float *src = P.ws_acc + (base + p) * D + c * EPL;
#pragma unroll
            for (int e = 0; e < EPL; e += 4) {
                const float4 a = *reinterpret_cast<const float4 *>(src + e);
                acc[e] = __builtin_fmaf(a.x, f, acc[e]);
                acc[e + 1] = __builtin_fmaf(a.y, f, acc[e + 1]);
                acc[e + 2] = __builtin_fmaf(a.z, f, acc[e + 2]);
                acc[e + 3] = __builtin_fmaf(a.w, f, acc[e + 3]);
            }
        }
        const float inv = 1.0f / l;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] *= inv;
    }
    reinterpret_cast<uint4 *>(P.out)[((int64_t)s * H + h) * LPT + c] = Tr::pack(acc);
}

// Group discovery for the shared-prefix path.  Consecutive sequences whose
// block tables start with the same physical blocks form a group (that is how
// forked sequences sit in a batch: samples of one prompt, beams of one
// search).  Only blocks that are full for both neighbours count, so every
// token of a shared prefix is valid for every member.
//   adj[s] = leading blocks s has in common with s-1 (0 for s = 0).
// A sequence with adj = 0 starts a run; runs are independent, so one thread
// walks each run: a sequence joins the current group while the group has room
// and the common prefix would keep at least three quarters of its length,
// otherwise it starts a new group.  One workgroup, state in LDS when it fits.
constexpr int kGroupScanLds = 2048;   // sequences whose scan state fits in LDS
constexpr int kGroupThreads = 1024;

__device__ __forceinline__ void group_walk_run(const int32_t *adj, int32_t *range_begin, int32_t *g_size,
                                               int32_t *g_prefix, int first, int S, int block_size,
                                               int group_max)
{
    int start = first, size = 1, prefix = 0;
    auto close = [&]() {
        const int tokens = size > 1 ? prefix * block_size : 0;
        g_size[start] = size;
        g_prefix[start] = tokens;
        for (int j = 0; j < size; ++j) range_begin[start + j] = tokens;
    };
    for (int sq = first + 1; sq < S; ++sq) {
        const int a = adj[sq];
        if (a == 0) break;   // the next run belongs to another thread
        bool join = false;
        if (size < group_max) {
            const int np = size == 1 ? a : (a < prefix ? a : prefix);
            join = size == 1 || 4 * np >= 3 * prefix;
            if (join) prefix = np;
        }
        if (join) {
            ++size;
        } else {
            close();
            start = sq;
            size = 1;
            prefix = 0;
        }
    }
    close();
}

__global__ __launch_bounds__(kGroupThreads) void find_groups_kernel(
    const int32_t *__restrict__ block_tables, int32_t max_blocks,
    const int32_t *__restrict__ context_lens, int32_t S, int32_t block_size, int32_t group_max,
    int32_t *__restrict__ ginfo)
{
    __shared__ int32_t s_adj[kGroupScanLds], s_range[kGroupScanLds], s_size[kGroupScanLds],
        s_prefix[kGroupScanLds];
    const bool in_lds = S <= kGroupScanLds;

    // adj[s]: one wavefront compares the table rows of s-1 and s, 64 entries per
    // step (lanes in parallel, first mismatch by ballot), four sequences per trip
    // so that their loads are in flight together
    const int lane = threadIdx.x & (kWave - 1);
    const int w = threadIdx.x / kWave;
    constexpr int NW = kGroupThreads / kWave, UN = 4;
    for (int base = w * UN; base < S; base += NW * UN) {
        int lim[UN], e0[UN], e1[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int sq = base + u;
            lim[u] = 0;
            if (sq > 0 && sq < S) {
                const int n0 = context_lens[sq - 1], n1 = context_lens[sq];
                lim[u] = (n0 < n1 ? n0 : n1) / block_size;
            }
            e0[u] = e1[u] = 0;
            if (lane < lim[u]) {
                e0[u] = block_tables[(int64_t)(sq - 1) * max_blocks + lane];
                e1[u] = block_tables[(int64_t)sq * max_blocks + lane];
            }
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int sq = base + u;
            if (sq >= S) break;
            int a = 0;
            unsigned long long diff = __ballot(lane < lim[u] && e0[u] != e1[u]);
            if (diff) {
                a = __builtin_ctzll(diff);
            } else {
                a = lim[u] < kWave ? lim[u] : kWave;
                // the first 64 blocks all agree: keep comparing (long shared prefixes)
                for (int j0 = kWave; j0 < lim[u] && a == j0; j0 += kWave) {
                    const int j = j0 + lane;
                    bool ne = false;
                    if (j < lim[u])
                        ne = block_tables[(int64_t)(sq - 1) * max_blocks + j] !=
                             block_tables[(int64_t)sq * max_blocks + j];
                    diff = __ballot(ne);
                    const int rest = lim[u] - j0 < kWave ? lim[u] - j0 : kWave;
                    a = j0 + (diff ? (int)__builtin_ctzll(diff) : rest);
                }
            }
            if (lane == 0) {
                if (in_lds) {
                    s_adj[sq] = a;
                    s_size[sq] = 0;
                } else {
                    ginfo[ginfo_adj(S, sq)] = a;
                    ginfo[ginfo_group_size(S, sq)] = 0;
                }
            }
        }
    }
    __syncthreads();
    if (in_lds) {
        for (int sq = threadIdx.x; sq < S; sq += kGroupThreads)
            if (s_adj[sq] == 0) group_walk_run(s_adj, s_range, s_size, s_prefix, sq, S, block_size, group_max);
        __syncthreads();
        for (int i = threadIdx.x; i < S; i += kGroupThreads) {
            ginfo[ginfo_range_begin(S, i)] = s_range[i];
            ginfo[ginfo_group_size(S, i)] = s_size[i];
            ginfo[ginfo_group_prefix(S, i)] = s_size[i] ? s_prefix[i] : 0;
        }
    } else {
        for (int sq = threadIdx.x; sq < S; sq += kGroupThreads)
            if (ginfo[ginfo_adj(S, sq)] == 0)
                group_walk_run(ginfo + ginfo_adj(S, 0), ginfo + ginfo_range_begin(S, 0),
                               ginfo + ginfo_group_size(S, 0), ginfo + ginfo_group_prefix(S, 0), sq, S,
                               block_size, group_max);
    }
    __syncthreads();
    // compact the first sequences of shared groups (two or more members), in order, so that
    // the prefix kernel's workgroups with work come first in its grid
    __shared__ int32_t wave_count[NW];
    __shared__ int32_t running;
    if (threadIdx.x == 0) running = 0;
    __syncthreads();
    for (int base = 0; base < S; base += kGroupThreads) {
        const int sq = base + threadIdx.x;
        const bool flag = sq < S && (in_lds ? s_size[sq] : ginfo[ginfo_group_size(S, sq)]) >= 2;
        const unsigned long long mask = __ballot(flag);
        if (lane == 0) wave_count[w] = __builtin_popcountll(mask);
        __syncthreads();
        int before = running;
        for (int i = 0; i < w; ++i) before += wave_count[i];
        if (flag) ginfo[ginfo_shared_list(S, before + __builtin_popcountll(mask & ((1ull << lane) - 1)))] = sq;
        __syncthreads();
        if (threadIdx.x == 0) {
            int total = running;
            for (int i = 0; i < NW; ++i) total += wave_count[i];
            running = total;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) ginfo[ginfo_shared_count(S)] = running;
}

// ---- reshape_and_cache -------------------------------------------------------
// One thread moves one 16-byte fragment.  A token is frags_per_token = H*D*E/16
// fragments; fragment r of token t belongs to head r / frags_per_row.
__global__ __launch_bounds__(256) void reshape_and_cache_kernel(
    const uint4 *__restrict__ k, const uint4 *__restrict__ v, uint4 *__restrict__ k_cache,
    uint4 *__restrict__ v_cache, const int64_t *__restrict__ slot_mapping, int64_t total_frags,
    int32_t frags_per_token, int32_t frags_per_row, int32_t block_size)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total_frags) return;
    const int64_t t = idx / frags_per_token;
    const int32_t r = (int32_t)(idx - t * frags_per_token);
    const int64_t slot = slot_mapping[t];
    if (slot < 0) return;
    const int64_t pb = slot / block_size;
    const int32_t off = (int32_t)(slot - pb * block_size);
    const int32_t h = r / frags_per_row;
    const int32_t cfrag = r - h * frags_per_row;
    // [NB][H][B][D] in fragments: ((pb*H + h)*B + off)*frags_per_row + cfrag
    const int32_t H = frags_per_token / frags_per_row;
    const int64_t dst = ((pb * H + h) * block_size + off) * frags_per_row + cfrag;
    const uint4 *src = blockIdx.y ? v : k;
    uint4 *cache = blockIdx.y ? v_cache : k_cache;
    store_frag_stream(cache + dst, load_frag_stream(src + idx));
}

// ---- copy_blocks -------------------------------------------------------------
constexpr int kMaxCopyPtrs = 128;   // K and V pointers of up to 64 layers per launch
constexpr int kMaxPairsPerLaunch = 65535;   // grid.y limit; longer pair lists take several launches
struct CachePtrs {
    uint4 *p[kMaxCopyPtrs];
};

// grid = (256-fragment slices of a block, pairs, caches); a block of one cache
// is frags_per_block consecutive 16-byte fragments.  One fragment per thread:
// with randomly placed pairs, many small workgroups measured 5.9 TB/s of
// read+write traffic against 5.2 TB/s with four fragments per thread.
__global__ __launch_bounds__(256) void copy_blocks_kernel(CachePtrs caches,
                                                           const int64_t *__restrict__ pairs,
                                                           int64_t frags_per_block)
{
    uint4 *cache = caches.p[blockIdx.z];
    const int64_t src = pairs[2 * (int64_t)blockIdx.y];
    const int64_t dst = pairs[2 * (int64_t)blockIdx.y + 1];
    const int64_t f = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (f < frags_per_block)
        store_frag_stream(cache + dst * frags_per_block + f, load_frag_stream(cache + src * frags_per_block + f));
}

// Block copy between two sets of caches (swap to and from host memory, Sec. 4.5):
// the same one-fragment-per-thread copy with separate source and destination
// arrays, either of which may be pinned host memory mapped into the device's
// address space.  grid = (slices, pairs, 2 x layers).
constexpr int kMaxSwapLayers = kMaxCopyPtrs / 4;
struct SwapPtrs {
    const uint4 *src[kMaxCopyPtrs / 2];
    uint4 *dst[kMaxCopyPtrs / 2];
};
__global__ __launch_bounds__(256) void swap_blocks_kernel(SwapPtrs caches,
                                                           const int64_t *__restrict__ pairs,
                                                           int64_t frags_per_block)
{
    const uint4 *from = caches.src[blockIdx.z];
    uint4 *to = caches.dst[blockIdx.z];
    const int64_t src = pairs[2 * (int64_t)blockIdx.y];
    const int64_t dst = pairs[2 * (int64_t)blockIdx.y + 1];
    const int64_t f = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (f < frags_per_block)
        store_frag_stream(to + dst * frags_per_block + f, load_frag_stream(from + src * frags_per_block + f));
}

// ---- bandwidth probe ---------------------------------------------------------
// Each workgroup streams one contiguous 256 KiB tile with non-temporal 16-byte
// loads, eight in flight per thread: the access shape that reads fastest here.
constexpr int kProbeTileFrags = 256 * 1024 / 16;
__global__ __launch_bounds__(256) void stream_read_kernel(const char *__restrict__ src,
                                                           int64_t frags, uint32_t *sink)
{
    constexpr int U = 8;
    const int64_t base = (int64_t)blockIdx.x * kProbeTileFrags;
    uint32_t a = 0;
    for (int i = threadIdx.x; i < kProbeTileFrags; i += 256 * U) {
        uint4 x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t f = base + i + u * 256;
            x[u] = f < frags ? load16_stream(src + f * 16) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) a += x[u].x ^ x[u].y ^ x[u].z ^ x[u].w;
    }
    // a store that (almost) never happens keeps the loads alive without write traffic
    if (a == 0x9e3779b9u) sink[blockIdx.x & 65535] = a;
}

// ---- host side -----------------------------------------------------------------
int elem_bytes(pa_dtype dt) { return dt == PA_F32 ? 4 : 2; }

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool shape_supported(pa_dtype dt, int D, int B)
{
    if (dt != PA_F32 && dt != PA_F16 && dt != PA_BF16) return false;
    if (D != 64 && D != 128) return false;
    if (B != 8 && B != 16 && B != 32 && B != 64 && B != 128) return false;
    const int lpt = D * elem_bytes(dt) / 16;   // lanes per token row
    const int tpl = kWave / lpt;
    return lpt >= 8 && lpt <= 32 && B % tpl == 0;
}

struct DecodeArgs {
    DecodeParams p;
    int32_t waves;   // wavefronts per workgroup
    hipStream_t stream;
};

template <int DT, int D, int B, int W, int MODE, int G = 1>
void launch_decode_kernel(const DecodeArgs &a, unsigned items)
{
    hipLaunchKernelGGL((pa_decode_kernel<DT, D, B, W, (G > 1 ? 1 : kChunksPerTrip), MODE, G>),
                       dim3(items * (unsigned)a.p.H),
                       dim3(W * kWave), 0, a.stream, a.p);
}

template <int DT, int D, int B>
void dispatch_mode(const DecodeArgs &a, int mode)
{
    const unsigned S = (unsigned)a.p.S;
    const unsigned rows = S * (unsigned)a.p.H;
    if (mode == MODE_PART) {
        if (a.waves >= 8)
            launch_decode_kernel<DT, D, B, 8, MODE_PART>(a, S * (unsigned)a.p.max_parts);
        else
            launch_decode_kernel<DT, D, B, 4, MODE_PART>(a, S * (unsigned)a.p.max_parts);
        hipLaunchKernelGGL((pa_reduce_kernel<DT, D, false>), dim3(rows), dim3(kWave), 0, a.stream, a.p);
    } else if (mode == MODE_PREFIX) {
        // shared-prefix path: group table, prefixes once per group, private suffixes, merge
        constexpr bool kMfma = DT != PA_F32 && D == 128 && B % 16 == 0;
        hipLaunchKernelGGL(find_groups_kernel, dim3(1), dim3(kGroupThreads), 0, a.stream, a.p.block_tables,
                           a.p.max_blocks, a.p.context_lens, a.p.S, B, kMfma ? kGroupMaxMfma : kGroupMax,
                           const_cast<int32_t *>(a.p.ginfo));
        if constexpr (kMfma) {
            // a shared group has two or more members: at most S/2 groups
            DecodeArgs f = a;
            f.p.prefix_blocks = (int32_t)(((S + 1) / 2) * (unsigned)a.p.H);
            const unsigned blocks = (unsigned)f.p.prefix_blocks + rows;
            // eight waves per workgroup: two workgroups share a compute unit, so a short prefix
            // item's load latency is covered by a streaming suffix item (measured better than sixteen)
            if (a.waves >= 8)
                hipLaunchKernelGGL((pa_shared_fused_kernel<DT, B, 8, 8>), dim3(blocks), dim3(8 * kWave), 0, a.stream, f.p);
            else
                hipLaunchKernelGGL((pa_shared_fused_kernel<DT, B, 4, 4>), dim3(blocks), dim3(4 * kWave), 0, a.stream, f.p);
        } else {
            launch_decode_kernel<DT, D, B, 8, MODE_PREFIX, kGroupMax>(a, S);
            if (a.waves >= 16)
                launch_decode_kernel<DT, D, B, 16, MODE_SUFFIX>(a, S);
            else if (a.waves >= 8)
                launch_decode_kernel<DT, D, B, 8, MODE_SUFFIX>(a, S);
            else
                launch_decode_kernel<DT, D, B, 4, MODE_SUFFIX>(a, S);
        }
        hipLaunchKernelGGL((pa_reduce_kernel<DT, D, true>), dim3(rows), dim3(kWave), 0, a.stream, a.p);
    } else {
        switch (a.waves) {
        case 2: launch_decode_kernel<DT, D, B, 2, MODE_SINGLE>(a, S); break;
        case 4: launch_decode_kernel<DT, D, B, 4, MODE_SINGLE>(a, S); break;
        case 8: launch_decode_kernel<DT, D, B, 8, MODE_SINGLE>(a, S); break;
        default: launch_decode_kernel<DT, D, B, 16, MODE_SINGLE>(a, S); break;
        }
    }
}

template <int DT, int D>
bool dispatch_block(const DecodeArgs &a, int B, int mode)
{
    switch (B) {
    case 8: dispatch_mode<DT, D, 8>(a, mode); return true;
    case 16: dispatch_mode<DT, D, 16>(a, mode); return true;
    case 32: dispatch_mode<DT, D, 32>(a, mode); return true;
    case 64: dispatch_mode<DT, D, 64>(a, mode); return true;
    case 128: dispatch_mode<DT, D, 128>(a, mode); return true;
    }
    return false;
}

bool dispatch_decode(const DecodeArgs &a, pa_dtype dt, int D, int B, int mode)
{
    if (dt == PA_F32 && D == 64) return dispatch_block<PA_F32, 64>(a, B, mode);
    if (dt == PA_F32 && D == 128) return dispatch_block<PA_F32, 128>(a, B, mode);
    if (dt == PA_F16 && D == 64) return dispatch_block<PA_F16, 64>(a, B, mode);
    if (dt == PA_F16 && D == 128) return dispatch_block<PA_F16, 128>(a, B, mode);
    if (dt == PA_BF16 && D == 64) return dispatch_block<PA_BF16, 64>(a, B, mode);
    if (dt == PA_BF16 && D == 128) return dispatch_block<PA_BF16, 128>(a, B, mode);
    return false;
}

// ---- launch planning -----------------------------------------------------------
// Measured on MI355X at the OPT-13B shape: a workgroup should have about one
// wave per four chunks of its longest possible item - fewer waves leave the end
// of the launch to a few slow workgroups, more waves cost launch time that
// short items cannot pay back.  Splitting the context costs 3-8% at large
// batches (workspace traffic, empty workgroups, the second kernel) and pays
// when there are too few (sequence, head) pairs to fill the compute units
// evenly (one sequence of 8192 tokens: 79 us in one pass, 31 us split).
int compute_units()
{
    static int cached = 0;
    if (cached > 0) return cached;
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
        (void)hipGetLastError();
        return 256;   // MI355X; not cached, so a later call with a device present asks again
    }
    cached = n;
    return n;
}

int chunk_tokens(pa_dtype dt, int D, int B)
{
    const int tpl = kWave / (D * elem_bytes(dt) / 16);
    const int lpc = B / tpl < 4 ? B / tpl : 4;
    return lpc * tpl;
}

int waves_for(int tokens_per_item, int ct)
{
    const int chunks = (tokens_per_item + ct - 1) / ct;
    if (chunks <= 4) return 2;
    if (chunks <= 16) return 4;
    if (chunks <= 32) return 8;
    return 16;
}

int auto_partition(int S, int H, int max_context_len)
{
    // One pass when there are at least four (sequence, head) items per compute unit.
    // Fewer items leave units idle or the last round of workgroups mostly empty
    // (8 sequences x 40 heads x 2048 tokens: 61 us in one pass, 53 us split), so
    // the context is cut until there are about four items per unit, in ranges of
    // at least 512 tokens (a multiple of every supported block size).
    const int cus = compute_units();
    const int64_t items = (int64_t)S * H;
    if (items >= 4 * (int64_t)cus || max_context_len <= 512) return 0;
    const int64_t want_parts = (4 * (int64_t)cus + items - 1) / items;
    int64_t ps = (max_context_len + want_parts - 1) / want_parts;
    ps = ((ps + 255) / 256) * 256;
    if (ps < 512) ps = 512;
    return ps >= max_context_len ? 0 : (int)ps;
}

template <int DT>
bool launch_multi(const DecodeArgs &a, int B, unsigned blocks)
{
    constexpr int W = 4;   // 16 query rows of partial results per wave: four waves fill 32 KiB of LDS
    switch (B) {
    case 16: hipLaunchKernelGGL((pa_decode_multi_kernel<DT, 16, W>), dim3(blocks), dim3(W * kWave), 0, a.stream, a.p); return true;
    case 32: hipLaunchKernelGGL((pa_decode_multi_kernel<DT, 32, W>), dim3(blocks), dim3(W * kWave), 0, a.stream, a.p); return true;
    case 64: hipLaunchKernelGGL((pa_decode_multi_kernel<DT, 64, W>), dim3(blocks), dim3(W * kWave), 0, a.stream, a.p); return true;
    case 128: hipLaunchKernelGGL((pa_decode_multi_kernel<DT, 128, W>), dim3(blocks), dim3(W * kWave), 0, a.stream, a.p); return true;
    }
    return false;
}

void fill_common(DecodeArgs &a, void *out, const void *q, const void *k_cache, const void *v_cache,
                 const int32_t *block_tables, int32_t max_blocks, const int32_t *context_lens, int32_t S,
                 int32_t H, float scale, void *stream)
{
    a.p.out = out;
    a.p.q = q;
    a.p.k_cache = static_cast<const char *>(k_cache);
    a.p.v_cache = static_cast<const char *>(v_cache);
    a.p.block_tables = block_tables;
    a.p.max_blocks = max_blocks;
    a.p.context_lens = context_lens;
    a.p.S = S;
    a.p.H = H;
    a.p.scale_log2 = scale * kLog2e;
    a.stream = static_cast<hipStream_t>(stream);
}

} // namespace

extern "C" {

int pa_version(void) { return 1; }

const char *pa_status_string(pa_status st)
{
    switch (st) {
    case PA_OK: return "ok";
    case PA_ERR_NULL: return "null pointer";
    case PA_ERR_SHAPE: return "bad shape or size";
    case PA_ERR_UNSUPPORTED: return "unsupported dtype / head_dim / block_size";
    case PA_ERR_ALIGN: return "pointer not 16-byte aligned";
    case PA_ERR_WORKSPACE: return "workspace missing or too small";
    case PA_ERR_HIP: return "HIP runtime error";
    case PA_ERR_INVALID: return "invalid index found by pa_debug_validate";
    }
    return "unknown status";
}

size_t pa_decode_workspace_bytes(int32_t num_seqs, int32_t num_heads, int32_t head_dim,
                                 int32_t block_size, int32_t max_context_len, int32_t partition_size)
{
    if (num_seqs <= 0 || num_heads <= 0 || head_dim <= 0 || block_size <= 0 || max_context_len <= 0) return 0;
    if (partition_size == PA_PARTITION_AUTO) partition_size = auto_partition(num_seqs, num_heads, max_context_len);
    if (partition_size <= 0 || partition_size >= max_context_len) return 0;
    const size_t parts = (size_t)((max_context_len + partition_size - 1) / partition_size);
    return (size_t)num_seqs * num_heads * parts * ((size_t)head_dim + 2) * sizeof(float);
}

pa_status pa_decode(void *out, const void *q, const void *k_cache, const void *v_cache,
                    const int32_t *block_tables, int32_t max_blocks_per_seq,
                    const int32_t *context_lens, int32_t num_seqs, int32_t num_heads,
                    int32_t head_dim, int32_t block_size, int64_t num_blocks, pa_dtype dtype,
                    float scale, int32_t max_context_len, int32_t partition_size, void *workspace,
                    size_t workspace_bytes, void *stream)
{
    if (num_seqs < 0 || num_heads <= 0 || head_dim <= 0 || block_size <= 0 || num_blocks <= 0 ||
        max_blocks_per_seq <= 0 || max_context_len < 0)
        return PA_ERR_SHAPE;
    if (!shape_supported(dtype, head_dim, block_size)) return PA_ERR_UNSUPPORTED;
    if ((int64_t)max_context_len > (int64_t)max_blocks_per_seq * block_size) return PA_ERR_SHAPE;
    if (partition_size < PA_PARTITION_AUTO) return PA_ERR_SHAPE;
    if (partition_size > 0 && partition_size % block_size) return PA_ERR_SHAPE;
    if (num_seqs == 0) return PA_OK;
    if (!out || !q || !k_cache || !v_cache || !block_tables || !context_lens) return PA_ERR_NULL;
    if (!aligned16(out) || !aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache)) return PA_ERR_ALIGN;
    if ((int64_t)num_seqs * num_heads > (int64_t)0x7fffffff / 64) return PA_ERR_SHAPE;

    if (partition_size == PA_PARTITION_AUTO)
        partition_size = workspace ? auto_partition(num_seqs, num_heads, max_context_len) : 0;
    if (partition_size >= max_context_len) partition_size = 0;   // one range: plain single pass

    DecodeArgs a;
    memset(&a, 0, sizeof(a));
    fill_common(a, out, q, k_cache, v_cache, block_tables, max_blocks_per_seq, context_lens, num_seqs,
                num_heads, scale, stream);
    a.p.partition_size = partition_size;
    a.p.max_parts = 1;
    a.waves = waves_for(partition_size > 0 ? partition_size : max_context_len,
                        chunk_tokens(dtype, head_dim, block_size));
    if (partition_size > 0) {
        a.p.max_parts = (max_context_len + partition_size - 1) / partition_size;
        const size_t need = pa_decode_workspace_bytes(num_seqs, num_heads, head_dim, block_size,
                                                      max_context_len, partition_size);
        if (!workspace || workspace_bytes < need) return PA_ERR_WORKSPACE;
        if (!aligned16(workspace)) return PA_ERR_ALIGN;
        if ((int64_t)num_seqs * num_heads * a.p.max_parts > 0x7fffffff) return PA_ERR_SHAPE;
        a.p.ws_acc = static_cast<float *>(workspace);
        a.p.ws_ml = a.p.ws_acc + (size_t)num_seqs * num_heads * a.p.max_parts * head_dim;
    }
    if (!dispatch_decode(a, dtype, head_dim, block_size, partition_size > 0 ? MODE_PART : MODE_SINGLE))
        return PA_ERR_UNSUPPORTED;
    return hipGetLastError() == hipSuccess ? PA_OK : PA_ERR_HIP;
}

size_t pa_decode_shared_workspace_bytes(int32_t num_seqs, int32_t num_heads, int32_t head_dim)
{
    if (num_seqs <= 0 || num_heads <= 0 || head_dim <= 0) return 0;
    const size_t partials = (size_t)num_seqs * num_heads * 2 * ((size_t)head_dim + 2) * sizeof(float);
    return partials + ((ginfo_words(num_seqs) * sizeof(int32_t) + 15) & ~(size_t)15);
}

pa_status pa_decode_shared(void *out, const void *q, const void *k_cache, const void *v_cache,
                           const int32_t *block_tables, int32_t max_blocks_per_seq,
                           const int32_t *context_lens, int32_t num_seqs, int32_t num_heads,
                           int32_t head_dim, int32_t block_size, int64_t num_blocks, pa_dtype dtype,
                           float scale, int32_t max_context_len, void *workspace,
                           size_t workspace_bytes, void *stream)
{
    if (num_seqs < 0 || num_heads <= 0 || head_dim <= 0 || block_size <= 0 || num_blocks <= 0 ||
        max_blocks_per_seq <= 0 || max_context_len < 0)
        return PA_ERR_SHAPE;
    if (!shape_supported(dtype, head_dim, block_size)) return PA_ERR_UNSUPPORTED;
    if ((int64_t)max_context_len > (int64_t)max_blocks_per_seq * block_size) return PA_ERR_SHAPE;
    if (num_seqs == 0) return PA_OK;
    if (!out || !q || !k_cache || !v_cache || !block_tables || !context_lens) return PA_ERR_NULL;
    if (!aligned16(out) || !aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache)) return PA_ERR_ALIGN;
    if ((int64_t)num_seqs * num_heads > (int64_t)0x7fffffff / 64) return PA_ERR_SHAPE;
    const size_t need = pa_decode_shared_workspace_bytes(num_seqs, num_heads, head_dim);
    if (!workspace || workspace_bytes < need) return PA_ERR_WORKSPACE;
    if (!aligned16(workspace)) return PA_ERR_ALIGN;

    DecodeArgs a;
    memset(&a, 0, sizeof(a));
    fill_common(a, out, q, k_cache, v_cache, block_tables, max_blocks_per_seq, context_lens, num_seqs,
                num_heads, scale, stream);
    a.p.max_parts = 2;
    a.waves = waves_for(max_context_len, chunk_tokens(dtype, head_dim, block_size));
    const size_t rows2 = (size_t)num_seqs * num_heads * 2;
    a.p.ws_acc = static_cast<float *>(workspace);
    a.p.ws_ml = a.p.ws_acc + rows2 * head_dim;
    a.p.ginfo = reinterpret_cast<const int32_t *>(a.p.ws_ml + rows2 * 2);
    if (!dispatch_decode(a, dtype, head_dim, block_size, MODE_PREFIX)) return PA_ERR_UNSUPPORTED;
    return hipGetLastError() == hipSuccess ? PA_OK : PA_ERR_HIP;
}

pa_status pa_decode_multi(void *out, const void *q, const void *k_cache, const void *v_cache,
                          const int32_t *block_tables, int32_t max_blocks_per_seq,
                          const int32_t *context_lens, const int32_t *q_start, int32_t num_seqs,
                          int32_t max_q_len, int32_t num_heads, int32_t head_dim, int32_t block_size,
                          int64_t num_blocks, pa_dtype dtype, float scale, int32_t max_context_len,
                          void *stream)
{
    if (num_seqs < 0 || num_heads <= 0 || head_dim <= 0 || block_size <= 0 || num_blocks <= 0 ||
        max_blocks_per_seq <= 0 || max_context_len < 0 || max_q_len < 0)
        return PA_ERR_SHAPE;
    if ((dtype != PA_F16 && dtype != PA_BF16) || head_dim != 128 || block_size % 16 ||
        !shape_supported(dtype, head_dim, block_size))
        return PA_ERR_UNSUPPORTED;
    if ((int64_t)max_context_len > (int64_t)max_blocks_per_seq * block_size) return PA_ERR_SHAPE;
    if (num_seqs == 0 || max_q_len == 0) return PA_OK;
    if (!out || !q || !k_cache || !v_cache || !block_tables || !context_lens || !q_start) return PA_ERR_NULL;
    if (!aligned16(out) || !aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache)) return PA_ERR_ALIGN;
    const int64_t q_blocks = (max_q_len + 15) / 16;
    const int64_t blocks = (int64_t)num_seqs * q_blocks * num_heads;
    if (blocks > 0x7fffffff) return PA_ERR_SHAPE;
    DecodeArgs a;
    memset(&a, 0, sizeof(a));
    fill_common(a, out, q, k_cache, v_cache, block_tables, max_blocks_per_seq, context_lens, num_seqs,
                num_heads, scale, stream);
    a.p.q_start = q_start;
    a.p.q_blocks = (int32_t)q_blocks;
    const bool ok = dtype == PA_F16 ? launch_multi<PA_F16>(a, block_size, (unsigned)blocks)
                                    : launch_multi<PA_BF16>(a, block_size, (unsigned)blocks);
    if (!ok) return PA_ERR_UNSUPPORTED;
    return hipGetLastError() == hipSuccess ? PA_OK : PA_ERR_HIP;
}

pa_status pa_reshape_and_cache(const void *k, const void *v, void *k_cache, void *v_cache,
                               const int64_t *slot_mapping, int32_t num_tokens, int32_t num_heads,
                               int32_t head_dim, int32_t block_size, int64_t num_blocks,
                               pa_dtype dtype, void *stream)
{
    if (num_tokens < 0 || num_heads <= 0 || head_dim <= 0 || block_size <= 0 || num_blocks <= 0)
        return PA_ERR_SHAPE;
    if (dtype != PA_F32 && dtype != PA_F16 && dtype != PA_BF16) return PA_ERR_UNSUPPORTED;
    const int row_bytes = head_dim * elem_bytes(dtype);
    if (row_bytes % 16) return PA_ERR_UNSUPPORTED;
    if (num_tokens == 0) return PA_OK;
    if (!k || !v || !k_cache || !v_cache || !slot_mapping) return PA_ERR_NULL;
    if (!aligned16(k) || !aligned16(v) || !aligned16(k_cache) || !aligned16(v_cache)) return PA_ERR_ALIGN;
    const int32_t frags_per_row = row_bytes / 16;
    const int64_t frags_per_token = (int64_t)frags_per_row * num_heads;
    if (frags_per_token > 0x7fffffff) return PA_ERR_SHAPE;
    const int64_t total = frags_per_token * num_tokens;
    const int64_t groups = (total + 255) / 256;
    if (groups > 0x7fffffff) return PA_ERR_SHAPE;
    hipLaunchKernelGGL(reshape_and_cache_kernel, dim3((unsigned)groups, 2), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const uint4 *>(k),
                       static_cast<const uint4 *>(v), static_cast<uint4 *>(k_cache),
                       static_cast<uint4 *>(v_cache), slot_mapping, total, (int32_t)frags_per_token,
                       frags_per_row, block_size);
    return hipGetLastError() == hipSuccess ? PA_OK : PA_ERR_HIP;
}

pa_status pa_copy_blocks(void *const *k_caches, void *const *v_caches, int32_t num_layers,
                         const int64_t *src_dst_pairs, int32_t num_pairs, int32_t num_heads,
                         int32_t head_dim, int32_t block_size, int64_t num_blocks, pa_dtype dtype,
                         void *stream)
{
    if (num_layers <= 0 || num_pairs < 0 || num_heads <= 0 || head_dim <= 0 || block_size <= 0 ||
        num_blocks <= 0)
        return PA_ERR_SHAPE;
    if (dtype != PA_F32 && dtype != PA_F16 && dtype != PA_BF16) return PA_ERR_UNSUPPORTED;
    const int64_t block_bytes = (int64_t)num_heads * block_size * head_dim * elem_bytes(dtype);
    if (block_bytes % 16) return PA_ERR_UNSUPPORTED;
    if (num_pairs == 0) return PA_OK;
    if (!k_caches || !v_caches || !src_dst_pairs) return PA_ERR_NULL;
    for (int l = 0; l < num_layers; ++l) {
        if (!k_caches[l] || !v_caches[l]) return PA_ERR_NULL;
        if (!aligned16(k_caches[l]) || !aligned16(v_caches[l])) return PA_ERR_ALIGN;
    }
    const int64_t frags = block_bytes / 16;
    const unsigned slices = (unsigned)((frags + 255) / 256);
    for (int l0 = 0; l0 < num_layers; l0 += kMaxCopyPtrs / 2) {
        const int nl = num_layers - l0 < kMaxCopyPtrs / 2 ? num_layers - l0 : kMaxCopyPtrs / 2;
        CachePtrs ptrs;
        memset(&ptrs, 0, sizeof(ptrs));
        for (int l = 0; l < nl; ++l) {
            ptrs.p[2 * l] = static_cast<uint4 *>(k_caches[l0 + l]);
            ptrs.p[2 * l + 1] = static_cast<uint4 *>(v_caches[l0 + l]);
        }
        for (int p0 = 0; p0 < num_pairs; p0 += kMaxPairsPerLaunch) {
            const int np = num_pairs - p0 < kMaxPairsPerLaunch ? num_pairs - p0 : kMaxPairsPerLaunch;
            hipLaunchKernelGGL(copy_blocks_kernel, dim3(slices, (unsigned)np, (unsigned)(2 * nl)), dim3(256), 0,
                               static_cast<hipStream_t>(stream), ptrs, src_dst_pairs + 2 * (int64_t)p0, frags);
            if (hipGetLastError() != hipSuccess) return PA_ERR_HIP;
        }
    }
    return PA_OK;
}

pa_status pa_swap_blocks(void *const *src_k_caches, void *const *src_v_caches,
                         void *const *dst_k_caches, void *const *dst_v_caches, int32_t num_layers,
                         const int64_t *src_dst_pairs, int32_t num_pairs, int32_t num_heads,
                         int32_t head_dim, int32_t block_size, int64_t src_num_blocks,
                         int64_t dst_num_blocks, pa_dtype dtype, void *stream)
{
    if (num_layers <= 0 || num_pairs < 0 || num_heads <= 0 || head_dim <= 0 || block_size <= 0 ||
        src_num_blocks <= 0 || dst_num_blocks <= 0)
        return PA_ERR_SHAPE;
    if (dtype != PA_F32 && dtype != PA_F16 && dtype != PA_BF16) return PA_ERR_UNSUPPORTED;
    const int64_t block_bytes = (int64_t)num_heads * block_size * head_dim * elem_bytes(dtype);
    if (block_bytes % 16) return PA_ERR_UNSUPPORTED;
    if (num_pairs == 0) return PA_OK;
    if (!src_k_caches || !src_v_caches || !dst_k_caches || !dst_v_caches || !src_dst_pairs) return PA_ERR_NULL;
    for (int l = 0; l < num_layers; ++l) {
        if (!src_k_caches[l] || !src_v_caches[l] || !dst_k_caches[l] || !dst_v_caches[l]) return PA_ERR_NULL;
        if (!aligned16(src_k_caches[l]) || !aligned16(src_v_caches[l]) || !aligned16(dst_k_caches[l]) ||
            !aligned16(dst_v_caches[l]))
            return PA_ERR_ALIGN;
    }
    const int64_t frags = block_bytes / 16;
    const unsigned slices = (unsigned)((frags + 255) / 256);
    for (int l0 = 0; l0 < num_layers; l0 += kMaxSwapLayers) {
        const int nl = num_layers - l0 < kMaxSwapLayers ? num_layers - l0 : kMaxSwapLayers;
        SwapPtrs ptrs;
        memset(&ptrs, 0, sizeof(ptrs));
        for (int l = 0; l < nl; ++l) {
            ptrs.src[2 * l] = static_cast<const uint4 *>(src_k_caches[l0 + l]);
            ptrs.src[2 * l + 1] = static_cast<const uint4 *>(src_v_caches[l0 + l]);
            ptrs.dst[2 * l] = static_cast<uint4 *>(dst_k_caches[l0 + l]);
            ptrs.dst[2 * l + 1] = static_cast<uint4 *>(dst_v_caches[l0 + l]);
        }
        for (int p0 = 0; p0 < num_pairs; p0 += kMaxPairsPerLaunch) {
            const int np = num_pairs - p0 < kMaxPairsPerLaunch ? num_pairs - p0 : kMaxPairsPerLaunch;
            hipLaunchKernelGGL(swap_blocks_kernel, dim3(slices, (unsigned)np, (unsigned)(2 * nl)), dim3(256), 0,
                               static_cast<hipStream_t>(stream), ptrs, src_dst_pairs + 2 * (int64_t)p0, frags);
            if (hipGetLastError() != hipSuccess) return PA_ERR_HIP;
        }
    }
    return PA_OK;
}

pa_status pa_debug_validate(const int32_t *block_tables, int32_t max_blocks_per_seq,
                            const int32_t *context_lens, int32_t num_seqs, int32_t max_context_len,
                            const int64_t *slot_mapping, int32_t num_tokens,
                            const int64_t *src_dst_pairs, int32_t num_pairs, int32_t block_size,
                            int64_t num_blocks, void *stream)
{
    if (block_size <= 0 || num_blocks <= 0 || num_seqs < 0 || num_tokens < 0 || num_pairs < 0)
        return PA_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    pa_status result = PA_OK;
    if (block_tables && context_lens && num_seqs > 0) {
        if (max_blocks_per_seq <= 0) return PA_ERR_SHAPE;
        const size_t nt = (size_t)num_seqs * max_blocks_per_seq;
        int32_t *tab = static_cast<int32_t *>(malloc(nt * sizeof(int32_t)));
        int32_t *len = static_cast<int32_t *>(malloc((size_t)num_seqs * sizeof(int32_t)));
        if (!tab || !len) { free(tab); free(len); return PA_ERR_HIP; }
        bool ok = hipMemcpyAsync(tab, block_tables, nt * sizeof(int32_t), hipMemcpyDeviceToHost, st) == hipSuccess &&
                  hipMemcpyAsync(len, context_lens, (size_t)num_seqs * sizeof(int32_t), hipMemcpyDeviceToHost, st) == hipSuccess &&
                  hipStreamSynchronize(st) == hipSuccess;
        if (!ok) result = PA_ERR_HIP;
        for (int s = 0; ok && s < num_seqs && result == PA_OK; ++s) {
            const int64_t n = len[s];
            if (n < 0 || n > max_context_len || n > (int64_t)max_blocks_per_seq * block_size) { result = PA_ERR_INVALID; break; }
            const int64_t nb = (n + block_size - 1) / block_size;
            for (int64_t j = 0; j < nb; ++j) {
                const int64_t pb = tab[(size_t)s * max_blocks_per_seq + j];
                if (pb < 0 || pb >= num_blocks) { result = PA_ERR_INVALID; break; }
            }
        }
        free(tab);
        free(len);
        if (result != PA_OK) return result;
    }
    if (slot_mapping && num_tokens > 0) {
        int64_t *sl = static_cast<int64_t *>(malloc((size_t)num_tokens * sizeof(int64_t)));
        if (!sl) return PA_ERR_HIP;
        bool ok = hipMemcpyAsync(sl, slot_mapping, (size_t)num_tokens * sizeof(int64_t), hipMemcpyDeviceToHost, st) == hipSuccess &&
                  hipStreamSynchronize(st) == hipSuccess;
        if (!ok) result = PA_ERR_HIP;
        const int64_t total = num_blocks * block_size;
        // duplicate detection with one bit per slot
        uint8_t *seen = ok ? static_cast<uint8_t *>(calloc((size_t)(total + 7) / 8, 1)) : nullptr;
        if (ok && !seen) result = PA_ERR_HIP;
        for (int t = 0; seen && t < num_tokens; ++t) {
            const int64_t x = sl[t];
            if (x < 0) continue;
            if (x >= total || (seen[x >> 3] >> (x & 7)) & 1) { result = PA_ERR_INVALID; break; }
            seen[x >> 3] |= (uint8_t)(1u << (x & 7));
        }
        free(seen);
        free(sl);
        if (result != PA_OK) return result;
    }
    if (src_dst_pairs && num_pairs > 0) {
        int64_t *pr = static_cast<int64_t *>(malloc((size_t)num_pairs * 2 * sizeof(int64_t)));
        if (!pr) return PA_ERR_HIP;
        bool ok = hipMemcpyAsync(pr, src_dst_pairs, (size_t)num_pairs * 2 * sizeof(int64_t), hipMemcpyDeviceToHost, st) == hipSuccess &&
                  hipStreamSynchronize(st) == hipSuccess;
        if (!ok) result = PA_ERR_HIP;
        uint8_t *role = ok ? static_cast<uint8_t *>(calloc((size_t)num_blocks, 1)) : nullptr;   // 1 = src, 2 = dst
        if (ok && !role) result = PA_ERR_HIP;
        for (int i = 0; role && i < num_pairs && result == PA_OK; ++i) {
            const int64_t src = pr[2 * i], dst = pr[2 * i + 1];
            if (src < 0 || src >= num_blocks || dst < 0 || dst >= num_blocks) { result = PA_ERR_INVALID; break; }
            if (role[dst] != 0 || role[src] == 2) { result = PA_ERR_INVALID; break; }
            role[src] = 1;
            role[dst] = 2;
        }
        free(role);
        free(pr);
    }
    return result;
}

pa_status pa_stream_read(const void *src, size_t bytes, void *sink, void *stream)
{
    if (!src || !sink) return PA_ERR_NULL;
    if (bytes == 0 || bytes % 16) return PA_ERR_SHAPE;
    if (!aligned16(src)) return PA_ERR_ALIGN;
    const int64_t frags = (int64_t)(bytes / 16);
    const int64_t groups = (frags + kProbeTileFrags - 1) / kProbeTileFrags;
    if (groups > 0x7fffffff) return PA_ERR_SHAPE;
    hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)groups), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const char *>(src), frags,
                       static_cast<uint32_t *>(sink));
    return hipGetLastError() == hipSuccess ? PA_OK : PA_ERR_HIP;
}

} // extern "C"
