// libpa paged decode: the VALU decode kernel (one pass or fixed partitions) and the merge kernel.
#ifndef PA_PA_DECODE_HPP
#define PA_PA_DECODE_HPP

#include "pa_common.hpp"

namespace {

// ---- decode ----------------------------------------------------------------
// One workgroup of W wavefronts serves one work item: a (sequence, head) over
// its whole context, or over one fixed-size partition of it.
//
// Lane roles: a token row is LPT = D*E/16 lanes wide, so one 1 KiB wavefront
// load covers TPL = 64/LPT consecutive tokens; lane = g*LPT + c holds
// dimensions [c*EPL, (c+1)*EPL) of token (base + g).  Work advances in chunks
// of LPC loads (CT = LPC*TPL tokens, at most one block); wave w takes chunks
// w, w+W, ...; the loads of U chunks (2*U*LPC KiB of K and V) are written
// together ahead of their use, and the compiler spreads them over the trip.
//
// Each group g of lanes runs its own online softmax over the tokens it sees
// (running maximum m, sum l, weighted V sum acc, all fp32, exponents in base
// 2 with log2(e) folded into the scale).  Groups and waves are merged once at
// the end with the log-sum-exp rule, so the inner loop has no cross-group
// traffic.  Summation order depends only on logical token positions, so the
// result does not change with the physical placement of blocks.
enum DecodeMode {
    MODE_SINGLE = 0,   // whole context, writes the output row
    MODE_PART = 1      // tokens [part*PS, (part+1)*PS), writes partial `part` of max_parts
};

struct DecodeParams {
    void *out;
    const void *q;
    const char *k_cache, *v_cache;
    const int32_t *block_tables;
    const int32_t *context_lens;
    const int32_t *ginfo;   // sharing plan of pa_decode_shared: group table (find_groups_kernel)
    const int4 *tiles;      // sharing plan: per-group tile lists (build_tiles_kernel)
    const int32_t *q_start; // multi-query path: first query row of every sequence, [S+1]
    float *ws_acc, *ws_ml;
    int32_t max_blocks, S, H;
    int32_t partition_size, max_parts;
    int32_t q_blocks;        // multi-query path: blocks of 64 queries per sequence in the grid
    float scale_log2;
};

// Sharing plan of pa_decode_shared.  The group table is 6 arrays of S int32 entries, two
// counters, and, from the next multiple of four words at or after word 6S + 4, S work items of
// four int32 each:
//   in_group[s]      1 if sequence s belongs to a group (two or more members), else 0
//   group_size[s]    members of the group whose first sequence is s (consecutive sequences
//                    s .. s + size - 1); 0 if no group starts at s
//   tile_count[s]    entries on the tile list of the group that starts at s (written only where a
//                    group starts; elsewhere undefined)
//   adj[s]           leading full blocks that s maps to the same physical blocks as s - 1
//   single_list[i]   the sequences outside any group, ascending, i < single_count
//   group_list[i]    first sequences of the groups, ascending, i < group_count
//   group_count, single_count
//   item[i]          what workgroup (i, head) of the decode launch does: (kind, first sequence,
//                    members, tile-list entries) with kind 2 = group (i < group_count, order of
//                    group_list), 1 = single sequence (the next single_count items, order of
//                    single_list), 0 = nothing (the rest: every group takes the place of two or
//                    more sequences)
// The tile list of the group that starts at s begins at entry s * max_blocks of the tile array
// (a group's members own that many entries between them).  It holds every physical block
// that a member maps, once per logical position, ordered by position:
//   x  physical block id
//   y  bits 0..15: members (bit j = sequence s + j) that map this block at this position;
//      bit 16: some member in the set sees only part of the tokens stored
//   z  logical block index (position / block_size)
//   w  tokens of the block that the longest member of the set sees (1 .. block_size)
constexpr int kGroupMax = 16;    // members of a group: one query column of the MFMA tiles each
__device__ __host__ __forceinline__ int ginfo_in_group(int S, int s) { (void)S; return s; }
__device__ __host__ __forceinline__ int ginfo_group_size(int S, int s) { return S + s; }
__device__ __host__ __forceinline__ int ginfo_tile_count(int S, int s) { return 2 * S + s; }
__device__ __host__ __forceinline__ int ginfo_adj(int S, int s) { return 3 * S + s; }
__device__ __host__ __forceinline__ int ginfo_single_list(int S, int i) { return 4 * S + i; }
__device__ __host__ __forceinline__ int ginfo_group_list(int S, int i) { return 5 * S + i; }
__device__ __host__ __forceinline__ int ginfo_group_count(int S) { return 6 * S; }
__device__ __host__ __forceinline__ int ginfo_single_count(int S) { return 6 * S + 1; }
// (items are 16-byte records: they start at the next multiple of four words)
__device__ __host__ __forceinline__ int ginfo_item(int S, int i) { return (6 * S + 4 + 3) / 4 * 4 + 4 * i; }
__device__ __host__ __forceinline__ size_t ginfo_words(int S) { return (size_t)ginfo_item(S, 0) + 4 * (size_t)S; }

// A sixteen-wave workgroup is kept alone on its compute unit (at most 7 waves
// per SIMD, so a second one does not fit): measured on batches of mixed
// lengths, two resident workgroups each run at half speed and stretch the end
// of the launch by more than their overlap gains.
#define PA_OCC_ATTR __attribute__((amdgpu_waves_per_eu(W == 16 ? 4 : 1, W == 16 ? 7 : 8)))

// One wave's share of tokens [t_begin, t_end) of sequence s against head h (t_begin < t_end,
// t_begin a multiple of the chunk size): the wave takes chunks wv, wv + nw, ... of the range.
// On return its lanes with g == 0 hold the running maximum m (log2 units), exp-sum l and
// unnormalised weighted V sum acc[] of those chunks for their EPL dimensions (m = -big, l = 0
// if it had none).
template <int DT, int D, int B, int U>
__device__ __forceinline__ void stream_range(const DecodeParams &P, const int s, const int h, const int t_begin,
                                             const int t_end, const int wv, const int nw, float &m, float &l,
                                             float (&acc)[Traits<DT>::EPL])
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

    const int lane = threadIdx.x & (kWave - 1);
    const int g = lane / LPT;
    const int c = lane % LPT;
    const uint32_t lane16 = (uint32_t)lane * 16u;
    const int H = P.H;

    const uint4 qf = reinterpret_cast<const uint4 *>(P.q)[((int64_t)s * H + h) * LPT + c];
    const int32_t *__restrict__ table = P.block_tables + (int64_t)s * P.max_blocks;
    const int nchunks = (t_end - t_begin + CT - 1) / CT;

    m = kNegBig;
    l = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;

    struct Chunk {
        uint4 k[LPC], v[LPC];
    };

    auto block_of = [&](int ci) -> int {
        // ci is wave-uniform: this is a scalar load
        return table[(t_begin + ci * CT) / B];
    };
    // TAIL is set only for a chunk that may reach past t_end (the last one): rows that hold no
    // token of the range are not fetched at all (with contexts of a few dozen tokens they would
    // be a tenth of the traffic) and read as zeros
    auto issue = [&](Chunk &ck, int ci, int pb, auto tail_tag) {
        constexpr bool TAIL = decltype(tail_tag)::value;
        const int t0 = t_begin + ci * CT;
        const int64_t off = ((int64_t)pb * H + h) * TILE_BYTES + (int64_t)(t0 % B) * ROW_BYTES;
        const char *kp = P.k_cache + off + lane16;
        const char *vp = P.v_cache + off + lane16;
#pragma unroll
        for (int i = 0; i < LPC; ++i) {
            ck.k[i] = make_uint4(0, 0, 0, 0);
            if (!TAIL || t0 + i * TPL + g < t_end) ck.k[i] = load16_stream(kp + i * 1024);
        }
#pragma unroll
        for (int i = 0; i < LPC; ++i) {
            ck.v[i] = make_uint4(0, 0, 0, 0);
            if (!TAIL || t0 + i * TPL + g < t_end) ck.v[i] = load16_stream(vp + i * 1024);
        }
    };
    // MASK is set only for a chunk that may reach past t_end (the last one)
    auto consume = [&](Chunk &ck, int ci, auto mask_tag) {
        constexpr bool MASK = decltype(mask_tag)::value;
        const int t0 = t_begin + ci * CT;
        float x[LPC];
#pragma unroll
        for (int i = 0; i < LPC; ++i) x[i] = group_sum<LPT>(Tr::dot(ck.k[i], qf, 0.f)) * P.scale_log2;
        if (MASK) {
            // slots at or past t_end hold no token and may contain anything, NaN
            // included - select them away, never multiply
#pragma unroll
            for (int i = 0; i < LPC; ++i) {
                const bool dead = t0 + i * TPL + g >= t_end;
                x[i] = dead ? -INFINITY : x[i];
                ck.v[i].x = dead ? 0u : ck.v[i].x;
                ck.v[i].y = dead ? 0u : ck.v[i].y;
                ck.v[i].z = dead ? 0u : ck.v[i].z;
                ck.v[i].w = dead ? 0u : ck.v[i].w;
            }
        }
        float m_new = m;
#pragma unroll
        for (int i = 0; i < LPC; ++i) m_new = fmaxf(m_new, x[i]);
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        float p[LPC], psum = 0.f;
#pragma unroll
        for (int i = 0; i < LPC; ++i) {
            p[i] = __builtin_amdgcn_exp2f(x[i] - m_new);
            psum += p[i];
        }
        l = l * alpha + psum;
        m = m_new;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] *= alpha;
#pragma unroll
        for (int i = 0; i < LPC; ++i) {
            Tr::axpy(acc, p[i], ck.v[i]);
            // bf16 widening is two VALU ops per pair; without a fence the
            // scheduler widens every fragment first and doubles the live registers
            if (Tr::FENCE_AXPY) __builtin_amdgcn_sched_barrier(0);
        }
    };
    const std::false_type full{};
    const std::true_type masked{};

    // Steady state: U chunks per trip in one straight-line block; nothing loaded is
    // carried across the back edge, so the compiler is free to place each load where
    // register pressure allows and waits exactly for the fragment it needs next.
    // Chunks before the last one of the range are full; the remainder loop takes
    // one chunk at a time with masking.  Latency is hidden by the other waves
    // resident on the SIMD.
    {
        int ci = wv;
        for (; ci + (U - 1) * nw <= nchunks - 2; ci += U * nw) {
            Chunk ck[U];
            int pb[U];
#pragma unroll
            for (int u = 0; u < U; ++u) pb[u] = block_of(ci + u * nw);
#pragma unroll
            for (int u = 0; u < U; ++u) issue(ck[u], ci + u * nw, pb[u], full);
#pragma unroll
            for (int u = 0; u < U; ++u) consume(ck[u], ci + u * nw, full);
        }
        for (; ci < nchunks; ci += nw) {
            Chunk ck;
            issue(ck, ci, block_of(ci), masked);
            consume(ck, ci, masked);
        }
    }

    // merge the TPL token groups of this wave (lanes with equal c)
    {
        float M = m;
#pragma unroll
        for (int d = LPT; d < kWave; d <<= 1) M = fmaxf(M, __shfl_xor(M, d));
        const float f = __builtin_amdgcn_exp2f(m - M);
        l *= f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] *= f;
#pragma unroll
        for (int d = LPT; d < kWave; d <<= 1) {
            l += __shfl_xor(l, d);
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] += __shfl_xor(acc[e], d);
        }
        m = M;
    }

}

// Tokens [t_begin, t_end) of sequence s against head h with all W waves of the workgroup: on
// return wave 0's lanes with g == 0 hold m, l and acc[] of the whole range; other lanes hold
// nothing useful.  Every wave of the workgroup must call it (it synchronises those with work),
// and must not meet another workgroup barrier afterwards: waves without work have gone.
template <int DT, int D, int B, int W, int U>
__device__ __forceinline__ void decode_range(const DecodeParams &P, const int s, const int h, const int t_begin,
                                             const int t_end, float &m, float &l,
                                             float (&acc)[Traits<DT>::EPL])
{
    using Tr = Traits<DT>;
    constexpr int EPL = Tr::EPL;
    constexpr int LPT = D * Tr::E / 16;
    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int g = lane / LPT;
    const int c = lane % LPT;
    // A range shorter than W chunks leaves waves without work.  They leave at once (a barrier waits
    // for the surviving waves of a workgroup only), so that their slots are free for the next
    // workgroup while this one's few busy waves stream: a launch is planned from its longest
    // context, and in a batch of mixed lengths most items are much shorter.
    constexpr int TPL = kWave / LPT, LPC = (B / TPL) < 4 ? (B / TPL) : 4, CT = LPC * TPL;   // as in stream_range
    const int nchunks = (t_end - t_begin + CT - 1) / CT;
    const int active = nchunks < W ? nchunks : W;
    if (w >= active) {
        m = kNegBig;
        l = 0.f;
        return;
    }
    stream_range<DT, D, B, U>(P, s, h, t_begin, t_end, w, W, m, l, acc);

    // merge the busy waves of the workgroup through LDS
    if (W > 1) {
        __shared__ float sm_acc[W][D];
        __shared__ float sm_m[W], sm_l[W];
        if (g == 0) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) sm_acc[w][c * EPL + e] = acc[e];
            if (c == 0) {
                sm_m[w] = m;
                sm_l[w] = l;
            }
        }
        __syncthreads();
        if (w != 0) return;
        float M;
        auto merge = [&](const int nb) {
            M = sm_m[0];
#pragma unroll
            for (int i = 1; i < nb; ++i) M = fmaxf(M, sm_m[i]);
            l = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
            // (not fully unrolled: sixteen waves' worth of LDS reads hoisted at once would spill)
#pragma unroll 2
            for (int i = 0; i < nb; ++i) {
                const float f = __builtin_amdgcn_exp2f(sm_m[i] - M);
                l = __builtin_fmaf(sm_l[i], f, l);
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[e] = __builtin_fmaf(sm_acc[i][c * EPL + e], f, acc[e]);
            }
        };
        // (the usual case with its loop bounds known at compile time)
        if (active == W)
            merge(W);
        else
            merge(active);
        m = M;
    }
}

// One work item of the decode kernel: a (sequence, head) over its whole context, or over one
// fixed-size partition of it.
template <int DT, int D, int B, int W, int U, int MODE>
__device__ __forceinline__ void decode_body(const DecodeParams &P, const int s, const int h, const int part)
{
    using Tr = Traits<DT>;
    constexpr int EPL = Tr::EPL;
    constexpr int LPT = D * Tr::E / 16;
    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int g = lane / LPT;
    const int c = lane % LPT;
    const int H = P.H;
    const int n = P.context_lens[s];
    const int t_begin = MODE == MODE_PART ? part * P.partition_size : 0;
    const int t_end = MODE == MODE_PART ? (t_begin + P.partition_size < n ? t_begin + P.partition_size : n) : n;
    if (t_begin >= t_end) {
        if (MODE == MODE_SINGLE && w == 0 && g == 0) {
            // empty context: zero row
            reinterpret_cast<uint4 *>(P.out)[((int64_t)s * H + h) * LPT + c] = make_uint4(0, 0, 0, 0);
        }
        return;
    }

    float m, l, acc[EPL];
    decode_range<DT, D, B, W, U>(P, s, h, t_begin, t_end, m, l, acc);
    if (w != 0 || g != 0) return;

    if (MODE == MODE_SINGLE) {
        const float inv = 1.0f / l;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] *= inv;
        reinterpret_cast<uint4 *>(P.out)[((int64_t)s * H + h) * LPT + c] = Tr::pack(acc);
    } else {
        // unnormalised partial: the reduce kernel divides once
        const int64_t slot = ((int64_t)s * H + h) * P.max_parts + part;
        float *dst = P.ws_acc + slot * D + c * EPL;
#pragma unroll
        for (int e = 0; e < EPL; e += 4)
            *reinterpret_cast<float4 *>(dst + e) = make_float4(acc[e], acc[e + 1], acc[e + 2], acc[e + 3]);
        if (c == 0) *reinterpret_cast<float2 *>(P.ws_ml + slot * 2) = make_float2(m, l);
    }
}

template <int DT, int D, int B, int W, int U, int MODE>
__global__ __launch_bounds__(W *kWave) PA_OCC_ATTR void pa_decode_kernel(const DecodeParams P)
{
    // grid index: head fastest, then sequence, then partition - the heads of a sequence start
    // together and read neighbouring tiles, and the (sequence, partition) pairs past a sequence's
    // end, which only exit, gather towards the end of the launch
    int item = (int)blockIdx.x;
    const int h = item % P.H;
    item /= P.H;
    const int s = item % P.S;
    const int part = item / P.S;
    decode_body<DT, D, B, W, U, MODE>(P, s, h, part);
}

// Merge of the split-context partials: out = sum_p 2^(m_p-M) a_p / sum_p 2^(m_p-M) l_p
// with a_p the unnormalised partial sums.  A (sequence, head) row takes LPT lanes (lane c
// handles the same 16-byte output fragment as in the decode kernel), so a wavefront merges
// 64 / LPT rows and a workgroup of four wavefronts four times that.
constexpr int kReduceWaves = 4;
template <int DT, int D>
__global__ __launch_bounds__(kReduceWaves *kWave) void pa_reduce_kernel(const DecodeParams P)
{
    using Tr = Traits<DT>;
    constexpr int EPL = Tr::EPL;
    constexpr int LPT = D * Tr::E / 16;
    constexpr int ROWS = kReduceWaves * kWave / LPT;      // rows per workgroup
    const int c = threadIdx.x % LPT;
    const int64_t row = (int64_t)blockIdx.x * ROWS + threadIdx.x / LPT;
    const int H = P.H;
    if (row >= (int64_t)P.S * H) return;
    const int s = (int)(row / H);
    const int n = P.context_lens[s];
    int parts = (n + P.partition_size - 1) / P.partition_size;
    if (parts > P.max_parts) parts = P.max_parts;
    const int64_t base = row * P.max_parts;
    float acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
    if (parts > 0) {
        float M = kNegBig;
        for (int p = 0; p < parts; ++p) M = fmaxf(M, P.ws_ml[(base + p) * 2]);
        float l = 0.f;
        for (int p = 0; p < parts; ++p) {
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
    reinterpret_cast<uint4 *>(P.out)[row * LPT + c] = Tr::pack(acc);
}

} // namespace

#endif
