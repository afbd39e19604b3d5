// libpa matrix-core bodies: shared prefixes of a group and several causal queries per sequence.
#ifndef PA_PA_MFMA_HPP
#define PA_PA_MFMA_HPP

#include "pa_decode.hpp"

namespace {

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


} // namespace

#endif
