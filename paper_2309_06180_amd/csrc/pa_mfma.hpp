// libpa matrix-core tile engine (several queries against one K/V tile) and the kernels built on it:
// several causal queries per sequence, and groups of sequences that share blocks.
#ifndef PA_PA_MFMA_HPP
#define PA_PA_MFMA_HPP

#include "pa_decode.hpp"

namespace {

typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));

// ---- the tile engine for gfx950 ---------------------------------------------
// One step of attention for up to 16 queries against one 16-token K/V tile that sits in
// LDS, with the matrix instructions of CDNA4 (k = 32) and its transposing LDS read.
//
// A wave owns 16 query columns: lane l = 16g + c holds query c.
//   S^T = K Q^T   4 x v_mfma_f32_16x16x32: A = K (lane: token row c, 16 bytes of it per step,
//                 ds_read_b128 out of the padded LDS tile), B = Q^T (lane: query c, the same
//                 byte ranges of the query row, kept in registers).  Result: lane holds
//                 tokens 4g .. 4g+3 of query c.
//   softmax       per query, running maximum and sum kept in the lane (replicated over g);
//                 two cross-lane maxima per tile, by v_permlane16_swap / v_permlane32_swap.
//   O^T += V^T P^T  8 x v_mfma_f32_16x16x32: B = P^T (lane: query c), A = V^T (lane: head
//                 dimension 16e + c, four tokens 4g .. 4g+3 fetched with one
//                 ds_read_b64_tr_b16).  The result keeps query c in lane c, so rescaling
//                 the output when a maximum moves needs no cross-lane traffic.
// A 16-bit P would eat the tolerance, so P is cut into two 16-bit pieces whose sum is P to
// 2^-18 (bf16, both pieces rounded to nearest) or 2^-21 (f16, with a factor 2^14 that keeps
// small weights in range).  The contraction of the PV instruction is 32 deep and the tile
// has 16 tokens: slots 8g + 0..3 carry the leading pieces and slots 8g + 4..7 the trailing
// pieces of tokens 4g .. 4g+3 against the same V values, so one instruction applies both.
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2v_t __attribute__((ext_vector_type(2)));

constexpr int kTileTokens = 16;
constexpr int kKPitch = 256 + 16;   // 16 rows of one ds_read_b128 fall in 16 different bank groups
constexpr int kVPitch = 256 + 32;   // 8 rows of one half-wave transposing read likewise
constexpr int kTileLds = kTileTokens * (kKPitch + kVPitch);   // K tile, then V tile

template <int DT>
__device__ __forceinline__ float4_t mfma_k32(const uint4 &a, const uint4 &b, float4_t c)
{
    if (DT == PA_F16)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, a),
                                                      __builtin_bit_cast(half8_t, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                       __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// maximum / sum over the four lanes that hold the same query (l, l^16, l^32, l^48)
__device__ __forceinline__ float quad_rows_max(float x)
{
    auto a = __builtin_amdgcn_permlane16_swap(as_u32(x), as_u32(x), false, false);
    x = fmaxf(as_f32(a[0]), as_f32(a[1]));
    auto b = __builtin_amdgcn_permlane32_swap(as_u32(x), as_u32(x), false, false);
    return fmaxf(as_f32(b[0]), as_f32(b[1]));
}
__device__ __forceinline__ float quad_rows_sum(float x)
{
    auto a = __builtin_amdgcn_permlane16_swap(as_u32(x), as_u32(x), false, false);
    x = as_f32(a[0]) + as_f32(a[1]);
    auto b = __builtin_amdgcn_permlane32_swap(as_u32(x), as_u32(x), false, false);
    return as_f32(b[0]) + as_f32(b[1]);
}

// the four weights of a lane as the B operand: leading pieces in slots 0..3, trailing in 4..7
template <int DT>
__device__ __forceinline__ uint4 weight_operand(const float (&p)[4])
{
    uint4 o;
    if (DT == PA_F16) {
        typedef _Float16 half2v __attribute__((ext_vector_type(2)));
        const float a0 = p[0] * 16384.0f, a1 = p[1] * 16384.0f, a2 = p[2] * 16384.0f, a3 = p[3] * 16384.0f;
        const half2v h01 = __builtin_bit_cast(half2v, __builtin_amdgcn_cvt_pkrtz(a0, a1));
        const half2v h23 = __builtin_bit_cast(half2v, __builtin_amdgcn_cvt_pkrtz(a2, a3));
        o.x = __builtin_bit_cast(uint32_t, h01);
        o.y = __builtin_bit_cast(uint32_t, h23);
        o.z = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(a0 - (float)h01.x, a1 - (float)h01.y));
        o.w = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(a2 - (float)h23.x, a3 - (float)h23.y));
    } else {
        // v_cvt_pk_bf16_f32 rounds to nearest even
        typedef float float2v __attribute__((ext_vector_type(2)));
        const uint32_t h01 = __builtin_bit_cast(uint32_t, __builtin_convertvector(float2v{p[0], p[1]}, bf16x2v_t));
        const uint32_t h23 = __builtin_bit_cast(uint32_t, __builtin_convertvector(float2v{p[2], p[3]}, bf16x2v_t));
        const float2v r01 = {p[0] - as_f32(h01 << 16), p[1] - as_f32(h01 & 0xffff0000u)};
        const float2v r23 = {p[2] - as_f32(h23 << 16), p[3] - as_f32(h23 & 0xffff0000u)};
        o.x = h01;
        o.y = h23;
        o.z = __builtin_bit_cast(uint32_t, __builtin_convertvector(r01, bf16x2v_t));
        o.w = __builtin_bit_cast(uint32_t, __builtin_convertvector(r23, bf16x2v_t));
    }
    return o;
}

// query-side state of a wave
struct QueryCols {
    uint4 qf[4];       // Q^T operand: bytes [64cc + 16g, +16) of the row of query c
    float4_t O[8];     // O^T: O[e][v] = output dimension 16e + 4g + v of query c (unnormalised)
    float m, lsum;     // running maximum (log2 units); exp-sum over this lane's tokens
    int limit;         // last token position query c sees; -1 if column c holds no query
};

template <int DT>
__device__ __forceinline__ void query_cols_init(QueryCols &Q, const void *q, int64_t row, int H, int h, bool present,
                                                int limit)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int g = lane / 16;
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) {
        Q.qf[cc] = make_uint4(0, 0, 0, 0);
        if (present)
            Q.qf[cc] = *reinterpret_cast<const uint4 *>(static_cast<const char *>(q) + (row * H + h) * 256 + 64 * cc + 16 * g);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) Q.O[e] = float4_t{0.f, 0.f, 0.f, 0.f};
    Q.m = kNegBig;
    Q.lsum = 0.f;
    Q.limit = present ? limit : -1;
}

// One tile: kt / vt point at the K and V tile in LDS (rows kKPitch / kVPitch apart), its first
// token is position t0; `mask` = query columns that map the tile; `check` = some entry may
// need masking (a column outside the mask, or a token past a query's limit).  V rows that
// hold no token any query sees must be zeros (whoever fills the tile does not fetch them).
template <int DT>
__device__ __forceinline__ void tile_step(QueryCols &Q, const char *kt, const char *vt, int t0, uint32_t mask,
                                          bool check, float scale_log2)
{
    typedef short4_t __attribute__((address_space(3))) *lds_tr_ptr;
    const int lane = threadIdx.x & (kWave - 1);
    const int g = lane / 16, c = lane % 16;
    uint4 kf[4];
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) kf[cc] = *reinterpret_cast<const uint4 *>(kt + c * kKPitch + 16 * g + 64 * cc);
    float4_t S = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) S = mfma_k32<DT>(kf[cc], Q.qf[cc], S);
    float x[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) x[v] = S[v] * scale_log2;
    if (check) {
        // by select, never by multiplying: rows past the stored tokens may hold anything
        const bool mine = (mask >> c) & 1u;
#pragma unroll
        for (int v = 0; v < 4; ++v) x[v] = (mine && t0 + 4 * g + v <= Q.limit) ? x[v] : -INFINITY;
    }
    const float tmax = quad_rows_max(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])));
    const float m_new = fmaxf(Q.m, tmax);
    if (__any(m_new > Q.m)) {
        const float alpha = __builtin_amdgcn_exp2f(Q.m - m_new);
        Q.lsum *= alpha;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
#pragma unroll
            for (int v = 0; v < 4; ++v) Q.O[e][v] *= alpha;
        }
        Q.m = m_new;
    }
    float p[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        p[v] = __builtin_amdgcn_exp2f(x[v] - Q.m);
        Q.lsum += p[v];
    }
    const uint4 pw = weight_operand<DT>(p);
    // V^T operand of dimensions 16e .. 16e+15: in lane group g, lane 4t + u fetches 8 bytes of
    // token row 4g + t at dimension 16e + 4u; the transposing read hands lane c dimension
    // 16e + c of tokens 4g .. 4g+3
    const char *vsrc = vt + (4 * g + c / 4) * kVPitch + 8 * (c % 4);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const short4_t va = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_tr_ptr)(vsrc + 32 * e));
        const uint2 v2 = __builtin_bit_cast(uint2, va);
        Q.O[e] = mfma_k32<DT>(make_uint4(v2.x, v2.y, v2.x, v2.y), pw, Q.O[e]);
    }
}

// Two tiles at once (32 tokens), for the kernel whose tiles arrive in LDS by direct loads (rows
// 256 bytes apart and rotated: row r keeps its 16-byte chunk q at chunk position (q + r) mod 16 in a
// K tile and (q + 3 r) mod 16 in a V tile - the layout a direct load can produce, since it writes 16
// bytes per lane at consecutive addresses but each lane may fetch any chunk, with the bank pattern of
// rows 272 / 304 bytes apart).  `pair` is the LDS byte address of the
// K tile, V tile, K tile, V tile of tokens t0 .. t0+15 and t0+16 .. t0+31 (4 KiB each); koff /
// voff are this lane's offsets inside a K / V tile (pair_offsets).  Differences to two calls of
// tile_step, all of them fewer vector instructions per token:
//   - one running-maximum round per 32 tokens;
//   - the contraction slots of the P V products are tokens 4g..4g+3 of the first tile (slots
//     8g+0..3) and of the second (slots 8g+4..7), so the V^T operand is two transposing reads
//     side by side, and the leading and trailing 16-bit pieces of P go through two instructions
//     on the same V^T registers (no register copies);
//   - f16: the factor 2^6 that keeps small weights in the range of the 16-bit pieces is part of
//     the exponent, so it is in the running sum as well and cancels in the final division.
constexpr float kPairSlack = 8.0f;        // log2 units: a weight is at most 2^8
constexpr float kPairShiftF16 = 6.0f;     // so the f16 pieces hold at most 2^14
// An opaque 1.0f in a scalar register: p * one - (float)h is then a fused multiply-add with one 16-bit
// operand, which the compiler issues as a single v_fma_mix_f32 (it would turn p - (float)h into a
// conversion and a subtraction).  Vector instructions are what this kernel is bound by: measured,
// each takes ~4.5 cycles of a SIMD's issue port (v_exp_f32 ~8, a 16x16x32 matrix instruction 8),
// whatever the number of resident waves.  (Written as compiler-visible arithmetic, not as inline
// assembly: the compiler places the wait states that instruction pairs such as matrix result ->
// vector read need only around instructions it can see.)
__device__ __forceinline__ float opaque_one()
{
    float one;
    asm("s_mov_b32 %0, 1.0" : "=s"(one));
    return one;
}
// LDS accesses by byte address (a 32-bit number, so that a lane offset plus a constant folds into
// the instruction's immediate offset)
__device__ __forceinline__ uint4 lds_read16(uint32_t at)
{
    typedef const u32x4_t __attribute__((address_space(3))) *lds_u4_ptr;
    const u32x4_t v = *(lds_u4_ptr)(uintptr_t)at;
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint2 lds_read8_transposed(uint32_t at)
{
    typedef short4_t __attribute__((address_space(3))) *lds_tr_ptr;
    return __builtin_bit_cast(uint2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_tr_ptr)(uintptr_t)at));
}
__device__ __forceinline__ void pair_offsets(uint32_t (&koff)[4], uint32_t (&voff)[8])
{
    const int lane = threadIdx.x & (kWave - 1);
    const int g = lane / 16, c = lane % 16;
    const int vrow = 4 * g + c / 4;
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) koff[cc] = (uint32_t)(c * 256 + 16 * ((g + 4 * cc + c) & 15));
#pragma unroll
    for (int e = 0; e < 8; ++e)
        voff[e] = (uint32_t)(vrow * 256 + 16 * ((2 * e + (c % 4) / 2 + 3 * vrow) & 15) + 8 * (c & 1));
}
template <int DT, int NQ>
__device__ __forceinline__ void pair_step(QueryCols (&Q)[NQ], const uint32_t pair, const uint32_t (&koff)[4],
                                          const uint32_t (&voff)[8], const int t0, const bool (&check)[NQ],
                                          const float scale_log2, const float one)
{
    constexpr uint32_t TILE = 4096;                    // K tile | V tile | K tile | V tile
    const int lane = threadIdx.x & (kWave - 1);
    const int g = lane / 16;
    // every K fragment is read once and serves the NQ sets of query columns
    float4_t S0[NQ], S1[NQ];
#pragma unroll
    for (int j = 0; j < NQ; ++j) S0[j] = S1[j] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) {
        const uint4 k0 = lds_read16(pair + koff[cc]);
        const uint4 k1 = lds_read16(pair + 2 * TILE + koff[cc]);
#pragma unroll
        for (int j = 0; j < NQ; ++j) {
            S0[j] = mfma_k32<DT>(k0, Q[j].qf[cc], S0[j]);
            S1[j] = mfma_k32<DT>(k1, Q[j].qf[cc], S1[j]);
        }
    }
    float x[NQ][8], m_new[NQ];
    bool moved = false;
#pragma unroll
    for (int j = 0; j < NQ; ++j) {
        if (check[j]) {
            // by select, never by multiplying: rows past the stored tokens may hold anything
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                S0[j][v] = (t0 + 4 * g + v <= Q[j].limit) ? S0[j][v] : -INFINITY;
                S1[j][v] = (t0 + 16 + 4 * g + v <= Q[j].limit) ? S1[j][v] : -INFINITY;
            }
        }
        // (scaled after the masking, by a positive scale: products of a multiplication are known to be
        // canonical numbers, so the maxima below are one instruction each)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            x[j][v] = S0[j][v] * scale_log2;
            x[j][4 + v] = S1[j][v] * scale_log2;
        }
        const float tmax = fmaxf(fmaxf(fmaxf(x[j][0], x[j][1]), fmaxf(x[j][2], x[j][3])),
                                 fmaxf(fmaxf(x[j][4], x[j][5]), fmaxf(x[j][6], x[j][7])));
        // The reference point of the exponents follows the running maximum lazily: it moves only
        // when a score exceeds it by more than kPairSlack, so weights reach 2^kPairSlack at most and
        // the 33 multiplications that rescale a query's sums are rare instead of the rule (with
        // 32 queries in a wave some maximum moves in almost every step).  Any reference point gives
        // the same softmax; sums and products share it.
        const float qmax = quad_rows_max(tmax);
        m_new[j] = qmax > Q[j].m + kPairSlack ? qmax : Q[j].m;
        moved = moved || m_new[j] != Q[j].m;
    }
    if (__any(moved)) {
#pragma unroll
        for (int j = 0; j < NQ; ++j) {
            const float alpha = __builtin_amdgcn_exp2f(Q[j].m - m_new[j]);
            Q[j].lsum *= alpha;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
#pragma unroll
                for (int v = 0; v < 4; ++v) Q[j].O[e][v] *= alpha;
            }
            Q[j].m = m_new[j];
        }
    }
    // leading and trailing 16-bit pieces of the eight weights, in contraction-slot order
    uint4 ph[NQ], pl[NQ];
#pragma unroll
    for (int j = 0; j < NQ; ++j) {
        const float shift = (DT == PA_F16 ? kPairShiftF16 : 0.0f) - Q[j].m;
        float p[8];
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            p[v] = __builtin_amdgcn_exp2f(x[j][v] + shift);
            Q[j].lsum += p[v];
        }
        if (DT == PA_F16) {
            typedef _Float16 half2v __attribute__((ext_vector_type(2)));
            uint32_t hi[4], lo[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                hi[i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(p[2 * i], p[2 * i + 1]));
                const half2v hh = __builtin_bit_cast(half2v, hi[i]);
                lo[i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(__builtin_fmaf(p[2 * i], one, -(float)hh.x),
                                                                                 __builtin_fmaf(p[2 * i + 1], one, -(float)hh.y)));
            }
            ph[j] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
            pl[j] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
        } else {
            typedef float float2v __attribute__((ext_vector_type(2)));
            uint32_t hi[4], lo[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                hi[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(float2v{p[2 * i], p[2 * i + 1]}, bf16x2v_t));
                const float2v r = {p[2 * i] - as_f32(hi[i] << 16), p[2 * i + 1] - as_f32(hi[i] & 0xffff0000u)};
                lo[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, bf16x2v_t));
            }
            ph[j] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
            pl[j] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
        }
    }
    // V^T operand of dimensions 16e .. 16e+15: tokens 4g..4g+3 of the first tile, then of the second;
    // read once for the NQ sets.  Several operands at a time, so that the two products into one
    // accumulator are four instructions apart.
    constexpr int EG = NQ == 1 ? 4 : 2;
#pragma unroll
    for (int e4 = 0; e4 < 8; e4 += EG) {
        uint4 va[EG];
#pragma unroll
        for (int i = 0; i < EG; ++i) {
            const uint2 a = lds_read8_transposed(pair + TILE + voff[e4 + i]);
            const uint2 b = lds_read8_transposed(pair + 3 * TILE + voff[e4 + i]);
            va[i] = make_uint4(a.x, a.y, b.x, b.y);
        }
#pragma unroll
        for (int j = 0; j < NQ; ++j) {
#pragma unroll
            for (int i = 0; i < EG; ++i) Q[j].O[e4 + i] = mfma_k32<DT>(va[i], ph[j], Q[j].O[e4 + i]);
        }
#pragma unroll
        for (int j = 0; j < NQ; ++j) {
#pragma unroll
            for (int i = 0; i < EG; ++i) Q[j].O[e4 + i] = mfma_k32<DT>(va[i], pl[j], Q[j].O[e4 + i]);
        }
    }
}

// A tile on its way from HBM to LDS: the same coalesced 1 KiB-per-instruction loads as the
// single-query kernel (lane 16r + c: 16 bytes at column 16c of token rows r, r+4, r+8, r+12).
struct TileRegs {
    uint4 k[4], v[4];
};
// (rows at or past `rows` hold no token that any query of the tile sees: they are not fetched and
// read as zeros)
__device__ __forceinline__ void tile_fetch(TileRegs &R, const char *k_cache, const char *v_cache, int64_t base, int rows)
{
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t off = (uint32_t)lane * 16u;
    if (rows >= kTileTokens) {
#pragma unroll
        for (int j = 0; j < 4; ++j) R.k[j] = load16_stream(k_cache + base + off + 1024 * j);
#pragma unroll
        for (int j = 0; j < 4; ++j) R.v[j] = load16_stream(v_cache + base + off + 1024 * j);
    } else {
        const int r = lane / 16;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            R.k[j] = R.v[j] = make_uint4(0, 0, 0, 0);
            if (r + 4 * j < rows) {
                R.k[j] = load16_stream(k_cache + base + off + 1024 * j);
                R.v[j] = load16_stream(v_cache + base + off + 1024 * j);
            }
        }
    }
}
__device__ __forceinline__ void tile_store(const TileRegs &R, char *kt, char *vt)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int r = lane / 16, c = lane % 16;
#pragma unroll
    for (int j = 0; j < 4; ++j) *reinterpret_cast<uint4 *>(kt + (r + 4 * j) * kKPitch + 16 * c) = R.k[j];
#pragma unroll
    for (int j = 0; j < 4; ++j) *reinterpret_cast<uint4 *>(vt + (r + 4 * j) * kVPitch + 16 * c) = R.v[j];
}

// End of a token-splitting item: the W waves of the workgroup each hold partial results for
// the same 16 query columns.  Each leaves its 16 x 128 partial sums in its own staging region
// (rows 16 bytes apart from a multiple of the bank count, so the 16 queries of one store
// spread out), then all threads merge by the log-sum-exp rule and write the finished rows:
// query j goes to row (row0 + j * row_step) of `out` ([rows][H][128]).
template <int DT, int W>
__device__ __forceinline__ void split_merge_store(QueryCols &Q, char (*sm_region)[kTileLds], float (*sm_m)[16],
                                                  float (*sm_l)[16], int members, void *out, int64_t row0,
                                                  int row_step, int H, int h)
{
    using Tr = Traits<DT>;
    constexpr int D = 128, ROW_BYTES = 256;
    constexpr float kUnscale = DT == PA_F16 ? 1.0f / 16384.0f : 1.0f;
    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int g = lane / 16, c = lane % 16;
    Q.lsum = quad_rows_sum(Q.lsum);
    constexpr int MROW = D + 4;
    static_assert(16 * MROW * 4 <= kTileLds, "partial sums fit the staging region");
    float(*const mine)[MROW] = reinterpret_cast<float(*)[MROW]>(sm_region[w]);
#pragma unroll
    for (int e = 0; e < 8; ++e)
        *reinterpret_cast<float4 *>(&mine[c][16 * e + 4 * g]) =
            make_float4(Q.O[e][0] * kUnscale, Q.O[e][1] * kUnscale, Q.O[e][2] * kUnscale, Q.O[e][3] * kUnscale);
    if (g == 0) {
        sm_m[w][c] = Q.m;
        sm_l[w][c] = Q.lsum;
    }
    __syncthreads();
    constexpr int TPQ = W * kWave / 16;     // threads per query row
    constexpr int DPT = D / TPQ;            // output dimensions per thread: 2, 4 or 8 (16, 8, 4 waves)
    static_assert(DPT == 2 || DPT == 4 || DPT == 8, "workgroup width");
    const int j = threadIdx.x / TPQ, d0 = (threadIdx.x % TPQ) * DPT;
    if (j >= members) return;
    float M = sm_m[0][j];
#pragma unroll
    for (int i = 1; i < W; ++i) M = fmaxf(M, sm_m[i][j]);
    float l = 0.f, acc[DPT];
#pragma unroll
    for (int e = 0; e < DPT; ++e) acc[e] = 0.f;
#pragma unroll
    for (int i = 0; i < W; ++i) {
        const float f = __builtin_amdgcn_exp2f(sm_m[i][j] - M);
        l = __builtin_fmaf(sm_l[i][j], f, l);
        const float *src = &reinterpret_cast<const float(*)[MROW]>(sm_region[i])[j][d0];
#pragma unroll
        for (int e = 0; e < DPT; ++e) acc[e] = __builtin_fmaf(src[e], f, acc[e]);
    }
    const float inv = l > 0.f ? 1.0f / l : 0.f;
#pragma unroll
    for (int e = 0; e < DPT; ++e) acc[e] *= inv;
    char *dst = static_cast<char *>(out) + ((row0 + (int64_t)j * row_step) * H + h) * ROW_BYTES + d0 * 2;
    // Output rows are written with the streaming hint: on this device small writes in the middle of
    // a read stream cost several times their size in read bandwidth (a 256-byte row per 32 KiB read
    // slows a pure streaming kernel by 13%), and least so when they bypass the caches.
    if constexpr (DPT == 8) {
        store_frag_stream(reinterpret_cast<uint4 *>(dst), __builtin_bit_cast(u32x4_t, Tr::pack(acc)));
    } else if constexpr (DPT == 4) {
        float half_row[8] = {acc[0], acc[1], acc[2], acc[3], 0.f, 0.f, 0.f, 0.f};
        const uint4 pk = Tr::pack(half_row);
        const u32x2_t two = {pk.x, pk.y};
        __builtin_nontemporal_store(two, reinterpret_cast<u32x2_t *>(dst));
    } else {
        float pair[8] = {acc[0], acc[1], 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        __builtin_nontemporal_store(Tr::pack(pair).x, reinterpret_cast<uint32_t *>(dst));
    }
}

// ---- several query tokens per sequence ----------------------------------------
// (the tail of a prompt over an already cached prefix, Sec. 4.4 "shared prefix"; or draft
// tokens to verify).  Query i of sequence s sits at position n - q_len + i and sees tokens
// 0 .. n - q_len + i.
//
// Up to 16 queries per sequence: grid = (sequence, head); the W waves of the workgroup share
// the 16 query columns and split the tiles (wave w takes tiles w, w+W, ...), each staging
// its tiles in an LDS region of its own with the next tile's loads in flight meanwhile; the
// waves' partial results are merged through LDS at the end.
template <int DT, int B, int W>
__global__ __launch_bounds__(W *kWave) __attribute__((amdgpu_waves_per_eu(4, 8))) void pa_multi_split_kernel(
    const DecodeParams P)
{
    using Tr = Traits<DT>;
    constexpr int D = 128, ROW_BYTES = 256;
    constexpr int64_t TILE_BYTES = (int64_t)B * ROW_BYTES;
    static_assert(DT != PA_F32 && B % kTileTokens == 0, "two-byte elements, whole 16-token tiles per block");
    constexpr float kUnscale = DT == PA_F16 ? 1.0f / 16384.0f : 1.0f;
    __shared__ __align__(16) char sm_region[W][kTileLds];
    __shared__ float sm_m[W][16], sm_l[W][16];

    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int g = lane / 16, c = lane % 16;
    const int H = P.H;
    const int h = blockIdx.x % H;
    const int s = blockIdx.x / H;
    const int n = P.context_lens[s];
    const int qs = P.q_start[s];
    const int qlen = P.q_start[s + 1] - qs;
    if (qlen <= 0 || n <= 0) return;
    const int members = qlen < 16 ? qlen : 16;
    const int t_lo = n - qlen + 1;             // tokens the first query sees
    const int t_hi = n - qlen + members;       // tokens the last one of these 16 sees
    const int ntiles = (t_hi + kTileTokens - 1) / kTileTokens;

    QueryCols Q;
    query_cols_init<DT>(Q, P.q, (int64_t)qs + c, H, h, c < members, t_lo - 1 + c);
    const int32_t *__restrict__ table = P.block_tables + (int64_t)s * P.max_blocks;
    char *const kt = sm_region[w];
    char *const vt = kt + kTileTokens * kKPitch;

    // block ids are looked up two tiles ahead (wave-uniform scalar loads), tiles fetched one ahead
    auto block_of = [&](int ti) -> int { return ti < ntiles ? table[ti * kTileTokens / B] : 0; };
    auto base_of = [&](int ti, int pb) -> int64_t {
        return ((int64_t)pb * H + h) * TILE_BYTES + (int64_t)(ti * kTileTokens % B) * ROW_BYTES;
    };
    TileRegs R;
    if (w < ntiles) tile_fetch(R, P.k_cache, P.v_cache, base_of(w, block_of(w)), t_hi - w * kTileTokens);
    int pb_next = block_of(w + W);
    for (int ti = w; ti < ntiles; ti += W) {
        const int t0 = ti * kTileTokens;
        // masking starts where the tile reaches past what the first query sees
        const bool check = t0 + kTileTokens > t_lo;
        tile_store(R, kt, vt);
        if (ti + W < ntiles) tile_fetch(R, P.k_cache, P.v_cache, base_of(ti + W, pb_next), t_hi - (ti + W) * kTileTokens);
        pb_next = block_of(ti + 2 * W);
        __builtin_amdgcn_wave_barrier();
        tile_step<DT>(Q, kt, vt, t0, 0xffffu, check, P.scale_log2);
        __builtin_amdgcn_wave_barrier();
    }
    split_merge_store<DT, W>(Q, sm_region, sm_m, sm_l, members, P.out, (int64_t)qs, 1, H, h);
}

// More than 16 queries per sequence: grid = (sequence, block of queries, head); the kernel itself
// follows the load helpers below.
// One 16-byte-per-lane load straight from global memory into LDS (no register staging): lane i
// fetches from src_uniform + its own lane_offset and the data lands at lds_base + 16 i.  Completion counts
// on vmcnt like any vector load; the compiler does not know that the instruction writes LDS, so
// the kernel places its own waits (the "memory" clobber keeps compiler-issued LDS accesses on
// their side of the statement).  The five idle cycles cover what the compiler cannot see either:
// M0 written just before its use, and a base address that a vector instruction may have produced.
template <bool STREAM>
__device__ __forceinline__ void load16_to_lds(uint32_t lds_base, const char *src_uniform, uint32_t lane_offset)
{
    // (M0 carries the LDS address; it is put back afterwards because the compiler does not expect
    // inline assembly to change it)
    uint32_t m0_before;
    if (STREAM)
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %2, %3 nt\n\ts_mov_b32 m0, %0"
                     : "=&s"(m0_before)
                     : "s"(lds_base), "v"(lane_offset), "s"(src_uniform)
                     : "memory");
    else
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %2, %3\n\ts_mov_b32 m0, %0"
                     : "=&s"(m0_before)
                     : "s"(lds_base), "v"(lane_offset), "s"(src_uniform)
                     : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vector_loads_but()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// More than 16 queries per sequence.  Grid = (sequence, block of 64 NQ queries, head); the four waves
// of a workgroup own NQ sets of 16 query columns each and share every K/V tile, so K/V comes from
// memory once per 64 NQ queries (NQ = 1 up to 64 queries per sequence, 2 beyond).
//   Loads   every thread moves one 16-byte fragment of each K and V tile of a 32-token step straight
//           into a ring of NS LDS stages (load16_to_lds); NS - 1 steps are in flight while one is
//           computed, one barrier per step.  NS = 2 with four workgroups per compute unit (NQ = 1) or
//           3 with three (NQ = 2, 156 registers): the depth of the ring matters little, the number
//           of resident workgroups does (NQ = 2: four stages with two workgroups measure 6% slower).  With several blocks of queries per sequence the same
//           K/V is wanted again soon by the neighbouring workgroup (same head: with 40 heads the
//           same XCD), so the loads then leave it in the caches (STREAM unset).
//   Compute pair_step: 24 NQ matrix instructions per step and wave; each K and V^T fragment read
//           from LDS serves the wave's NQ sets.
// What bounds it (measured on MI355X): not the matrix pipes - a SIMD issues one vector or matrix
// instruction at a time, ~4.5 cycles per vector instruction and 8 per 16x16x32 product whatever the
// number of resident waves, so the softmax and conversion arithmetic between the products costs
// more issue time than the products; the kernel is written to that count (pair_step).  Next come
// the LDS reads (a product's 1 KiB K or V^T operand against ~100 B/clk for ds_read_b128 and ~50
// for the transposing read, per compute unit) - hence the NQ sets per fragment - and, at one block
// of queries per sequence, the output rows: 256-byte pieces scattered at the stride of a token
// cost ~1.7 us per MB on top of the read stream whichever store flavour or workgroup placement
// (non-temporal or plain, XCD-contiguous items or round-robin) is used.
// Measured and not adopted: a deeper ring (no change: the loads are not latency-bound), wave
// priorities that would put one wave's products beside another's arithmetic (no change), work
// items laid out contiguously per XCD (worse on mixed lengths).
template <int DT, int B, bool STREAM, int NQ>
__global__ __launch_bounds__(4 * kWave) __attribute__((amdgpu_waves_per_eu(NQ == 1 ? 4 : 3, 8))) void pa_multi_block_kernel(
    const DecodeParams P)
{
    using Tr = Traits<DT>;
    typedef char __attribute__((address_space(3))) *lds_char_ptr;
    constexpr int W = 4, ROW_BYTES = 256, STEP = 2, NS = NQ == 1 ? 2 : 3, QW = 16 * NQ, QB = W * QW;
    constexpr int TILE_LDS = 2 * kTileTokens * ROW_BYTES;            // K tile, then V tile, rows unpadded
    constexpr int STAGE_LDS = STEP * TILE_LDS;
    constexpr int LOADS_PER_STEP = 2 * STEP;                         // per thread
    constexpr int64_t TILE_BYTES = (int64_t)B * ROW_BYTES;
    static_assert(DT != PA_F32 && B % kTileTokens == 0, "two-byte elements, whole 16-token tiles per block");
    static_assert(STEP == 2, "pair_step takes two tiles");
    __shared__ __align__(1024) char sm_stage[NS][STAGE_LDS];

    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int g = lane / 16, c = lane % 16;
    const int H = P.H;
    const int h = blockIdx.x % H;
    const int rest = blockIdx.x / H;
    const int qb = rest % P.q_blocks;
    const int s = rest / P.q_blocks;
    const int n = P.context_lens[s];
    const int qs = P.q_start[s];
    const int qlen = P.q_start[s + 1] - qs;
    const int q0 = qb * QB;
    if (q0 >= qlen || n <= 0) return;
    const int wg_members = qlen - q0 < QB ? qlen - q0 : QB;
    const int wg_hi = n - qlen + q0 + wg_members;      // tokens the last query of the workgroup sees
    if (wg_hi <= 0) return;                            // (more queries than tokens: outside the interface)
    const int nsteps = (wg_hi + STEP * kTileTokens - 1) / (STEP * kTileTokens);
    // this wave's NQ sets of 16 columns: set j holds queries q0 + QW w + 16 j + (0 .. 15)
    QueryCols Q[NQ];
    int members[NQ], t_lo[NQ];
    int t_hi = 0;                                      // tokens the wave's last query sees
#pragma unroll
    for (int j = 0; j < NQ; ++j) {
        const int first = QW * w + 16 * j;
        int mem = wg_members - first;
        members[j] = mem < 0 ? 0 : (mem > 16 ? 16 : mem);
        t_lo[j] = n - qlen + q0 + first + 1;           // tokens the set's first query sees
        if (members[j] > 0) t_hi = t_lo[j] + members[j] - 1;
        query_cols_init<DT>(Q[j], P.q, (int64_t)qs + q0 + first + c, H, h, c < members[j], t_lo[j] - 1 + c);
    }
    uint32_t koff[4], voff[8];
    pair_offsets(koff, voff);
    const float one = opaque_one();
    // (the table is read-only for the whole launch: through the constant address space these
    // uniform loads go through the scalar unit and its own counter, not in line with the tile loads)
    typedef const int32_t __attribute__((address_space(4))) *uniform_i32_ptr;
    const uniform_i32_ptr table = (uniform_i32_ptr)(uintptr_t)(P.block_tables + (int64_t)s * P.max_blocks);

    // Wave w moves rows 4w .. 4w+3 of every tile: lane 16j + c fills chunk position c of LDS row
    // r16 = 4w + j, i.e. fetches chunk (c - r16) mod 16 of a K row and (c - 3 r16) mod 16 of a V row.
    // A row past the last token any query of the workgroup sees fetches that last token's row instead
    // (finite data with weight zero: rows past the stored tokens may hold anything).
    const int r16 = threadIdx.x / 16;
    const int k_chunk = 16 * ((c - r16) & 15), v_chunk = 16 * ((c - 3 * r16) & 15);
    const int last_tile = ((wg_hi - 1) / kTileTokens) * kTileTokens;
    const int last_row = wg_hi - 1 - last_tile;                  // last visible row of the last visible tile
    const uint32_t k_lane = (uint32_t)(r16 * ROW_BYTES + k_chunk), v_lane = (uint32_t)(r16 * ROW_BYTES + v_chunk);
    const uint32_t k_lane_last = (uint32_t)((r16 < last_row ? r16 : last_row) * ROW_BYTES + k_chunk);
    const uint32_t v_lane_last = (uint32_t)((r16 < last_row ? r16 : last_row) * ROW_BYTES + v_chunk);
    const uint32_t lds_stage0 = (uint32_t)(uintptr_t)(lds_char_ptr)(&sm_stage[0][0]);
    const uint32_t lds0 = lds_stage0 + (uint32_t)w * 1024u;
    auto issue = [&](int stage, int st) {
#pragma unroll
        for (int u = 0; u < STEP; ++u) {
            int t0 = (st * STEP + u) * kTileTokens;            // uniform over the workgroup
            const bool last = t0 >= last_tile;
            t0 = last ? last_tile : t0;
            const int pb = table[t0 / B];
            const int64_t off = ((int64_t)pb * H + h) * TILE_BYTES + (int64_t)(t0 % B) * ROW_BYTES;   // uniform
            const uint32_t at = lds0 + (uint32_t)(stage * STAGE_LDS + u * TILE_LDS);
            load16_to_lds<STREAM>(at, P.k_cache + off, last ? k_lane_last : k_lane);
            load16_to_lds<STREAM>(at + kTileTokens * ROW_BYTES, P.v_cache + off, last ? v_lane_last : v_lane);
        }
    };
    // NS - 1 steps of loads are in flight while one is computed.  Every step issues its loads, also
    // past the last one (they re-read the last tile into a stage nobody reads), so that the wait at
    // the top of a step can name how many younger loads it leaves in flight.
#pragma unroll
    for (int j = 0; j < NS - 1; ++j) issue(j, j);
    // the query fragments are needed from here on: have the compiler wait for their loads now, not
    // at their first use inside the loop, where its wait would also drain the tile loads in flight
#pragma unroll
    for (int j = 0; j < NQ; ++j) {
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) asm volatile("" ::"v"(__builtin_bit_cast(u32x4_t, Q[j].qf[cc])));
    }
    // pair_step masks scores with -inf before it scales them, which wants a positive scale: a negative
    // one moves into the queries (a sign flip, exact), and zero becomes 1e-30 (every product then rounds
    // to the same exponent, the uniform weights that zero asks for, and -inf stays -inf)
    float scale_log2 = P.scale_log2;
    if (scale_log2 < 0.f) {
        scale_log2 = -scale_log2;
#pragma unroll
        for (int j = 0; j < NQ; ++j) {
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
                Q[j].qf[cc].x ^= 0x80008000u;
                Q[j].qf[cc].y ^= 0x80008000u;
                Q[j].qf[cc].z ^= 0x80008000u;
                Q[j].qf[cc].w ^= 0x80008000u;
            }
        }
    }
    scale_log2 = scale_log2 < 1e-30f ? 1e-30f : scale_log2;
    for (int st0 = 0; st0 < nsteps; st0 += NS) {
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            const int st = st0 + j;
            if (st < nsteps) {                                  // uniform over the workgroup
                wait_vector_loads_but<(NS - 2) * LOADS_PER_STEP>();   // this thread's part of step st is in LDS
                // everyone's part is; and everyone is done with step st - 1, whose stage is loaded next
                __syncthreads();
                issue((j + NS - 1) % NS, st + NS - 1);
                const int t0 = st * STEP * kTileTokens;
                if (t0 < t_hi) {
                    bool check[NQ];
#pragma unroll
                    for (int i = 0; i < NQ; ++i) check[i] = t0 + STEP * kTileTokens > t_lo[i];
                    pair_step<DT, NQ>(Q, lds_stage0 + (uint32_t)(j * STAGE_LDS), koff, voff, t0, check, scale_log2, one);
                }
            }
        }
    }
    wait_vector_loads_but<0>();                        // the loads issued past the last step have landed
    // finished rows: through the wave's share of the (now idle) staging buffers, so that every store
    // instruction writes whole 256-byte rows
    __syncthreads();                                   // all waves are done reading the tiles
    // packed to the storage type first: 16 rows of 256 bytes (+16 of padding) per set
    constexpr int OROW = ROW_BYTES + 16;
    static_assert(W * QW * OROW <= NS * STAGE_LDS, "output rows fit the staging buffers");
#pragma unroll
    for (int j = 0; j < NQ; ++j) {
        if (members[j] <= 0) continue;
        const float l = quad_rows_sum(Q[j].lsum);
        const float inv = l > 0.f ? 1.0f / l : 0.f;     // (f16: sum and products both carry the factor 2^14)
        char *const rows = &sm_stage[0][0] + (w * NQ + j) * 16 * OROW;
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            const float v8[8] = {Q[j].O[e][0] * inv,     Q[j].O[e][1] * inv,     Q[j].O[e][2] * inv,
                                 Q[j].O[e][3] * inv,     Q[j].O[e + 1][0] * inv, Q[j].O[e + 1][1] * inv,
                                 Q[j].O[e + 1][2] * inv, Q[j].O[e + 1][3] * inv};
            const uint4 pk = Tr::pack(v8);
            *reinterpret_cast<uint2 *>(rows + c * OROW + 32 * e + 8 * g) = make_uint2(pk.x, pk.y);
            *reinterpret_cast<uint2 *>(rows + c * OROW + 32 * (e + 1) + 8 * g) = make_uint2(pk.z, pk.w);
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = g + 4 * i;                    // lane 16g + c: bytes 16c .. 16c+15 of query r of the set
            if (r < members[j]) {
                const uint4 v = *reinterpret_cast<const uint4 *>(rows + r * OROW + 16 * c);
                char *dst = static_cast<char *>(P.out) +
                            (((int64_t)qs + q0 + QW * w + 16 * j + r) * H + h) * ROW_BYTES + 16 * c;
                store_frag_stream(reinterpret_cast<uint4 *>(dst), __builtin_bit_cast(u32x4_t, v));
            }
        }
    }
}

// ---- sequences that share blocks ----------------------------------------------------
// One (group, head) item of pa_decode_shared: up to 16 neighbouring sequences that map common
// physical blocks (Sec. 4.4: samples of one prompt, beams of one search, requests behind one
// prefix) are the 16 query columns of the tile engine.  The group's tile list names every
// block a member maps, once, with the set of members that map it; the W waves split the
// list (wave w takes 16-token tiles w, w+W, ...), exactly like pa_multi_split_kernel, and a
// column outside a tile's set is masked like a token outside a query's context.  A shared
// block is therefore read once for all its readers, an unshared one once for its owner.
template <int DT, int B, int W>
__device__ __forceinline__ void group_item(const DecodeParams &P, const int s0, int members, const int entries,
                                           const int h)
{
    constexpr int ROW_BYTES = 256, SUBS = B / kTileTokens;
    constexpr int64_t TILE_BYTES = (int64_t)B * ROW_BYTES;
    static_assert(DT != PA_F32 && B % kTileTokens == 0, "two-byte elements, whole 16-token tiles per block");
    __shared__ __align__(16) char sm_region[W][kTileLds];
    __shared__ float sm_m[W][16], sm_l[W][16];

    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int c = lane % 16;
    const int H = P.H;
    members = members > kGroupMax ? kGroupMax : members;
    const int nwork = entries * SUBS;                          // 16-token tiles on the list
    const uint32_t everyone = (1u << members) - 1u;

    QueryCols Q;
    query_cols_init<DT>(Q, P.q, (int64_t)s0 + c, H, h, c < members, c < members ? P.context_lens[s0 + c] - 1 : -1);
    const int4 *__restrict__ list = P.tiles + (int64_t)s0 * P.max_blocks;
    char *const kt = sm_region[w];
    char *const vt = kt + kTileTokens * kKPitch;

    // list entries are looked up two tiles ahead (wave-uniform scalar loads), tiles fetched one ahead
    auto entry_of = [&](int wi) -> int4 { return wi < nwork ? list[wi / SUBS] : make_int4(0, 0, 0, 0); };
    auto base_of = [&](int wi, const int4 &ent) -> int64_t {
        return ((int64_t)ent.x * H + h) * TILE_BYTES + (int64_t)(wi % SUBS) * kTileTokens * ROW_BYTES;
    };
    // token rows of tile wi that anybody sees
    auto rows_of = [&](int wi, const int4 &ent) -> int { return ent.w - (wi % SUBS) * kTileTokens; };
    TileRegs R;
    int4 ent = entry_of(w);
    if (w < nwork) tile_fetch(R, P.k_cache, P.v_cache, base_of(w, ent), rows_of(w, ent));
    int4 ent_next = entry_of(w + W);
    for (int wi = w; wi < nwork; wi += W) {
        const int sub = wi % SUBS;
        const uint32_t mask = (uint32_t)ent.y & 0xffffu;
        const bool ragged = ((uint32_t)ent.y >> 16) & 1u;      // some member of the set sees only part of the block
        const int t0 = ent.z * B + sub * kTileTokens;
        tile_store(R, kt, vt);
        if (wi + W < nwork) tile_fetch(R, P.k_cache, P.v_cache, base_of(wi + W, ent_next), rows_of(wi + W, ent_next));
        ent = ent_next;
        ent_next = entry_of(wi + 2 * W);
        __builtin_amdgcn_wave_barrier();
        // a block that every member maps and sees in full needs no masking
        tile_step<DT>(Q, kt, vt, t0, mask, mask != everyone || ragged, P.scale_log2);
        __builtin_amdgcn_wave_barrier();
    }
    split_merge_store<DT, W>(Q, sm_region, sm_m, sm_l, members, P.out, (int64_t)s0, 1, H, h);
}

// pa_decode_shared's main launch, grid = S x H workgroups, the plan's work item i for workgroups
// (i, head): first the (group, head) items, longest first, then the (sequence, head) items of
// the ordinary one-pass kernel for the sequences outside any group; what is left of the grid
// (every group takes the place of two or more sequences) ends at once.
template <int DT, int B, int W>
__global__ __launch_bounds__(W *kWave) __attribute__((amdgpu_waves_per_eu(4, 8))) void pa_shared_fused_kernel(
    const DecodeParams P)
{
    const int h = (int)blockIdx.x % P.H;
    const int item = (int)blockIdx.x / P.H;
    // (kind, first sequence, members, tile-list entries): one scalar load says what to do
    const int4 d = *reinterpret_cast<const int4 *>(P.ginfo + ginfo_item(P.S, item));
    if (d.x == 2)
        group_item<DT, B, W>(P, d.y, d.z, d.w, h);
    else if (d.x == 1)
        decode_body<DT, 128, B, W, kChunksPerTrip, MODE_SINGLE>(P, d.y, h, 0);
}

} // namespace

#endif
