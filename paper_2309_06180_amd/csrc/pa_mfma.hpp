// libpa matrix-core body (blocks shared by a group of sequences; several causal queries per
// sequence) and the kernels built on it.
#ifndef PA_PA_MFMA_HPP
#define PA_PA_MFMA_HPP

#include "pa_decode.hpp"

namespace {

// ---- several queries against shared K/V tiles, on the matrix cores -----------
// Where several queries meet the same K/V tile the work is a small dense
// contraction: up to 16 queries against 16-token tiles.  Two uses:
//   GROUP  a group of sequences that map common physical blocks (Sec. 4.4):
//          the workgroup of a (group, head) walks the group's tile list - the
//          blocks members share, once each, with the set of members that map
//          it - and leaves every member's unnormalised partial result in LDS
//          (group_item adds the members' own blocks and finishes the rows);
//   MULTI  the last q_len tokens of one sequence as causal queries; the
//          finished rows are written.
// Wave w takes tiles w, w+W, ...  Per 16-token tile:
//   S^T = K Q^T   8 x v_mfma_f32_16x16x16 (f16 or bf16 operands, fp32 result):
//                 A rows are tokens, B columns are queries.  The K tile is
//                 loaded like V, 1 KiB per instruction (a lane-per-row load
//                 would fetch half cache lines and runs about 15% slower),
//                 and turned into MFMA rows through the wave's own LDS
//                 region: lane l reads back 4 x 16 bytes of row l%16, each
//                 feeding two MFMAs, with the same (arbitrary but consistent)
//                 assignment of head dimensions to contraction slots on the
//                 Q side.
//   softmax       the result leaves lane l with query l%16 and four tokens;
//                 entries of queries that do not map the block, or of tokens a
//                 query does not see, are set to -inf by select; the running
//                 maximum is kept per query (two cross-lane maxima per tile),
//                 exp2 in fp32, the output rescaled only when a maximum moved.
//   O += P V      v_mfma_f32_16x16x16 again, 16 (f16) or 24 (bf16) per tile: A = P
//                 straight from the softmax registers, cut into two or three
//                 16-bit pieces that add up to P to fp32 accuracy (split_weights),
//                 B = V: lane l needs dim 16e + l%16 of its four tokens, so the V
//                 tile of the ordinary coalesced load is parked in the wave's LDS
//                 region (where K was) and read back two bytes at a time.  (fp32
//                 operands - v_mfma_f32_16x16x4_f32 with V widened in registers,
//                 no LDS round trip - cost 1024 instead of 256-384 matrix-pipe
//                 cycles per tile and were 2-7% slower end to end.)
// K rows are read back in the order token(i) = i/4 + 4*(i%4) so that result
// register v of lane l belongs to token l/16 + 4v: the four weights a lane holds
// are exactly the A operand of the P V product (contraction slot 4*(l/16) + v
// stands for token l/16 + 4v on both sides), so P never moves between lanes.
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

// Softmax weights as 16-bit MFMA operands without giving up fp32 accuracy: P is cut
// into pieces whose sum is P to about 2^-22 (f16: two pieces of 11 bits) or 2^-24
// (bf16: three pieces of 8 bits); every piece times a 16-bit V element is exact in the
// fp32 accumulator.  f16 has a narrow exponent range, so its weights carry a factor
// 2^14 (the largest, 1.0, becomes 16384; anything that still underflows is below
// 4e-9 of the largest weight); the factor is taken out when a wave's result is stored.
template <int DT> struct WeightPieces { static constexpr int N = DT == PA_F16 ? 2 : 3; };
template <int DT>
__device__ __forceinline__ void split_weights(const float (&p)[4], uint32_t (&out)[WeightPieces<DT>::N][2])
{
    if (DT == PA_F16) {
        typedef _Float16 half2v __attribute__((ext_vector_type(2)));
        float rest[4];
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            const float a = p[2 * hh] * 16384.0f, b = p[2 * hh + 1] * 16384.0f;
            const half2v hi = __builtin_bit_cast(half2v, __builtin_amdgcn_cvt_pkrtz(a, b));
            out[0][hh] = __builtin_bit_cast(uint32_t, hi);
            rest[2 * hh] = a - (float)hi.x;
            rest[2 * hh + 1] = b - (float)hi.y;
        }
#pragma unroll
        for (int hh = 0; hh < 2; ++hh)
            out[1][hh] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(rest[2 * hh], rest[2 * hh + 1]));
    } else {
        float rest[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) rest[v] = p[v];
#pragma unroll
        for (int pc = 0; pc < 3; ++pc) {
            uint32_t top[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                top[v] = __builtin_bit_cast(uint32_t, rest[v]) & 0xffff0000u;   // the leading 8 bits of what is left
                rest[v] -= as_f32(top[v]);
            }
            out[pc][0] = (top[0] >> 16) | top[1];
            out[pc][1] = (top[2] >> 16) | top[3];
        }
    }
}

// GROUP leaves, for member j, the unnormalised result of the tiles on the list in LDS
// (part_acc[j][128], part_m[j] in log2 units, part_l[j]); MULTI writes the finished rows.
template <int DT, int B, int W, int GQ, bool MULTI>
__device__ __forceinline__ void mfma_body(const DecodeParams &P, const int block_index, float (*part_acc)[128],
                                          float *part_m, float *part_l)
{
    using Tr = Traits<DT>;
    constexpr int D = 128, ROW_BYTES = 256, SUBS = B / 16;
    constexpr int64_t TILE_BYTES = (int64_t)B * ROW_BYTES;
    static_assert(DT != PA_F32 && B % 16 == 0, "two-byte elements, whole 16-token tiles per block");
    static_assert(GQ <= 16, "one MFMA row per query");
    constexpr int PIECES = WeightPieces<DT>::N;
    constexpr float kUnscale = DT == PA_F16 ? 1.0f / 16384.0f : 1.0f;

    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int r = lane / 16;
    const int c = lane % 16;
    const int H = P.H;
    const int h = block_index % H;
    const int rest = block_index / H;

    // Query c of the item is row q_row0 + c of P.q (and of P.out) and sees tokens
    // 0 .. limit of its own sequence.  MULTI walks the block table of sequence s over
    // tokens [0, t_hi); GROUP walks the tile list of the group that starts at s.
    int s, members, nwork, t_hi = 0, t_lo = 0, limit = -1;
    int64_t q_row0;
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
        if (c < members) limit = t_lo - 1 + c;
        q_row0 = qs + q0;
        nwork = (t_hi + 15) / 16;            // 16-token tiles
    } else {
        if (rest >= P.ginfo[ginfo_shared_count(P.S)]) return;
        s = P.ginfo[ginfo_shared_list(P.S, rest)];   // a group is named by its first sequence
        members = P.ginfo[ginfo_group_size(P.S, s)];
        if (members > GQ) members = GQ;
        if (c < members) limit = P.context_lens[s + c] - 1;
        q_row0 = s;
        nwork = P.ginfo[ginfo_tile_count(P.S, s)];   // tile-list entries (blocks)
    }

    // Q^T as the B operand: lane l holds, for query l%16, the same byte ranges of the
    // query row that it will hold of each K row
    uint4 qf[4];
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) {
        qf[cc] = make_uint4(0, 0, 0, 0);
        if (c < members)
            qf[cc] = *reinterpret_cast<const uint4 *>(static_cast<const char *>(P.q) +
                                                      ((q_row0 + c) * H + h) * ROW_BYTES + 64 * cc + 16 * r);
    }
    float4_t O[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) O[e] = float4_t{0.f, 0.f, 0.f, 0.f};
    float m = kNegBig, lsum = 0.f;

    const int32_t *__restrict__ table = P.block_tables + (int64_t)s * P.max_blocks;
    const int2 *__restrict__ tiles = MULTI ? nullptr : P.tiles + (int64_t)s * P.max_blocks;
    const uint32_t v_lane_off = (uint32_t)lane * 16u;

    // One region of LDS per wave.  While the wave streams it is the staging area of its K
    // tile: K rows arrive by the same coalesced load as V (lane l: token l/16 + 4j, bytes
    // 16*(l%16) of the row) and are read back as MFMA rows (lane l: token row of l%16).
    // Rows are padded by 16 bytes so that the 16 rows one read touches fall in different
    // banks.  When the wave is done the region holds its partial result for the merge.
    constexpr int K_ROW_PAD = ROW_BYTES + 16;
    constexpr int V_ROW_PAD = ROW_BYTES + 32;
    constexpr int REGION = (16 * V_ROW_PAD > GQ * D * 4) ? 16 * V_ROW_PAD : GQ * D * 4;
    __shared__ __align__(16) char sm_region[W][REGION];
    char *const kst = sm_region[w];
    const uint32_t kst_write = (uint32_t)(r * K_ROW_PAD + 16 * c);                      // + 4j rows
    const uint32_t kst_read = (uint32_t)((c / 4 + 4 * (c % 4)) * K_ROW_PAD + 16 * r);   // + 64cc bytes
    const uint32_t vst_write = (uint32_t)(r * V_ROW_PAD + 16 * c);                      // + 4v rows
    const uint32_t vst_read = (uint32_t)(r * V_ROW_PAD + 2 * c);                        // + 4v rows, + 32e bytes

    // one 16-token tile: first token t0 (position in the sequence), at byte `base` of
    // the caches; rows at or past `rows` hold no token any query here sees;
    // `mask`: queries that map this block; `check`: some entry may need masking
    auto tile = [&](int64_t base, int t0, int rows, uint32_t mask, bool check) {
        uint4 kf[4], vf[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) kf[j] = load16_stream(P.k_cache + base + v_lane_off + 1024 * j);
#pragma unroll
        for (int v = 0; v < 4; ++v) vf[v] = load16_stream(P.v_cache + base + v_lane_off + 1024 * v);
#pragma unroll
        for (int j = 0; j < 4; ++j) *reinterpret_cast<uint4 *>(kst + kst_write + 4 * j * K_ROW_PAD) = kf[j];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) kf[cc] = *reinterpret_cast<const uint4 *>(kst + kst_read + 64 * cc);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();

        float4_t S = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
            S = mfma_qk<DT>(kf[cc].x, kf[cc].y, qf[cc].x, qf[cc].y, S);
            S = mfma_qk<DT>(kf[cc].z, kf[cc].w, qf[cc].z, qf[cc].w, S);
        }
        float x[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) x[v] = S[v] * P.scale_log2;
        if (check) {
            // by select, never by multiplying: rows past the stored tokens may hold anything
            const bool mine = (mask >> c) & 1u;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = r + 4 * v;
                x[v] = (mine && t0 + row <= limit) ? x[v] : -INFINITY;
                const bool unseen = row >= rows;
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
        // the V tile takes the K tile's place in the wave's LDS region (K is in registers by now)
#pragma unroll
        for (int v = 0; v < 4; ++v) *reinterpret_cast<uint4 *>(kst + vst_write + 4 * v * V_ROW_PAD) = vf[v];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        float p[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            p[v] = __builtin_amdgcn_exp2f(x[v] - m);
            lsum += p[v];
        }
        // P as the A operand, split into 16-bit pieces whose sum is P to fp32 accuracy
        uint32_t pa[PIECES][2];
        split_weights<DT>(p, pa);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            // B operand of dims 16e .. 16e+15: lane l takes dim 16e + l%16 of its four tokens
            uint32_t vb[2];
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                const uint32_t lo = *reinterpret_cast<const uint16_t *>(kst + vst_read + 4 * (2 * hh) * V_ROW_PAD + 32 * e);
                const uint32_t hi = *reinterpret_cast<const uint16_t *>(kst + vst_read + 4 * (2 * hh + 1) * V_ROW_PAD + 32 * e);
                vb[hh] = lo | (hi << 16);
            }
#pragma unroll
            for (int pc = 0; pc < PIECES; ++pc) O[e] = mfma_qk<DT>(pa[pc][0], pa[pc][1], vb[0], vb[1], O[e]);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };

    if (MULTI) {
        for (int ti = w; ti < nwork; ti += W) {
            const int t0 = ti * 16;
            const int pb = table[t0 / B];
            const int64_t base = ((int64_t)pb * H + h) * TILE_BYTES + (int64_t)(t0 % B) * ROW_BYTES;
            // masking starts where the tile reaches past what the item's first query sees
            tile(base, t0, t_hi - t0, 0xffffu, t0 + 16 > t_lo);
        }
    } else {
        const uint32_t everyone = (1u << members) - 1u;
        for (int ei = w; ei < nwork; ei += W) {
            const int2 ent = tiles[ei];                        // wave-uniform: a scalar load
            const uint32_t mask = (uint32_t)ent.y & 0xffu;
            const int tokens = ((uint32_t)ent.y >> 8) & 0xffu; // tokens stored in the block
            const int pos = ((uint32_t)ent.y >> 16) & 0x7fffu; // logical block index
            const bool ragged = (uint32_t)ent.y >> 31;         // some member sees only part of the block
            const int64_t base = ((int64_t)ent.x * H + h) * TILE_BYTES;
#pragma unroll 1
            for (int sub = 0; sub < SUBS; ++sub) {
                if (sub * 16 >= tokens) break;
                // a block that every member maps and sees in full needs no masking
                const bool check = mask != everyone || ragged;
                tile(base + (int64_t)sub * 16 * ROW_BYTES, pos * B + sub * 16, tokens - sub * 16, mask, check);
            }
        }
    }
    lsum += __shfl_xor(lsum, 16);
    lsum += __shfl_xor(lsum, 32);

    // merge the waves: per query, its 128 accumulators sit in the 16 lanes r = query/4
    auto sm_acc = [&](int wave) { return reinterpret_cast<float(*)[D]>(sm_region[wave]); };
    __shared__ float sm_m[W][GQ], sm_l[W][GQ];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int qi = 4 * r + v;
        if (qi < members) {
#pragma unroll
            for (int e = 0; e < 8; ++e) sm_acc(w)[qi][16 * e + c] = O[e][v] * kUnscale;
        }
    }
    if (r == 0 && c < members) {
        sm_m[w][c] = m;
        sm_l[w][c] = lsum;
    }
    __syncthreads();
    if (w == 0 && r == 0) {
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
                for (int e = 0; e < 8; ++e) acc[e] = __builtin_fmaf(sm_acc(i)[j][8 * c + e], f, acc[e]);
            }
            if (MULTI) {
                // a query with an empty context has l = 0: its row is zero
                const float inv = l > 0.f ? 1.0f / l : 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] *= inv;
                reinterpret_cast<uint4 *>(P.out)[((q_row0 + j) * H + h) * 16 + c] = Tr::pack(acc);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) part_acc[j][8 * c + e] = acc[e];
                if (c == 0) {
                    part_m[j] = M;
                    part_l[j] = l;
                }
            }
        }
    }
}

// Several query tokens per sequence (the tail of a prompt over an already cached
// prefix, Sec. 4.4 "shared prefix"; or draft tokens to verify): grid =
// (sequence, block of 16 queries, head).
// (at least four waves per SIMD, i.e. at most 128 VGPRs: otherwise the compiler takes 136 and a
// third of the residency is lost)
template <int DT, int B, int W>
__global__ __launch_bounds__(W *kWave) __attribute__((amdgpu_waves_per_eu(4, 8))) void pa_decode_multi_kernel(
    const DecodeParams P)
{
    mfma_body<DT, B, W, 16, true>(P, (int)blockIdx.x, nullptr, nullptr, nullptr);
}

// One (shared group, head) item of pa_decode_shared.  The blocks that members have in common
// are on the group's tile list and go through the matrix cores once for everybody who maps
// them.  From its own_start on, a member's remaining blocks are its own business: the waves
// of the workgroup are dealt out among the members (W / members waves each, at least one;
// more members than waves take several rounds) and stream them with the ordinary
// single-query pass.  A member's results - tile list, and one per wave - are merged by the
// log-sum-exp rule and the finished row is written: nothing partial leaves the workgroup.
template <int DT, int B, int W>
__device__ __forceinline__ void group_item(const DecodeParams &P, const int block_index)
{
    using Tr = Traits<DT>;
    constexpr int EPL = Tr::EPL, LPT = 16, D = 128;
    __shared__ float part_acc[kGroupMaxMfma][D];
    __shared__ float part_m[kGroupMaxMfma], part_l[kGroupMaxMfma];
    __shared__ float own_acc[W][D];
    __shared__ float own_m[W], own_l[W];
    const int H = P.H;
    const int h = block_index % H;
    const int rest = block_index / H;
    if (rest >= P.ginfo[ginfo_shared_count(P.S)]) return;
    const int s0 = P.ginfo[ginfo_shared_list(P.S, rest)];
    int members = P.ginfo[ginfo_group_size(P.S, s0)];
    if (members > kGroupMaxMfma) members = kGroupMaxMfma;

    mfma_body<DT, B, W, kGroupMaxMfma, false>(P, block_index, part_acc, part_m, part_l);

    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int g = lane / LPT;
    const int c = lane % LPT;
    const int per = W / members > 0 ? W / members : 1;   // waves per member
    const int slots = W / per;                           // members served at a time
    const int slot = w % slots, k = w / slots;           // this wave: k-th wave of the slot's member
    for (int first = 0; first < members; first += slots) {
        const int j = first + slot;
        const bool active = k < per && j < members;
        float m = kNegBig, l = 0.f, acc[EPL];
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
        int sq = s0, n = 0;
        if (active) {
            sq = s0 + j;
            n = P.context_lens[sq];
            const int own = P.ginfo[ginfo_own_start(P.S, sq)];
            if (own < n) stream_range<DT, D, B, kGroupChunksPerTrip>(P, sq, h, own, n, k, per, m, l, acc);
        }
        if (g == 0) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) own_acc[w][c * EPL + e] = acc[e];
            if (c == 0) {
                own_m[w] = m;
                own_l[w] = l;
            }
        }
        __syncthreads();   // also orders the tile-list results of wave 0 before their readers
        if (active && k == 0 && g == 0) {
            float M = part_m[j];
            for (int i = 0; i < per; ++i) M = fmaxf(M, own_m[slot + i * slots]);
            const float f_list = __builtin_amdgcn_exp2f(part_m[j] - M);
            l = part_l[j] * f_list;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] = part_acc[j][c * EPL + e] * f_list;
            for (int i = 0; i < per; ++i) {
                const int wi = slot + i * slots;
                const float f = __builtin_amdgcn_exp2f(own_m[wi] - M);
                l = __builtin_fmaf(own_l[wi], f, l);
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[e] = __builtin_fmaf(own_acc[wi][c * EPL + e], f, acc[e]);
            }
            const float inv = l > 0.f ? 1.0f / l : 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] *= inv;
            reinterpret_cast<uint4 *>(P.out)[((int64_t)sq * H + h) * LPT + c] = Tr::pack(acc);
        }
        __syncthreads();   // the next round reuses own_acc
    }
}

// pa_decode_shared's main launch.  The first P.group_blocks workgroups are
// (shared group, head) items; the rest are (sequence, head) items of the ordinary
// one-pass kernel for the sequences that share nothing (members of a shared group
// end at once there).
template <int DT, int B, int W>
__global__ __launch_bounds__(W *kWave) __attribute__((amdgpu_waves_per_eu(4, 8))) void pa_shared_fused_kernel(
    const DecodeParams P)
{
    if ((int)blockIdx.x < P.group_blocks) {
        group_item<DT, B, W>(P, (int)blockIdx.x);
    } else {
        const int idx = (int)blockIdx.x - P.group_blocks;
        if (P.ginfo[ginfo_in_group(P.S, idx / P.H)]) return;
        decode_body<DT, 128, B, W, kChunksPerTrip, MODE_SINGLE>(P, idx);
    }
}

} // namespace

#endif
