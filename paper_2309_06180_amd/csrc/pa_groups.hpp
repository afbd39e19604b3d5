// libpa sharing plan of pa_decode_shared: group discovery and tile lists, one launch.
#ifndef PA_PA_GROUPS_HPP
#define PA_PA_GROUPS_HPP

#include "pa_decode.hpp"

namespace {

// Consecutive sequences whose block tables start with the same physical blocks are candidates
// for a group (that is how forked sequences sit in a batch: samples of one prompt, beams of
// one search, requests behind one system prompt; Sec. 4.4).
//   adj[s] = leading full blocks s has in common with s-1 (0 for s = 0).
// Sequence s is tied to s-1 when the common run is worth it: at least kShareMinTokens
// tokens and at least 1/kShareMinFraction of the shorter of the two contexts.  (A group's
// tiles go through the matrix-core path, which streams unshared blocks a few percent slower
// than the single-query kernel: a short common run does not pay for that.)  A sequence not
// tied to its predecessor starts a run; runs are independent, so one thread walks each run,
// closing a group every kGroupMax members.  Groups of two or more are listed compactly
// (group_list / group_count) with their members flagged in in_group[]; all other sequences
// go on single_list.  Then wavefronts build the groups' tile lists.
//
// One launch of kPlanBlocks workgroups.  The scan is a few microseconds of dependent loads,
// so every workgroup does all of it for itself, in LDS (only workgroup 0 writes the group
// table); the tile lists, the larger part, are divided among the wavefronts of all
// workgroups.  Nothing is exchanged between workgroups.
constexpr int kPlanMaxSeqs = 16384;   // sequences whose scan state fits in LDS
constexpr int kPlanThreads = 512;
constexpr int kPlanBlocks = 16;
constexpr int kShareMinTokens = 32;
constexpr int kShareMinFraction = 8;
constexpr int kAdjStep = 16;          // table entries a thread compares per step

__device__ __host__ __forceinline__ bool share_is_worth_it(int common_blocks, int block_size, int n0, int n1)
{
    const int64_t t = (int64_t)common_blocks * block_size;
    const int shorter = n0 < n1 ? n0 : n1;
    return t >= kShareMinTokens && t * kShareMinFraction >= shorter;
}

// exclusive prefix sum over the lanes of a wavefront of a small count (< 32) per lane, and the
// wave's total: one ballot per bit of the count
__device__ __forceinline__ int wave_prefix_small(int count, int &total)
{
    int before = 0;
    total = 0;
#pragma unroll
    for (int b = 0; b < 5; ++b) {
        const unsigned long long m = __ballot((count >> b) & 1);
        before += (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u)) << b;
        total += __builtin_popcountll(m) << b;
    }
    return before;
}

// Tile list of the group of G sequences that starts at `start`, built by one wavefront: every
// physical block a member maps, once per logical position, with the set of members that map
// it there.  Forked sequences share a block only at the same logical position, so the
// members' tables are compared position by position: lane i looks at logical block base+i of
// all members (the next 64 positions' ids are requested before these are worked on), keeps
// the first member of every set of equal ids and records (block id, member set, position,
// tokens); a wave-wide prefix sum of the per-position counts places the entries, in position
// order.  Nothing about the sharing pattern is assumed (common prompt, beam tree,
// un-diverged forks).  `n` points at the members' context lengths (in LDS).
__device__ __forceinline__ int build_tile_list(const int32_t *__restrict__ block_tables, int32_t max_blocks,
                                               int32_t block_size, int start, int G, int4 *__restrict__ out,
                                               const int32_t *n)
{
    const int lane = threadIdx.x & (kWave - 1);
    int len[kGroupMax], maxnb = 0;
#pragma unroll
    for (int j = 0; j < kGroupMax; ++j) {
        len[j] = j < G ? n[j] : 0;
        const int nb = (len[j] + block_size - 1) / block_size;
        maxnb = nb > maxnb ? nb : maxnb;
    }
    auto fetch = [&](int (&id)[kGroupMax], int base) {
        const int i = base + lane;
#pragma unroll
        for (int j = 0; j < kGroupMax; ++j)
            id[j] = i * block_size < len[j] ? block_tables[(int64_t)(start + j) * max_blocks + i] : -1 - j;
    };
    int placed = 0;
    int id[kGroupMax], id_next[kGroupMax];
    fetch(id, 0);
    for (int base = 0; base < maxnb; base += kWave) {
        const int i = base + lane;
        if (base + kWave < maxnb) fetch(id_next, base + kWave);
        // the first member of every set of equal ids emits the set's entry (ids of absent members
        // are negative and all different)
        uint32_t emit = 0;
#pragma unroll
        for (int j = 0; j < kGroupMax; ++j) {
            bool first = id[j] >= 0;
#pragma unroll
            for (int j2 = 0; j2 < j; ++j2) first = first && id[j2] != id[j];
            emit |= first ? 1u << j : 0u;
        }
        int total;
        int at = placed + wave_prefix_small(__builtin_popcount(emit), total);
#pragma unroll
        for (int j = 0; j < kGroupMax; ++j) {
            if ((emit >> j) & 1u) {
                uint32_t mask = 0;
                int nmax = 0, nmin = 0x7fffffff;
#pragma unroll
                for (int j2 = j; j2 < kGroupMax; ++j2) {
                    const bool same = id[j2] == id[j];
                    mask |= same ? 1u << j2 : 0u;
                    nmax = same && len[j2] > nmax ? len[j2] : nmax;
                    nmin = same && len[j2] < nmin ? len[j2] : nmin;
                }
                int tokens = nmax - i * block_size;
                tokens = tokens < block_size ? tokens : block_size;
                const uint32_t ragged = nmin < (i + 1) * block_size ? 1u : 0u;
                out[at++] = make_int4(id[j], (int)(mask | (ragged << 16)), i, tokens);
            }
        }
        placed += total;
#pragma unroll
        for (int j = 0; j < kGroupMax; ++j) id[j] = id_next[j];
    }
    return placed;
}

__global__ __launch_bounds__(kPlanThreads) void shared_plan_kernel(
    const int32_t *__restrict__ block_tables, int32_t max_blocks,
    const int32_t *__restrict__ context_lens, int32_t S, int32_t block_size, int32_t *__restrict__ ginfo,
    int4 *__restrict__ tiles)
{
    constexpr int NW = kPlanThreads / kWave;
    __shared__ unsigned long long s_ties[kPlanMaxSeqs / kWave + 1];   // bit s: sequence s is tied to s-1
    __shared__ uint8_t s_in[kPlanMaxSeqs], s_size[kPlanMaxSeqs];
    __shared__ uint16_t s_list[kPlanMaxSeqs / 2];                     // the groups' first sequences
    __shared__ int32_t s_len[kPlanMaxSeqs];                           // context lengths
    __shared__ int32_t wave_count[NW];
    __shared__ int32_t running, n_groups;
    const int lane = threadIdx.x & (kWave - 1);
    const int w = threadIdx.x / kWave;
    const bool writer = blockIdx.x == 0;

    // adj[s]: every thread compares the table row of its sequence with its predecessor's,
    // kAdjStep entries at a time (their loads in flight together, the first step's together
    // with the lengths'); most pairs differ in the first step.  Every wavefront covers 64
    // consecutive sequences and leaves their tie bits as one word.
    for (int base = 0; base < S; base += kPlanThreads) {
        const int sq = base + threadIdx.x;
        int a = 0;
        bool tie = false;
        if (sq < S) {
            const int32_t *r1 = block_tables + (int64_t)sq * max_blocks;
            const int32_t *r0 = sq > 0 ? r1 - max_blocks : r1;
            const int width = max_blocks < kAdjStep ? max_blocks : kAdjStep;
            int e0[kAdjStep], e1[kAdjStep];
#pragma unroll
            for (int i = 0; i < kAdjStep; ++i) {     // any entry of the row may be read: the table is S x max_blocks
                e0[i] = i < width ? r0[i] : 0;
                e1[i] = i < width ? r1[i] : 0;
            }
            const int n1 = context_lens[sq];
            const int n0 = sq > 0 ? context_lens[sq - 1] : 0;
            s_len[sq] = n1;
            s_size[sq] = 0;
            const int lim = (n0 < n1 ? n0 : n1) / block_size;
            bool same = true;
            for (int b0 = 0; b0 < lim && same; b0 += kAdjStep) {
                if (b0 > 0) {
#pragma unroll
                    for (int i = 0; i < kAdjStep; ++i) {
                        e0[i] = b0 + i < lim ? r0[b0 + i] : 0;
                        e1[i] = b0 + i < lim ? r1[b0 + i] : 0;
                    }
                }
#pragma unroll
                for (int i = 0; i < kAdjStep; ++i) {
                    same = same && b0 + i < lim && e0[i] == e1[i];
                    a += same ? 1 : 0;
                }
            }
            tie = sq > 0 && share_is_worth_it(a, block_size, n0, n1);
            if (writer) ginfo[ginfo_adj(S, sq)] = a;
        }
        const unsigned long long word = __ballot(tie);
        if (lane == 0) s_ties[(base + threadIdx.x) / kWave] = word;
    }
    if (threadIdx.x == 0) s_ties[(S + kWave - 1) / kWave] = 0;     // a word past the end stops every scan
    __syncthreads();

    // a sequence not tied to its predecessor starts a run of tied sequences; its thread measures
    // the run on the tie words and cuts it into groups of at most kGroupMax
    for (int first = threadIdx.x; first < S; first += kPlanThreads) {
        if ((s_ties[first / kWave] >> (first % kWave)) & 1ull) continue;
        int end = first + 1;
        while (end < S) {
            const int room = kWave - end % kWave;
            const unsigned long long rest = ~(s_ties[end / kWave] >> (end % kWave));   // zeros: tied
            const int ones = rest ? (int)__builtin_ctzll(rest) : kWave;
            end += ones < room ? ones : room;
            if (ones < room) break;
        }
        end = end < S ? end : S;
        for (int start = first; start < end; start += kGroupMax)
            s_size[start] = (uint8_t)(end - start < kGroupMax ? end - start : kGroupMax);
    }
    __syncthreads();
    // membership: the group a sequence belongs to starts at most kGroupMax - 1 places before it
    for (int i = threadIdx.x; i < S; i += kPlanThreads) {
        int in = 0;
        for (int back = 0; back < kGroupMax && back <= i; ++back) {
            const int size = s_size[i - back];
            if (size > 0) {
                in = size >= 2 && size > back;
                break;
            }
        }
        s_in[i] = (uint8_t)in;
        if (writer) {
            ginfo[ginfo_in_group(S, i)] = in;
            ginfo[ginfo_group_size(S, i)] = s_size[i];
        }
    }
    __syncthreads();

    // in-order compaction: first sequences of the groups, then the sequences outside any group
    for (int which = 0; which < 2; ++which) {
        if (threadIdx.x == 0) running = 0;
        __syncthreads();
        for (int base = 0; base < S; base += kPlanThreads) {
            const int sq = base + threadIdx.x;
            const bool flag = sq < S && (which == 0 ? s_size[sq] >= 2 : s_in[sq] == 0);
            const unsigned long long mask = __ballot(flag);
            if (lane == 0) wave_count[w] = __builtin_popcountll(mask);
            __syncthreads();
            int before = running;
            for (int i = 0; i < w; ++i) before += wave_count[i];
            if (flag) {
                const int at = before + __builtin_popcountll(mask & ((1ull << lane) - 1));
                if (which == 0) s_list[at] = (uint16_t)sq;
                if (which == 1 && writer) {
                    ginfo[ginfo_single_list(S, at)] = sq;
                    *reinterpret_cast<int4 *>(ginfo + ginfo_item(S, n_groups + at)) = make_int4(1, sq, 1, 0);
                }
            }
            __syncthreads();
            if (threadIdx.x == 0) {
                int total = running;
                for (int i = 0; i < NW; ++i) total += wave_count[i];
                running = total;
            }
            __syncthreads();
        }
        if (threadIdx.x == 0) {
            if (writer) ginfo[which == 0 ? ginfo_group_count(S) : ginfo_single_count(S)] = running;
            if (which == 0) n_groups = running;
        }
        __syncthreads();
    }

    int32_t *const items = ginfo + ginfo_item(S, 0);
    if (writer) {
        const int n_single = running;      // left by the second compaction
        for (int i = threadIdx.x; i < S; i += kPlanThreads) {
            if (i < n_groups)
                ginfo[ginfo_group_list(S, i)] = s_list[i];
            else if (i >= n_groups + n_single)
                *reinterpret_cast<int4 *>(items + 4 * i) = make_int4(0, 0, 0, 0);
        }
    }

    // tile lists: the wavefronts of all workgroups take the groups in turn
    for (int gi = blockIdx.x * NW + w; gi < n_groups; gi += gridDim.x * NW) {
        const int start = s_list[gi];
        const int G = s_size[start];
        const int placed = build_tile_list(block_tables, max_blocks, block_size, start, G,
                                           tiles + (int64_t)start * max_blocks, s_len + start);
        if (lane == 0) {
            ginfo[ginfo_tile_count(S, start)] = placed;
            *reinterpret_cast<int4 *>(items + 4 * gi) = make_int4(2, start, G, placed);
        }
    }
}

} // namespace

#endif
