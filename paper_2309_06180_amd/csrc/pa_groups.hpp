// libpa group discovery and tile lists for pa_decode_shared.
#ifndef PA_PA_GROUPS_HPP
#define PA_PA_GROUPS_HPP

#include "pa_decode.hpp"

namespace {

// Group discovery.  Consecutive sequences whose block tables start with the
// same physical blocks form a group (that is how forked sequences sit in a
// batch: samples of one prompt, beams of one search).
//   adj[s] = leading full blocks s has in common with s-1 (0 for s = 0).
// A sequence with adj = 0 starts a run; runs are independent, so one thread
// walks each run, closing a group when it has group_max members.  Groups of
// two or more are listed compactly (shared_list / shared_count); their
// members are flagged in in_group[].  One workgroup, state in LDS when it fits.
constexpr int kGroupScanLds = 2048;   // sequences whose scan state fits in LDS
constexpr int kGroupThreads = 1024;

__device__ __forceinline__ void group_walk_run(const int32_t *adj, int32_t *in_group, int32_t *g_size,
                                               int first, int S, int group_max)
{
    int start = first, size = 1;
    auto close = [&]() {
        g_size[start] = size;
        for (int j = 0; j < size; ++j) in_group[start + j] = size > 1;
    };
    for (int sq = first + 1; sq < S; ++sq) {
        if (adj[sq] == 0) break;   // the next run belongs to another thread
        if (size < group_max) {
            ++size;
        } else {
            close();
            start = sq;
            size = 1;
        }
    }
    close();
}

__global__ __launch_bounds__(kGroupThreads) void find_groups_kernel(
    const int32_t *__restrict__ block_tables, int32_t max_blocks,
    const int32_t *__restrict__ context_lens, int32_t S, int32_t block_size, int32_t group_max,
    int32_t *__restrict__ ginfo)
{
    __shared__ int32_t s_adj[kGroupScanLds], s_in[kGroupScanLds], s_size[kGroupScanLds];
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
            // only "some block in common" matters here: the first 64 entries decide
            const unsigned long long diff = __ballot(lane < lim[u] && e0[u] != e1[u]);
            const int a = diff ? (int)__builtin_ctzll(diff) : (lim[u] < kWave ? lim[u] : kWave);
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
            if (s_adj[sq] == 0) group_walk_run(s_adj, s_in, s_size, sq, S, group_max);
        __syncthreads();
        for (int i = threadIdx.x; i < S; i += kGroupThreads) {
            ginfo[ginfo_in_group(S, i)] = s_in[i];
            ginfo[ginfo_group_size(S, i)] = s_size[i];
        }
    } else {
        for (int sq = threadIdx.x; sq < S; sq += kGroupThreads)
            if (ginfo[ginfo_adj(S, sq)] == 0)
                group_walk_run(ginfo + ginfo_adj(S, 0), ginfo + ginfo_in_group(S, 0),
                               ginfo + ginfo_group_size(S, 0), sq, S, group_max);
    }
    __syncthreads();
    // compact the first sequences of shared groups (two or more members), in order
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

// Tile list of a shared group.  Forked sequences share a block only at the same
// logical position, so the members' tables are compared position by position.
// For member j, run[j] is the number of leading positions at which its block is
// also mapped by another member: those blocks go on the group's list, once each,
// with the set of members that take them from the list; from position run[j]
// on, member j reads its blocks itself (own_start = run[j] * block_size tokens).
// Lane i of the group's wavefront looks at logical block base+i of all members,
// keeps the first member of every set of equal ids and records (block id,
// member mask, tokens stored in the block, position); a wave-wide prefix sum of
// the per-position counts places the entries, in position order, at
// tiles[first_sequence * max_blocks ...].  Nothing about the sharing pattern is
// assumed: a block mapped by several members past somebody's run is simply read
// by each of them.
//   entry.x = physical block,
//   entry.y = mask | tokens << 8 | position << 16 | ragged << 31, where ragged says that
//             some member in the mask sees fewer tokens of the block than it holds
constexpr int kTileWaves = 4;
__global__ __launch_bounds__(kTileWaves *kWave) void build_tiles_kernel(
    const int32_t *__restrict__ block_tables, int32_t max_blocks,
    const int32_t *__restrict__ context_lens, int32_t S, int32_t block_size,
    int32_t *__restrict__ ginfo, int2 *__restrict__ tiles)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int gi = blockIdx.x * kTileWaves + (int)(threadIdx.x / kWave);
    if (gi >= ginfo[ginfo_shared_count(S)]) return;
    const int start = ginfo[ginfo_shared_list(S, gi)];
    const int G = ginfo[ginfo_group_size(S, start)];
    int n[kGroupMaxMfma], nb[kGroupMaxMfma], maxnb = 0;
    int run[kGroupMaxMfma];      // closed runs: their length; open ones: -1
#pragma unroll
    for (int j = 0; j < kGroupMaxMfma; ++j) {
        n[j] = j < G ? context_lens[start + j] : 0;
        nb[j] = (n[j] + block_size - 1) / block_size;
        maxnb = nb[j] > maxnb ? nb[j] : maxnb;
        run[j] = j < G ? -1 : 0;
    }
    int2 *out = tiles + (int64_t)start * max_blocks;
    int placed = 0;
    bool any_open = true;
    for (int base = 0; base < maxnb && any_open; base += kWave) {
        const int i = base + lane;
        int id[kGroupMaxMfma];
#pragma unroll
        for (int j = 0; j < kGroupMaxMfma; ++j)
            id[j] = i < nb[j] ? block_tables[(int64_t)(start + j) * max_blocks + i] : -1 - j;
        uint32_t firsts = 0, mask[kGroupMaxMfma];
#pragma unroll
        for (int j = 0; j < kGroupMaxMfma; ++j) {
            mask[j] = 0;
            bool first = i < nb[j];
#pragma unroll
            for (int j2 = 0; j2 < kGroupMaxMfma; ++j2) {
                if (i < nb[j2] && id[j2] == id[j]) {
                    mask[j] |= 1u << j2;
                    if (j2 < j) first = false;
                }
            }
            if (first) firsts |= 1u << j;
        }
        // runs: member j stays on the list up to the first position where nobody shares its block
        uint32_t on_list = 0;    // this lane's position is inside the run of these members
        any_open = false;
#pragma unroll
        for (int j = 0; j < kGroupMaxMfma; ++j) {
            if (run[j] >= 0) continue;                       // closed in an earlier batch (uniform)
            const unsigned long long stop = __ballot(__builtin_popcount(mask[j]) < 2);
            const int len = stop ? (int)__builtin_ctzll(stop) : kWave;
            if (lane < len) on_list |= 1u << j;
            if (stop)
                run[j] = base + len;
            else
                any_open = true;
        }
        uint32_t emit = 0;
        int nmax[kGroupMaxMfma], nmin[kGroupMaxMfma];
#pragma unroll
        for (int j = 0; j < kGroupMaxMfma; ++j) {
            mask[j] &= on_list;
            nmax[j] = 0;
            nmin[j] = 0x7fffffff;
#pragma unroll
            for (int j2 = 0; j2 < kGroupMaxMfma; ++j2) {
                if ((mask[j] >> j2) & 1u) {
                    nmax[j] = n[j2] > nmax[j] ? n[j2] : nmax[j];
                    nmin[j] = n[j2] < nmin[j] ? n[j2] : nmin[j];
                }
            }
            if (((firsts >> j) & 1u) && mask[j]) emit |= 1u << j;
        }
        const int count = __builtin_popcount(emit);
        int incl = count;   // inclusive prefix sum over lanes
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const int up = __shfl_up(incl, d);
            if (lane >= d) incl += up;
        }
        const int total = __shfl(incl, kWave - 1);
        const int at = placed + incl - count;
#pragma unroll
        for (int j = 0; j < kGroupMaxMfma; ++j) {
            if ((emit >> j) & 1u) {
                int tokens = nmax[j] - i * block_size;
                tokens = tokens < block_size ? tokens : block_size;
                const uint32_t ragged = nmin[j] < (i + 1) * block_size ? 1u : 0u;
                out[at + __builtin_popcount(emit & ((1u << j) - 1u))] =
                    make_int2(id[j], (int)(mask[j] | ((uint32_t)tokens << 8) | ((uint32_t)i << 16) | (ragged << 31)));
            }
        }
        placed += total;
    }
    if (lane == 0) {
        ginfo[ginfo_tile_count(S, start)] = placed;
#pragma unroll
        for (int j = 0; j < kGroupMaxMfma; ++j) {
            // a run still open when the positions ran out covers the member's whole table
            const int blocks = run[j] >= 0 ? run[j] : nb[j];
            if (j < G) ginfo[ginfo_own_start(S, start + j)] = blocks * block_size;
        }
    }
}

} // namespace

#endif
