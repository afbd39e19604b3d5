// libpa group discovery for pa_decode_shared.
#ifndef PA_PA_GROUPS_HPP
#define PA_PA_GROUPS_HPP

#include "pa_decode.hpp"

namespace {

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


} // namespace

#endif
