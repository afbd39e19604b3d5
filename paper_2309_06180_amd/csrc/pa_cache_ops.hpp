// libpa cache maintenance kernels: reshape_and_cache, copy_blocks, swap_blocks, and the read-bandwidth probe.
#ifndef PA_PA_CACHE_OPS_HPP
#define PA_PA_CACHE_OPS_HPP

#include "pa_common.hpp"

namespace {

// ---- reshape_and_cache -------------------------------------------------------
// One thread moves one 16-byte fragment.  A token is frags_per_token = H*D*E/16
// fragments; fragment r of token t belongs to head r / frags_per_row.
// (Measured and not adopted: one workgroup per token with the slot looked up once, no
// divisions, and up to four fragments per thread issued before the first store - 5.26
// instead of 5.48 TB/s of read+write traffic at 65 536 tokens.  As with the block copy,
// many small workgroups of one fragment per thread are what this memory system likes.)
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
// is frags_per_block consecutive 16-byte fragments.  One fragment per thread in
// workgroups of 256: with 4096 randomly placed pairs that measured 5.86 TB/s of
// read+write traffic, against 5.25 with two fragments per thread, 5.53 / 5.07 with
// workgroups of 512 / 1024 threads and 5.06 with 512 threads x two fragments.
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


} // namespace

#endif
