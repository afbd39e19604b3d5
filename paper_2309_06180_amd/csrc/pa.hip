// libpa - paged single-query attention for gfx950 (MI355X): host side.
//
// Operations of PagedAttention's decode step (arxiv 2309.06180):
//   pa_decode            Sec. 4.1, Eq. (4): attention of one query per sequence
//                        over K/V blocks reached through a block table
//   pa_reshape_and_cache Sec. 4.3 / 5.1 (1): store new K/V vectors at their slots
//   pa_copy_blocks       Sec. 4.4 / 5.1 (3): batched copy-on-write block copies
//   pa_swap_blocks       Sec. 4.5: block swap between HBM and pinned host memory
//   pa_decode_shared     Sec. 4.4 workloads: blocks shared by neighbouring sequences read once
//   pa_decode_multi      Sec. 4.4 (shared prefix): several causal queries per sequence
//
// This file holds launch planning, dispatch over (dtype, head_dim, block_size)
// and the C ABI; the kernels are in the headers it includes:
//   pa_common.hpp     element types, cross-lane sums, streaming loads/stores
//   pa_decode.hpp     the VALU decode kernel and the merge kernel
//   pa_mfma.hpp       matrix-core bodies (shared prefixes, several queries)
//   pa_groups.hpp     group discovery for pa_decode_shared
//   pa_cache_ops.hpp  cache write, block copy, block swap, bandwidth probe
//
// Cache layout [NB][H][B][D]: the K (or V) vectors of one (block, head) are
// B*D*E contiguous bytes, a token row is D*E bytes.  Every wavefront load of
// the single-query path is 64 lanes x 16 bytes = 1 KiB of consecutive
// addresses.  That path is a batch of matrix-vector products (one flop per
// byte of KV at 2-byte elements), bound by HBM bandwidth, so it uses no MFMA:
// the design goal is bytes in flight per compute unit and few VALU
// instructions per byte.
#include <hip/hip_runtime.h>

#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <tuple>
#include <type_traits>

#include "pa.h"

#include "pa_common.hpp"
#include "pa_decode.hpp"
#include "pa_mfma.hpp"
#include "pa_groups.hpp"
#include "pa_cache_ops.hpp"

// ---- static scratch of pa_decode_static ------------------------------------------
// Split-context partials for callers that cannot hand over a workspace.  Every device the
// library runs on holds its own copy of the array until the process ends.  In host code the
// array's name is only a handle: the device address is asked for once per device, with that
// device current, and kept; kernels and copies are given that address, never the name.
static __device__ __align__(256) unsigned char scratch[PA_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

pa_status static_scratch(void **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return PA_ERR_HIP;
    }
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        // two threads racing here ask twice and get the same answer
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return PA_ERR_HIP;
        }
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *ptr = p;
    return PA_OK;
}

// ---- host side -----------------------------------------------------------------
// Kernel launches report their own status: the return value of hipLaunchKernel, kept per
// thread between the entry and the exit of one library call.  (hipGetLastError would also
// return, and clear, an error that an earlier call of the caller left behind.)
thread_local hipError_t t_launch_status = hipSuccess;

template <typename... KArgs, typename... Args>
void launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t stream, Args... args)
{
    static_assert(sizeof...(KArgs) == sizeof...(Args), "one argument per kernel parameter");
    std::tuple<std::remove_cv_t<KArgs>...> vals(static_cast<std::remove_cv_t<KArgs>>(args)...);
    void *ptrs[sizeof...(KArgs)];
    size_t i = 0;
    std::apply([&](auto &...v) { ((ptrs[i++] = static_cast<void *>(&v)), ...); }, vals);
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, ptrs, 0, stream);
    if (e != hipSuccess && t_launch_status == hipSuccess) t_launch_status = e;
}

void launches_begin() { t_launch_status = hipSuccess; }
pa_status launches_end() { return t_launch_status == hipSuccess ? PA_OK : PA_ERR_HIP; }

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
    int32_t steps;   // pa_decode_shared only: which of SHARED_PLAN, SHARED_DECODE to enqueue
    hipStream_t stream;
};

enum SharedSteps { SHARED_PLAN = 1, SHARED_DECODE = 2 };

template <int DT, int D, int B, int W, int MODE>
void launch_decode_kernel(const DecodeArgs &a, unsigned items)
{
    launch((pa_decode_kernel<DT, D, B, W, MODE == MODE_PART ? kPartChunksPerTrip : kChunksPerTrip, MODE>),
                       dim3(items * (unsigned)a.p.H),
                       dim3(W * kWave), a.stream, a.p);
}

enum PlanMode { PLAN_SINGLE = 0, PLAN_PART = 1, PLAN_SHARED = 2 };

// pa_decode_shared: the sharing plan (group discovery and tile lists, one launch), then one launch
// with the groups on the matrix cores and everything else on the ordinary one-pass kernel
template <int DT, int D, int B>
void launch_shared(const DecodeArgs &a)
{
    if constexpr (DT != PA_F32 && D == 128 && B % 16 == 0) {
        const unsigned S = (unsigned)a.p.S;
        if (a.steps & SHARED_PLAN)
            launch(shared_plan_kernel, dim3(kPlanBlocks), dim3(kPlanThreads), a.stream, a.p.block_tables,
                               a.p.max_blocks, a.p.context_lens, a.p.S, B, const_cast<int32_t *>(a.p.ginfo),
                               const_cast<int4 *>(a.p.tiles));
        if (!(a.steps & SHARED_DECODE)) return;
        // groups + singles <= S: one workgroup per (sequence, head) always suffices
        const dim3 grid(S * (unsigned)a.p.H);
        if (a.waves >= 16)
            launch((pa_shared_fused_kernel<DT, B, 16>), grid, dim3(16 * kWave), a.stream, a.p);
        else if (a.waves >= 8)
            launch((pa_shared_fused_kernel<DT, B, 8>), grid, dim3(8 * kWave), a.stream, a.p);
        else
            launch((pa_shared_fused_kernel<DT, B, 4>), grid, dim3(4 * kWave), a.stream, a.p);
    }
}

template <int DT, int D, int B>
void dispatch_mode(const DecodeArgs &a, int mode)
{
    const unsigned S = (unsigned)a.p.S;
    const unsigned rows = S * (unsigned)a.p.H;
    if (mode == PLAN_PART) {
        if (a.waves >= 8)
            launch_decode_kernel<DT, D, B, 8, MODE_PART>(a, S * (unsigned)a.p.max_parts);
        else
            launch_decode_kernel<DT, D, B, 4, MODE_PART>(a, S * (unsigned)a.p.max_parts);
        constexpr unsigned kRowsPerGroup = kReduceWaves * kWave / (D * (DT == PA_F32 ? 4 : 2) / 16);
        launch((pa_reduce_kernel<DT, D>), dim3((rows + kRowsPerGroup - 1) / kRowsPerGroup),
                           dim3(kReduceWaves * kWave), a.stream, a.p);
    } else if (mode == PLAN_SHARED) {
        launch_shared<DT, D, B>(a);
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

// Several queries per sequence.  Up to 16 of them: one workgroup per (sequence, head) whose waves
// split the tiles.  More: one workgroup of four waves per (sequence, block of queries, head) that
// share every tile through LDS, 64 queries per block up to 64 per sequence, 128 beyond.
template <int DT, int B>
void launch_multi_b(const DecodeArgs &a, int max_q_len)
{
    if (max_q_len <= 16) {
        // waves per item as in the single-query kernel: sixteen stream long contexts fastest (OPT-13B
        // shape, 64 sequences of up to 2048 tokens: 178 us against 185 us with eight)
        const dim3 grid((unsigned)a.p.S * (unsigned)a.p.H);
        if (a.waves >= 16)
            launch((pa_multi_split_kernel<DT, B, 16>), grid, dim3(16 * kWave), a.stream, a.p);
        else if (a.waves >= 8)
            launch((pa_multi_split_kernel<DT, B, 8>), grid, dim3(8 * kWave), a.stream, a.p);
        else
            launch((pa_multi_split_kernel<DT, B, 4>), grid, dim3(4 * kWave), a.stream, a.p);
    } else {
        const unsigned blocks = (unsigned)a.p.S * (unsigned)a.p.q_blocks * (unsigned)a.p.H;
        if (max_q_len <= 64)
            launch((pa_multi_block_kernel<DT, B, true, 1>), dim3(blocks), dim3(4 * kWave), a.stream, a.p);
        else if (a.p.q_blocks == 1)
            launch((pa_multi_block_kernel<DT, B, true, 2>), dim3(blocks), dim3(4 * kWave), a.stream, a.p);
        else
            launch((pa_multi_block_kernel<DT, B, false, 2>), dim3(blocks), dim3(4 * kWave), a.stream, a.p);
    }
}

template <int DT>
bool launch_multi(const DecodeArgs &a, int B, int max_q_len)
{
    switch (B) {
    case 16: launch_multi_b<DT, 16>(a, max_q_len); return true;
    case 32: launch_multi_b<DT, 32>(a, max_q_len); return true;
    case 64: launch_multi_b<DT, 64>(a, max_q_len); return true;
    case 128: launch_multi_b<DT, 128>(a, max_q_len); return true;
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

bool shared_on_matrix_cores(pa_dtype dtype, int32_t head_dim, int32_t block_size, int32_t num_seqs)
{
    // the planning kernel keeps its scan state for the whole batch in LDS
    return dtype != PA_F32 && head_dim == 128 && block_size % 16 == 0 && num_seqs <= kPlanMaxSeqs;
}

size_t ginfo_bytes(int32_t S) { return (ginfo_words(S) * sizeof(int32_t) + 15) & ~(size_t)15; }

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
    case PA_ERR_LIMIT: return "needs more scratch than the library's static array holds";
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

// pa_decode proper.  `static_limit` > 0 marks the caller as pa_decode_static: the workspace is
// the library's own static array of that many bytes and a larger need is refused as such.
static pa_status decode_core(void *out, const void *q, const void *k_cache, const void *v_cache,
                             const int32_t *block_tables, int32_t max_blocks_per_seq,
                             const int32_t *context_lens, int32_t num_seqs, int32_t num_heads,
                             int32_t head_dim, int32_t block_size, int64_t num_blocks, pa_dtype dtype,
                             float scale, int32_t max_context_len, int32_t partition_size, void *workspace,
                             size_t workspace_bytes, size_t static_limit, void *stream)
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

    launches_begin();
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
        if (static_limit && need > static_limit) return PA_ERR_LIMIT;
        if (!workspace || workspace_bytes < need) return PA_ERR_WORKSPACE;
        if (!aligned16(workspace)) return PA_ERR_ALIGN;
        if ((int64_t)num_seqs * num_heads * a.p.max_parts > 0x7fffffff) return PA_ERR_SHAPE;
        a.p.ws_acc = static_cast<float *>(workspace);
        a.p.ws_ml = a.p.ws_acc + (size_t)num_seqs * num_heads * a.p.max_parts * head_dim;
    }
    if (!dispatch_decode(a, dtype, head_dim, block_size, partition_size > 0 ? PLAN_PART : PLAN_SINGLE))
        return PA_ERR_UNSUPPORTED;
    return launches_end();
}

pa_status pa_decode(void *out, const void *q, const void *k_cache, const void *v_cache,
                    const int32_t *block_tables, int32_t max_blocks_per_seq,
                    const int32_t *context_lens, int32_t num_seqs, int32_t num_heads,
                    int32_t head_dim, int32_t block_size, int64_t num_blocks, pa_dtype dtype,
                    float scale, int32_t max_context_len, int32_t partition_size, void *workspace,
                    size_t workspace_bytes, void *stream)
{
    return decode_core(out, q, k_cache, v_cache, block_tables, max_blocks_per_seq, context_lens, num_seqs,
                       num_heads, head_dim, block_size, num_blocks, dtype, scale, max_context_len,
                       partition_size, workspace, workspace_bytes, 0, stream);
}

pa_status pa_decode_static(void *out, const void *q, const void *k_cache, const void *v_cache,
                           const int32_t *block_tables, int32_t max_blocks_per_seq,
                           const int32_t *context_lens, int32_t num_seqs, int32_t num_heads,
                           int32_t head_dim, int32_t block_size, int64_t num_blocks, pa_dtype dtype,
                           float scale, int32_t max_context_len, int32_t partition_size, void *stream)
{
    void *ws = nullptr;
    if (num_seqs > 0) {
        const pa_status st = static_scratch(&ws);
        if (st != PA_OK) return st;
    }
    return decode_core(out, q, k_cache, v_cache, block_tables, max_blocks_per_seq, context_lens, num_seqs,
                       num_heads, head_dim, block_size, num_blocks, dtype, scale, max_context_len,
                       partition_size, ws, PA_STATIC_SCRATCH_BYTES, PA_STATIC_SCRATCH_BYTES, stream);
}

size_t pa_decode_shared_workspace_bytes(int32_t num_seqs, int32_t num_heads, int32_t head_dim,
                                        int32_t max_blocks_per_seq)
{
    if (num_seqs <= 0 || num_heads <= 0 || head_dim <= 0 || max_blocks_per_seq <= 0) return 0;
    return ginfo_bytes(num_seqs) + (size_t)num_seqs * max_blocks_per_seq * sizeof(int4);
}

static pa_status decode_shared_steps(int steps, void *out, const void *q, const void *k_cache,
                                     const void *v_cache, const int32_t *block_tables,
                                     int32_t max_blocks_per_seq, const int32_t *context_lens,
                                     int32_t num_seqs, int32_t num_heads, int32_t head_dim,
                                     int32_t block_size, int64_t num_blocks, pa_dtype dtype, float scale,
                                     int32_t max_context_len, void *workspace, size_t workspace_bytes,
                                     void *stream)
{
    if (num_seqs < 0 || num_heads <= 0 || head_dim <= 0 || block_size <= 0 || num_blocks <= 0 ||
        max_blocks_per_seq <= 0 || max_context_len < 0)
        return PA_ERR_SHAPE;
    if (!shape_supported(dtype, head_dim, block_size)) return PA_ERR_UNSUPPORTED;
    if ((int64_t)max_context_len > (int64_t)max_blocks_per_seq * block_size) return PA_ERR_SHAPE;
    if (num_seqs == 0) return PA_OK;
    if (!block_tables || !context_lens) return PA_ERR_NULL;
    if ((steps & SHARED_DECODE) && (!out || !q || !k_cache || !v_cache)) return PA_ERR_NULL;
    if ((steps & SHARED_DECODE) &&
        (!aligned16(out) || !aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache)))
        return PA_ERR_ALIGN;
    if ((int64_t)num_seqs * num_heads > (int64_t)0x7fffffff / 64) return PA_ERR_SHAPE;
    if (!shared_on_matrix_cores(dtype, head_dim, block_size, num_seqs)) {
        // no several-query kernel for this shape: nothing to plan, and the plain one-pass
        // kernel gives the same result
        if (!(steps & SHARED_DECODE)) return PA_OK;
        return pa_decode(out, q, k_cache, v_cache, block_tables, max_blocks_per_seq, context_lens, num_seqs,
                         num_heads, head_dim, block_size, num_blocks, dtype, scale, max_context_len, 0,
                         nullptr, 0, stream);
    }
    const size_t need = pa_decode_shared_workspace_bytes(num_seqs, num_heads, head_dim, max_blocks_per_seq);
    if (!workspace || workspace_bytes < need) return PA_ERR_WORKSPACE;
    if (!aligned16(workspace)) return PA_ERR_ALIGN;

    launches_begin();
    DecodeArgs a;
    memset(&a, 0, sizeof(a));
    fill_common(a, out, q, k_cache, v_cache, block_tables, max_blocks_per_seq, context_lens, num_seqs,
                num_heads, scale, stream);
    a.p.max_parts = 1;
    a.steps = steps;
    a.waves = waves_for(max_context_len, chunk_tokens(dtype, head_dim, block_size));
    a.p.ginfo = static_cast<const int32_t *>(workspace);
    a.p.tiles = reinterpret_cast<const int4 *>(static_cast<const char *>(workspace) + ginfo_bytes(num_seqs));
    if (!dispatch_decode(a, dtype, head_dim, block_size, PLAN_SHARED)) return PA_ERR_UNSUPPORTED;
    return launches_end();
}

pa_status pa_decode_shared(void *out, const void *q, const void *k_cache, const void *v_cache,
                           const int32_t *block_tables, int32_t max_blocks_per_seq,
                           const int32_t *context_lens, int32_t num_seqs, int32_t num_heads,
                           int32_t head_dim, int32_t block_size, int64_t num_blocks, pa_dtype dtype,
                           float scale, int32_t max_context_len, void *workspace,
                           size_t workspace_bytes, void *stream)
{
    return decode_shared_steps(SHARED_PLAN | SHARED_DECODE, out, q, k_cache, v_cache, block_tables,
                               max_blocks_per_seq, context_lens, num_seqs, num_heads, head_dim, block_size,
                               num_blocks, dtype, scale, max_context_len, workspace, workspace_bytes, stream);
}

pa_status pa_shared_plan(const int32_t *block_tables, int32_t max_blocks_per_seq,
                         const int32_t *context_lens, int32_t num_seqs, int32_t num_heads,
                         int32_t head_dim, int32_t block_size, int64_t num_blocks, pa_dtype dtype,
                         int32_t max_context_len, void *workspace, size_t workspace_bytes, void *stream)
{
    return decode_shared_steps(SHARED_PLAN, nullptr, nullptr, nullptr, nullptr, block_tables,
                               max_blocks_per_seq, context_lens, num_seqs, num_heads, head_dim, block_size,
                               num_blocks, dtype, 0.f, max_context_len, workspace, workspace_bytes, stream);
}

pa_status pa_decode_shared_planned(void *out, const void *q, const void *k_cache, const void *v_cache,
                                   const int32_t *block_tables, int32_t max_blocks_per_seq,
                                   const int32_t *context_lens, int32_t num_seqs, int32_t num_heads,
                                   int32_t head_dim, int32_t block_size, int64_t num_blocks,
                                   pa_dtype dtype, float scale, int32_t max_context_len,
                                   const void *plan, size_t plan_bytes, void *stream)
{
    return decode_shared_steps(SHARED_DECODE, out, q, k_cache, v_cache, block_tables, max_blocks_per_seq,
                               context_lens, num_seqs, num_heads, head_dim, block_size, num_blocks, dtype,
                               scale, max_context_len, const_cast<void *>(plan), plan_bytes, stream);
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
    // 64 queries per workgroup up to 64 per sequence, 128 beyond
    const int64_t q_blocks = max_q_len <= 64 ? 1 : (max_q_len + 127) / 128;
    const int64_t blocks = (int64_t)num_seqs * q_blocks * num_heads;
    if (blocks > 0x7fffffff) return PA_ERR_SHAPE;
    launches_begin();
    DecodeArgs a;
    memset(&a, 0, sizeof(a));
    fill_common(a, out, q, k_cache, v_cache, block_tables, max_blocks_per_seq, context_lens, num_seqs,
                num_heads, scale, stream);
    a.p.q_start = q_start;
    a.p.q_blocks = (int32_t)q_blocks;
    a.waves = waves_for(max_context_len, kTileTokens);
    const bool ok = dtype == PA_F16 ? launch_multi<PA_F16>(a, block_size, max_q_len)
                                    : launch_multi<PA_BF16>(a, block_size, max_q_len);
    if (!ok) return PA_ERR_UNSUPPORTED;
    return launches_end();
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
    launches_begin();
    const int32_t frags_per_row = row_bytes / 16;
    const int64_t frags_per_token = (int64_t)frags_per_row * num_heads;
    if (frags_per_token > 0x7fffffff) return PA_ERR_SHAPE;
    const int64_t total = frags_per_token * num_tokens;
    const int64_t groups = (total + 255) / 256;
    if (groups > 0x7fffffff) return PA_ERR_SHAPE;
    launch(reshape_and_cache_kernel, dim3((unsigned)groups, 2), dim3(256),
                       static_cast<hipStream_t>(stream), static_cast<const uint4 *>(k),
                       static_cast<const uint4 *>(v), static_cast<uint4 *>(k_cache),
                       static_cast<uint4 *>(v_cache), slot_mapping, total, (int32_t)frags_per_token,
                       frags_per_row, block_size);
    return launches_end();
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
    launches_begin();
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
            launch(copy_blocks_kernel, dim3(slices, (unsigned)np, (unsigned)(2 * nl)), dim3(256),
                               static_cast<hipStream_t>(stream), ptrs, src_dst_pairs + 2 * (int64_t)p0, frags);
            if (launches_end() != PA_OK) return PA_ERR_HIP;
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
    launches_begin();
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
            launch(swap_blocks_kernel, dim3(slices, (unsigned)np, (unsigned)(2 * nl)), dim3(256),
                               static_cast<hipStream_t>(stream), ptrs, src_dst_pairs + 2 * (int64_t)p0, frags);
            if (launches_end() != PA_OK) return PA_ERR_HIP;
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
    launches_begin();
    const int64_t frags = (int64_t)(bytes / 16);
    const int64_t groups = (frags + kProbeTileFrags - 1) / kProbeTileFrags;
    if (groups > 0x7fffffff) return PA_ERR_SHAPE;
    launch(stream_read_kernel, dim3((unsigned)groups), dim3(256),
                       static_cast<hipStream_t>(stream), static_cast<const char *>(src), frags,
                       static_cast<uint32_t *>(sink));
    return launches_end();
}

} // extern "C"
