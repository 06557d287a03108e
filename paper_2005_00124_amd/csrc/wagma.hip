// libwagma: the per-iteration hot path of WAGMA-SGD (arXiv 2005.00124,
// Algorithm 2 lines 6-17 with the groups of Algorithm 1) for P model replicas
// stored as P rows in one MI355X's HBM.  gfx950 only.
//
// Work decomposition.  Every operation of the step is elementwise in the
// parameter index; only the P rows interact.  A thread therefore owns one
// 16-byte column slice (4 consecutive parameters) of one group and does the
// whole iteration for it: it loads W, G and the momentum of every member row
// (plus the send buffer of late members), applies the local update, sums the
// contributions in butterfly-phase order, and stores W, momentum and send
// buffer.  Each element is read once and written once, by one thread, so the
// in-place update needs no synchronisation, no LDS and no second buffer, and a
// wavefront's accesses are 1 KiB contiguous per row.  The step is bound by HBM
// bandwidth (about 0.25 flop per byte): no matrix cores are involved.
//
// Three kernels cover all group sizes:
//   step_rows_in_registers<S>  S <= 8 member rows are held in registers by one wavefront
//                              (3*S independent 128-bit loads in flight per lane).
//   step_rows_cooperative      S = 16, 32, 64: the S/8 wavefronts of a workgroup hold 8 rows
//                              each in the same way; the octets' sums meet in LDS.
//   step_rows_streamed         larger S (and the per-tensor layout from S = 32): member rows
//                              are streamed 8 at a time (4 when some processes are still
//                              computing), the partial sums kept on a pairwise stack; late
//                              members re-read their own W' from the send buffer they just
//                              wrote (an L2 hit).
// The global average (Algorithm 2 lines 15-16) is the same computation with
// one group of all P ranks in natural order and nobody late.  The same bodies serve the
// per-tensor layout (step_tensors_*) through an address functor, and each kernel has a
// second instantiation (LAG) that also honours the mask of processes still computing.
// The optional allocator lives in wagma_alloc.hip.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "wagma.h"
#include "wagma_internal.h"
#include "wagma_kernels.h"
#include "wagma_masks.h"

namespace {
thread_local int g_last_hip_error = 0;
}  // namespace

namespace wagma_detail {

void set_last_hip_error(hipError_t e)
{
    g_last_hip_error = (int)e;
}

int hip_failed(hipError_t e)
{
    g_last_hip_error = (int)e;
    return WAGMA_EHIP;
}

}  // namespace wagma_detail

using wagma_detail::hip_failed;

namespace {

int exact_log2(int64_t x)
{
    if (x < 1 || (x & (x - 1)) != 0)
        return -1;
    int l = 0;
    while ((int64_t(1) << l) < x)
        ++l;
    return l;
}

int gcd_int(int a, int b)
{
    while (b) {
        const int r = a % b;
        a = b;
        b = r;
    }
    return a;
}

// Everything of a context that needs no memory: the sizes, the row stride, the launch options.
void set_defaults(wagma_ctx* ctx, int P, int S, int G, int g, int64_t n, int tau)
{
    ctx->P = P;
    ctx->S = S;
    ctx->G = G;
    ctx->g = g;
    ctx->tau = tau;
    ctx->n = n;
    ctx->period = (g == 0 || G == 0) ? 1 : G / gcd_int(g, G);
    // Row stride.  Measured on MI355X: the launch shapes that split a wavefront's 1 KiB into two
    // pieces 32 KiB apart (kLaunchShapes) gain what they gain only where the two pieces differ in
    // address bit 15 and nothing else, so rows must begin on 64 KiB boundaries of the arrays, which
    // the allocators put on 2 MiB boundaries (workload with rows at odd multiples of 16 KiB: 6238
    // GB/s, on 64 KiB boundaries: 6615).  With a wavefront's 1 KiB in one piece: rows on 16 KiB
    // boundaries run about 1 % faster than rows on 256 B boundaries (and rows off a 128 B boundary
    // up to 10 % slower), and strides that are a multiple of 1 MiB put all member rows of a group
    // on the same memory channels (20 % slower), so such a stride is skewed by one row alignment.
    // Small models keep the padding small.
    const int64_t row_align = n >= (int64_t(1) << 18) ? 16384 : 64;  // floats
    ctx->ld = (n + row_align - 1) / row_align * row_align;
    if ((ctx->ld * 4) % (int64_t(1) << 20) == 0)
        ctx->ld += row_align;
    // Streaming hints help only when the arrays stream from HBM: four arrays that fit in the
    // 256 MB Infinity Cache together run 6 % faster without them (P=4, n=2^20).
    ctx->opt_nontemporal = (size_t)4 * (size_t)P * (size_t)ctx->ld * sizeof(float) > (size_t(256) << 20) ? 1 : 0;
    ctx->opt_force_stream = 0;
    // Measured best on MI355X (workgroups of 256 threads: three of them fit a compute unit with
    // the S = 8 kernel's registers): the wavefronts of a workgroup 4 KiB apart; how many
    // consecutive tiles an XCD takes is chosen per launch (step_flat).
    ctx->opt_stripe_log2 = 2;
    ctx->stripe_forced = 0;
    ctx->opt_xcd_chunk_log2 = -1;
    ctx->opt_map = 0;
    ctx->opt_tensor_tables = 0;
    ctx->placed_shape = 0;
    ctx->placed_coop_shape = 0;
    ctx->fixed_groups = 0;
    ctx->d_table = nullptr;
    ctx->h_table = nullptr;
    for (int k = 0; k < 4; ++k)
        ctx->placed[k] = nullptr;
    ctx->placed_ld = 0;
    ctx->vmm = nullptr;
    ctx->opt_placement = WAGMA_PLACE_AUTO;
    ctx->place_mode = WAGMA_PLACE_PLAIN;
    ctx->place_candidates = 0;
    ctx->place_regions = 0;
    ctx->place_g_with_w = 0;
    ctx->place_same_gbs = 0.0;
    ctx->place_split_gbs = 0.0;
}

enum class FlatKernel { in_registers, cooperative, streamed };

// LAG: the kernels that also look at the busy mask (chosen only when a bit of it is set).
template <bool NT, bool LAG>
void launch_flat(const StepParams& p, FlatKernel kind, unsigned grid, hipStream_t stream)
{
    const dim3 g(grid), b(kBlock);
    if (kind == FlatKernel::streamed) {
        hipLaunchKernelGGL((step_rows_streamed<NT, LAG>), g, b, 0, stream, p);
        return;
    }
    if (kind == FlatKernel::cooperative) {
        switch (p.members) {
        case 16: hipLaunchKernelGGL((step_rows_cooperative<2, NT, LAG>), g, dim3(128), 0, stream, p); break;
        case 32: hipLaunchKernelGGL((step_rows_cooperative<4, NT, LAG>), g, dim3(256), 0, stream, p); break;
        default: hipLaunchKernelGGL((step_rows_cooperative<8, NT, LAG>), g, dim3(512), 0, stream, p); break;
        }
        return;
    }
    switch (p.members) {
    case 1: hipLaunchKernelGGL((step_rows_in_registers<1, NT, LAG>), g, b, 0, stream, p); break;
    case 2: hipLaunchKernelGGL((step_rows_in_registers<2, NT, LAG>), g, b, 0, stream, p); break;
    case 4: hipLaunchKernelGGL((step_rows_in_registers<4, NT, LAG>), g, b, 0, stream, p); break;
    default: hipLaunchKernelGGL((step_rows_in_registers<8, NT, LAG>), g, b, 0, stream, p); break;
    }
}

}  // namespace

struct wagma_tensors {
    wagma_ctx* ctx;
    int T;
    int64_t tiles;      // workgroups per group
    void* d_blob;       // one device allocation: the tile table, and either its 64-byte entries or the pointers by place
    const TileRef* tile_ref;
    const AffineTile* affine_tile;  // not NULL: the tensors are spaced alike in every array, and the tile
                                    // table exists in this form too (the kernels then read nothing else)
    const SlotPointers* slot_ptrs;  // not NULL: [period + 1][units][P], every tensor's pointers by the places
                                    // of each row of the schedule table (instead of the pointer tables)
    int64_t units;                  // mapped blocks + tensors
    int64_t mapped_tiles;           // the first so many tiles of the tile table belong to mapped blocks
    uint64_t map;       // how the slices of the mapped blocks of the tile table are dealt out (0: no such blocks)
};

namespace {
constexpr int kTensorBlock = kBlock;  // threads per workgroup of the per-tensor kernels
constexpr int64_t kMaxByPlaceBytes = int64_t(4) << 30;  // a plan's pointers by place may take no more than this

template <bool NT, bool LAG, bool AFFINE>
void launch_tensors(const StepParams& p, bool cooperative, unsigned grid, hipStream_t stream)
{
    const dim3 g(grid), b(kTensorBlock);
    if (cooperative) {  // groups of 16: two wavefronts per group
        hipLaunchKernelGGL((step_tensors_cooperative<2, NT, LAG, AFFINE>), g, dim3(128), 0, stream, p);
        return;
    }
    switch (p.members) {
    case 1: hipLaunchKernelGGL((step_tensors_in_registers<1, NT, LAG, AFFINE>), g, b, 0, stream, p); break;
    case 2: hipLaunchKernelGGL((step_tensors_in_registers<2, NT, LAG, AFFINE>), g, b, 0, stream, p); break;
    case 4: hipLaunchKernelGGL((step_tensors_in_registers<4, NT, LAG, AFFINE>), g, b, 0, stream, p); break;
    case 8: hipLaunchKernelGGL((step_tensors_in_registers<8, NT, LAG, AFFINE>), g, b, 0, stream, p); break;
    default: hipLaunchKernelGGL((step_tensors_streamed<NT, LAG, AFFINE>), g, b, 0, stream, p); break;
    }
}

template <bool NT, bool LAG>
void launch_tensors(const StepParams& p, bool cooperative, unsigned grid, hipStream_t stream)
{
    if (p.affine_tile)
        launch_tensors<NT, LAG, true>(p, cooperative, grid, stream);
    else
        launch_tensors<NT, LAG, false>(p, cooperative, grid, stream);
}
}  // namespace

namespace {

// The part of the kernel arguments that both layouts share.  Returns true if some process is
// still computing in this iteration (then the kernels that look at the busy mask are needed).
bool fill_common(const wagma_ctx* ctx, StepParams& p, bool global, const uint64_t* stale_mask,
                 const uint64_t* busy_mask, float lr, float mu, int64_t iter)
{
    std::memset(&p, 0, sizeof(p));
    p.lr = lr;
    p.mu = mu;
    p.members = global ? ctx->P : ctx->S;
    p.inv_members = 1.0f / (float)p.members;
    p.members_plus_1 = (float)(p.members + 1);
    const int32_t* table = nullptr;
    wagma_group_schedule(ctx, iter, &table, nullptr);
    p.table = table;
    if (global)
        return false;  // a global iteration waits for everybody
    const int words = (ctx->P + 63) / 64;
    const uint64_t in_use = ctx->P < 64 ? (UINT64_C(1) << ctx->P) - 1 : ~UINT64_C(0);
    uint64_t any_busy = 0;
    for (int k = 0; k < words; ++k) {
        p.busy[k] = busy_mask ? busy_mask[k] & in_use : 0;
        // a process that is still computing contributes its send buffer like a late one
        p.late[k] = ((stale_mask ? stale_mask[k] : 0) & in_use) | p.busy[k];
        any_busy |= p.busy[k];
    }
    return any_busy != 0;
}

}  // namespace

namespace wagma_detail {

int step_flat(wagma_ctx* ctx, float* w, const float* g, float* m, float* pub, const uint64_t* stale_mask,
              const uint64_t* busy_mask, float lr, float mu, int64_t iter, void* stream, Force force)
{
    int global = wagma_is_global_iteration(ctx, iter);
    if (global < 0)
        return global;
    if (force != Force::none)
        global = force == Force::global ? 1 : 0;
    if (!w || !g || !m || !pub)
        return WAGMA_EINVAL;
    if ((((uintptr_t)w) | ((uintptr_t)g) | ((uintptr_t)m) | ((uintptr_t)pub)) & 15u)
        return WAGMA_EINVAL;
    {
        // every element is read and written by one thread only as long as the four arrays are
        // four different pieces of memory: refuse arrays that overlap
        const uintptr_t at[4] = {(uintptr_t)w, (uintptr_t)g, (uintptr_t)m, (uintptr_t)pub};
        const uintptr_t extent = (uintptr_t)ctx->P * (uintptr_t)ctx->ld * sizeof(float);
        for (int a = 0; a < 4; ++a)
            for (int b = a + 1; b < 4; ++b)
                if (at[a] < at[b] + extent && at[b] < at[a] + extent)
                    return WAGMA_EINVAL;
    }
    int device = -1;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess)
        return hip_failed(e);
    if (device != ctx->device)
        return WAGMA_EINVAL;

    StepParams p;
    const bool lag = fill_common(ctx, p, global != 0, stale_mask, busy_mask, lr, mu, iter);
    if (force == Force::group)
        p.table = ctx->d_table + (ctx->fixed_groups ? 0 : iter % ctx->period) * ctx->P;
    p.w = w;
    p.g = g;
    p.m = m;
    p.pub = pub;
    p.ld = ctx->ld;
    p.nvec = (ctx->n + 3) / 4;

    FlatKernel kind = FlatKernel::in_registers;
    if (p.members > kCooperativeRows || (ctx->opt_force_stream && p.members >= kRegisterRows))
        kind = FlatKernel::streamed;
    else if (p.members > kRegisterRows)
        kind = FlatKernel::cooperative;
    p.stripe_log2 = ctx->opt_stripe_log2;
    p.xcd_chunk_log2 = ctx->opt_xcd_chunk_log2;
    p.map = ctx->opt_map;
    if (p.map == 0 && p.xcd_chunk_log2 < 0 && ctx->stripe_forced) {
        // only the stripe is forced: tile by tile for the kernel that holds a group in registers,
        // the other kernels' usual runs
        p.xcd_chunk_log2 = kind == FlatKernel::in_registers ? 0 : kind == FlatKernel::cooperative ? 3 : 2;
    }
    if (p.map == 0 && p.xcd_chunk_log2 < 0) {
        // Nothing forced: the shape measured best on MI355X (the results do not depend on it).
        // Which shape is best depends on where the arrays lie.  The kernel that holds a group in
        // registers: on arrays whose writes all go to one HBM region (ordinary allocations on a GPU
        // whose memory is otherwise unused) shape 0 runs at 66 % of the peak and the shapes whose
        // wavefronts take 512 B here and 512 B 32 KiB further on at 82 %; on arrays with w, m and
        // pub in three regions all shapes are within 1 % of each other, in an order that changes
        // with the box and the workload.  A caller's arrays get shape 3, within 0.6 % of the best
        // in every case measured; the library's own arrays get what wagma_alloc_buffers measured on
        // them (a forced iteration is that measurement itself).  Groups of 16 to 64 rows, dealt out
        // to the wavefronts of a workgroup: with two wavefronts the split shape gains up to 24 % on
        // arrays in one region and stays within 3 % elsewhere; with four or eight the kernel runs
        // at 5100 GB/s on arrays in one region and at 6380 on arrays in three with its first
        // shape, at 5600 on both with the split one, and the row-streaming kernel with shape 3 at
        // 6180 on both: a caller's arrays get the split shape for groups of 16 and the
        // row-streaming kernel for larger ones.  Groups above 64 rows always run the row-streaming
        // kernel, with shape 3 too (against the 4 KiB stripe with runs of 4 tiles per XCD: 6180
        // against 4970 … 5080 GB/s on arrays in one region, 6180 against 6220 on arrays in three).
        const bool own = force != Force::none || (ctx->placed[0] && w == ctx->placed[0] && g == ctx->placed[1] &&
                                                  m == ctx->placed[2] && pub == ctx->placed[3]);
        LaunchShape shape = kLaunchShapes[kForeignShape];
        if (kind == FlatKernel::in_registers)
            shape = kLaunchShapes[own ? ctx->placed_shape : kForeignShape];
        else if (kind == FlatKernel::cooperative)
            shape = kCoopShapes[own ? ctx->placed_coop_shape : (p.members == 16 ? 1 : 2)];
        if (shape.row_streaming)
            kind = FlatKernel::streamed;
        if (shape.map != 0 && p.nvec <= 64 * kBlock)
            shape = LaunchShape{0u, 2, 0};  // rows shorter than one block of a map (256 KiB): no padding to it
        p.map = shape.map;
        p.stripe_log2 = shape.stripe_log2;
        p.xcd_chunk_log2 = shape.xcd_chunk_log2;
    }
    if (p.xcd_chunk_log2 < 0)
        p.xcd_chunk_log2 = 0;  // a forced map: unused
    p.log2_chunks = kind == FlatKernel::streamed ? exact_log2(p.members / streamed_chunk(lag)) : 0;
    // tiles is rounded up to whole rounds of the launch shape (the surplus lanes find col >= nvec)
    p.tiles = (p.nvec + kBlock - 1) / kBlock;
    int round_log2 = wagma_detail::round_log2_of(p.map, p.stripe_log2, p.xcd_chunk_log2);
    if (kind == FlatKernel::cooperative && round_log2 < 3)
        round_log2 = 3;  // its workgroups take the tiles in rounds of 8
    p.tiles = ((p.tiles + (int64_t(1) << round_log2) - 1) >> round_log2) << round_log2;
    p.blocks = (int64_t)(ctx->P / p.members) * p.tiles;
    if (kind == FlatKernel::cooperative)
        p.blocks *= 4;  // one workgroup per 1 KiB piece of a row instead of per 4 KiB tile
    const int64_t grid = p.blocks;
    if (grid > 0x7fffffff)
        return WAGMA_EINVAL;

    const hipStream_t on = (hipStream_t)stream;
    if (ctx->opt_nontemporal) {
        if (lag)
            launch_flat<true, true>(p, kind, (unsigned)grid, on);
        else
            launch_flat<true, false>(p, kind, (unsigned)grid, on);
    } else {
        if (lag)
            launch_flat<false, true>(p, kind, (unsigned)grid, on);
        else
            launch_flat<false, false>(p, kind, (unsigned)grid, on);
    }
    e = hipGetLastError();
    if (e != hipSuccess)
        return hip_failed(e);
    return WAGMA_OK;
}

}  // namespace wagma_detail

using wagma_detail::step_flat;

extern "C" {

int wagma_create(wagma_ctx** out, int P, int S, int64_t n, int tau)
{
    if (!out)
        return WAGMA_EINVAL;
    *out = nullptr;
    const int G = exact_log2(P), g = exact_log2(S);
    // lanes address their column with a 32-bit float offset inside a row
    if (G < 0 || g < 0 || P > WAGMA_MAX_P || S > P || n < 1 || tau < 0 || n > kMaxN)
        return WAGMA_EINVAL;

    wagma_ctx* ctx = new (std::nothrow) wagma_ctx();
    if (!ctx)
        return WAGMA_ENOMEM;
    set_defaults(ctx, P, S, G, g, n, tau);

    const size_t entries = (size_t)(ctx->period + 1) * (size_t)P;
    hipError_t e = hipGetDevice(&ctx->device);
    if (e != hipSuccess) {
        delete ctx;
        return hip_failed(e);
    }
    ctx->h_table = (int32_t*)std::malloc(entries * sizeof(int32_t));
    if (!ctx->h_table) {
        delete ctx;
        return WAGMA_ENOMEM;
    }
    e = hipMalloc((void**)&ctx->d_table, entries * sizeof(int32_t));
    if (e != hipSuccess) {
        std::free(ctx->h_table);
        delete ctx;
        g_last_hip_error = (int)e;
        return e == hipErrorOutOfMemory ? WAGMA_ENOMEM : WAGMA_EHIP;
    }
    const unsigned threads = 256;
    const unsigned grid = (unsigned)((entries + threads - 1) / threads);
    hipLaunchKernelGGL(build_schedule_table, dim3(grid), dim3(threads), 0, (hipStream_t) nullptr,
                       ctx->d_table, P, G, g, ctx->period);
    e = hipGetLastError();
    if (e == hipSuccess)
        e = hipMemcpy(ctx->h_table, ctx->d_table, entries * sizeof(int32_t), hipMemcpyDeviceToHost);
    if (e != hipSuccess) {
        (void)hipFree(ctx->d_table);
        std::free(ctx->h_table);
        delete ctx;
        return hip_failed(e);
    }
    *out = ctx;
    return WAGMA_OK;
}

int wagma_destroy(wagma_ctx* ctx)
{
    if (!ctx)
        return WAGMA_OK;
    int rc = wagma_free_buffers(ctx);
    if (ctx->d_table) {
        const hipError_t e = hipFree(ctx->d_table);
        if (e != hipSuccess)
            rc = hip_failed(e);
    }
    std::free(ctx->h_table);
    delete ctx;
    return rc;
}

int64_t wagma_row_stride(const wagma_ctx* ctx)
{
    return ctx ? ctx->ld : (int64_t)WAGMA_EINVAL;
}

int wagma_set_row_stride(wagma_ctx* ctx, int64_t ld)
{
    if (!ctx || ld % 4 != 0 || ld < (ctx->n + 3) / 4 * 4 || ld > 2 * kMaxN)
        return WAGMA_EINVAL;
    if (ctx->placed[0] && ld > ctx->placed_ld)
        return WAGMA_EINVAL;  // rows would reach beyond the arrays of wagma_alloc_buffers
    ctx->ld = ld;
    return WAGMA_OK;
}

int wagma_set_grouping(wagma_ctx* ctx, int mode)
{
    if (!ctx || (mode != WAGMA_GROUPING_DYNAMIC && mode != WAGMA_GROUPING_FIXED))
        return WAGMA_EINVAL;
    ctx->fixed_groups = mode == WAGMA_GROUPING_FIXED;
    return WAGMA_OK;
}

int wagma_schedule_period(const wagma_ctx* ctx)
{
    return ctx ? ctx->period : WAGMA_EINVAL;
}

int wagma_is_global_iteration(const wagma_ctx* ctx, int64_t iter)
{
    if (!ctx || iter < 0 || iter == INT64_MAX)
        return WAGMA_EINVAL;
    return wagma_masks::is_global_iteration(ctx->tau, iter) ? 1 : 0;
}

int wagma_group_schedule(const wagma_ctx* ctx, int64_t iter, const int32_t** dev_table,
                         const int32_t** host_table)
{
    const int global = wagma_is_global_iteration(ctx, iter);
    if (global < 0)
        return global;
    const int64_t row = global ? ctx->period : (ctx->fixed_groups ? 0 : iter % ctx->period);
    if (dev_table)
        *dev_table = ctx->d_table + row * ctx->P;
    if (host_table)
        *host_table = ctx->h_table + row * ctx->P;
    return WAGMA_OK;
}

int wagma_step(wagma_ctx* ctx, float* w, const float* g, float* m, float* pub,
               const uint64_t* stale_mask, float lr, float mu, int64_t iter, void* stream)
{
    return step_flat(ctx, w, g, m, pub, stale_mask, nullptr, lr, mu, iter, stream, wagma_detail::Force::none);
}

int wagma_step_lag(wagma_ctx* ctx, float* w, const float* g, float* m, float* pub,
                   const uint64_t* late_mask, const uint64_t* busy_mask, float lr, float mu, int64_t iter,
                   void* stream)
{
    return step_flat(ctx, w, g, m, pub, late_mask, busy_mask, lr, mu, iter, stream, wagma_detail::Force::none);
}

// ---- wagma_step without a context: the schedule table lives in a static device array ------

namespace {

// (period + 1) * P entries with period <= log2 P <= 10 and P <= WAGMA_MAX_P.
constexpr size_t kStaticTableEntries = (size_t)11 * WAGMA_MAX_P;
static_assert(kStaticTableEntries * sizeof(int32_t) == WAGMA_STATIC_TABLE_BYTES, "size stated in wagma.h");
static __device__ __align__(256) int32_t scratch[kStaticTableEntries];

// Device address of `scratch` on each GPU (every GPU holds its own copy of the array); looked up
// once per device, with that device current.  In host code the array's name is not that address.
constexpr int kMaxDevices = 64;
std::atomic<int32_t*> g_static_table[kMaxDevices];

int static_table(int device, int32_t** out)
{
    if (device < 0 || device >= kMaxDevices)
        return WAGMA_EINVAL;
    int32_t* ptr = g_static_table[device].load(std::memory_order_acquire);
    if (!ptr) {
        const hipError_t e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess)
            return hip_failed(e);
        if (!ptr)
            return WAGMA_EHIP;
        g_static_table[device].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return WAGMA_OK;
}

}  // namespace

int wagma_step_static(int P, int S, int64_t n, int tau, int64_t ld, float* w, const float* g, float* m,
                      float* pub, const uint64_t* stale_mask, float lr, float mu, int64_t iter, void* stream)
{
    const int G = exact_log2(P), log2_S = exact_log2(S);
    if (G < 0 || log2_S < 0 || P > WAGMA_MAX_P || S > P || n < 1 || tau < 0 || n > kMaxN)
        return WAGMA_EINVAL;
    wagma_ctx ctx;  // on the stack: nothing of it outlives the call
    set_defaults(&ctx, P, S, G, log2_S, n, tau);
    if ((size_t)(ctx.period + 1) * (size_t)P > kStaticTableEntries)
        return WAGMA_EINVAL;  // cannot happen while P <= WAGMA_MAX_P; the array's size is the limit
    if (ld != 0) {
        if (ld % 4 != 0 || ld < (n + 3) / 4 * 4 || ld > 2 * kMaxN)
            return WAGMA_EINVAL;
        ctx.ld = ld;
    }
    if (iter < 0 || iter == INT64_MAX || !w || !g || !m || !pub)
        return WAGMA_EINVAL;
    if ((((uintptr_t)w) | ((uintptr_t)g) | ((uintptr_t)m) | ((uintptr_t)pub)) & 15u)
        return WAGMA_EINVAL;
    hipError_t e = hipGetDevice(&ctx.device);
    if (e != hipSuccess)
        return hip_failed(e);
    int rc = static_table(ctx.device, &ctx.d_table);
    if (rc != WAGMA_OK)
        return rc;
    // The table of this (P, S) overwrites whatever the last call on this GPU left there, on the
    // caller's stream, ahead of the step that reads it.
    const unsigned entries = (unsigned)((ctx.period + 1) * P), threads = 256;
    hipLaunchKernelGGL(build_schedule_table, dim3((entries + threads - 1) / threads), dim3(threads), 0,
                       (hipStream_t)stream, ctx.d_table, P, G, log2_S, ctx.period);
    e = hipGetLastError();
    if (e != hipSuccess)
        return hip_failed(e);
    return step_flat(&ctx, w, g, m, pub, stale_mask, nullptr, lr, mu, iter, stream, wagma_detail::Force::none);
}

// ---- per-tensor layout ------------------------------------------------------------------

namespace {

// The plan for T tensors as they are given (arguments already checked: see wagma_tensors_create).
int create_plan(wagma_ctx* ctx, wagma_tensors** out, int T, const int64_t* sizes, float* const* w,
                const float* const* g, float* const* m, float* const* pub)
{
    // Every whole 256 KiB of a tensor becomes a mapped block whose slices are dealt out by the launch
    // shape for a caller's arrays (a plan's tensors are always the caller's), as in the flat layout;
    // the rest is contiguous 4 KiB tiles in runs of 8 per XCD (measured best: tile by tile is 2-5 %
    // slower on every kind of array); wagma_tiles.h builds the table.  Forcing a stripe or an XCD
    // run length switches the blocks off, forcing a map chooses theirs.
    const uint64_t block_map = ctx->opt_map != 0 ? ctx->opt_map
                               : (ctx->opt_xcd_chunk_log2 >= 0 || ctx->stripe_forced)
                                   ? 0
                                   : wagma_detail::kLaunchShapes[wagma_detail::kForeignShape].map;
    const int xcd_chunk_log2 = ctx->opt_xcd_chunk_log2 < 0 ? 2 : ctx->opt_xcd_chunk_log2;
    const int run_log2 = xcd_chunk_log2 > 0 ? (xcd_chunk_log2 < 7 ? xcd_chunk_log2 + 1 : 8) : 0;
    std::vector<TileRef> table;
    int64_t tiles = 0, mapped_tiles = 0;
    try {
        // a tensor's address modulo 64 KiB, if it is the same in every process and array
        std::vector<int> phase((size_t)T);
        for (int k = 0; k < T; ++k) {
            const uintptr_t first = (uintptr_t)w[k] & 65535u;
            bool same = true;
            for (int r = 0; r < ctx->P && same; ++r) {
                const size_t i = (size_t)r * T + k;
                same = ((uintptr_t)w[i] & 65535u) == first && ((uintptr_t)g[i] & 65535u) == first &&
                       ((uintptr_t)m[i] & 65535u) == first && ((uintptr_t)pub[i] & 65535u) == first;
            }
            phase[(size_t)k] = same ? (int)first : -1;
        }
        mapped_tiles = wagma_detail::build_tile_table(T, sizes, phase.data(), block_map, run_log2, table);
        tiles = (int64_t)table.size();
    } catch (const std::bad_alloc&) {
        return WAGMA_ENOMEM;
    }
    if (tiles * (int64_t)ctx->P > 0x7fffffff)
        return WAGMA_EINVAL;
    int device = -1;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess)
        return hip_failed(e);
    if (device != ctx->device)
        return WAGMA_EINVAL;

    // Where the replicas of every tensor are spaced alike in all four arrays, every tile's entry
    // also names its tensor's place, and the kernels look nothing else up.  Else every tensor's
    // pointers are laid out by the places of each row of the schedule table, once per mapped block
    // and once per tensor: a workgroup of a mapped block then asks for them by its own number,
    // together with its tile's entry and the ranks.
    const void* const* arrays[4] = {(const void* const*)w, (const void* const*)g, (const void* const*)m,
                                    (const void* const*)pub};
    std::vector<int64_t> step_bytes;
    std::vector<SlotPointers> by_place;
    bool affine = false;
    int64_t units = 0;
    try {
        affine = !ctx->opt_tensor_tables && wagma_detail::spaced_alike(ctx->P, T, arrays, step_bytes);
        if (!affine) {
            const int rows = ctx->period + 1;
            if (((mapped_tiles >> 6) + T) * rows * ctx->P * (int64_t)sizeof(SlotPointers) > kMaxByPlaceBytes)
                return WAGMA_ENOMEM;
            units = wagma_detail::build_slot_pointers(ctx->P, T, rows, ctx->h_table, table, mapped_tiles, arrays,
                                                      by_place);
        }
    } catch (const std::bad_alloc&) {
        return WAGMA_ENOMEM;
    }

    // blob layout: [tiles tile refs][tiles 64-byte entries, if the tensors are spaced alike, else
    // the pointers by place]; every part 64-byte aligned
    const size_t refs_bytes = ((size_t)tiles * sizeof(TileRef) + 63) / 64 * 64;
    const size_t affine_bytes = affine ? (size_t)tiles * sizeof(AffineTile) : 0;
    const size_t by_place_bytes = by_place.size() * sizeof(SlotPointers);
    const size_t blob_bytes = refs_bytes + affine_bytes + by_place_bytes;
    char* host = (char*)std::malloc(blob_bytes);
    wagma_tensors* plan = new (std::nothrow) wagma_tensors();
    if (!host || !plan) {
        std::free(host);
        delete plan;
        return WAGMA_ENOMEM;
    }
    std::memset(host, 0, blob_bytes);
    std::memcpy(host, table.data(), (size_t)tiles * sizeof(TileRef));
    if (affine) {
        AffineTile* entries = (AffineTile*)(host + refs_bytes);
        for (int64_t i = 0; i < tiles; ++i) {
            const TileRef& ref = table[(size_t)i];
            const int k = ref.tensor;  // an empty tile names tensor 0 and touches nothing
            entries[i] = AffineTile{ref, step_bytes[(size_t)k] / (int64_t)sizeof(float), w[k], g[k], m[k], pub[k], 0};
        }
    } else {
        std::memcpy(host + refs_bytes, by_place.data(), by_place_bytes);
    }
    char* dev = nullptr;
    e = hipMalloc((void**)&dev, blob_bytes);
    if (e == hipSuccess)
        e = hipMemcpy(dev, host, blob_bytes, hipMemcpyHostToDevice);
    std::free(host);
    if (e != hipSuccess) {
        if (dev)
            (void)hipFree(dev);
        delete plan;
        g_last_hip_error = (int)e;
        return e == hipErrorOutOfMemory ? WAGMA_ENOMEM : WAGMA_EHIP;
    }
    plan->ctx = ctx;
    plan->T = T;
    plan->tiles = tiles;
    plan->d_blob = dev;
    plan->tile_ref = (const TileRef*)dev;
    plan->affine_tile = affine ? (const AffineTile*)(dev + refs_bytes) : nullptr;
    plan->slot_ptrs = affine ? nullptr : (const SlotPointers*)(dev + refs_bytes);
    plan->units = units;
    plan->mapped_tiles = mapped_tiles;
    plan->map = block_map;
    *out = plan;
    return WAGMA_OK;
}

}  // namespace

int wagma_tensors_create(wagma_ctx* ctx, wagma_tensors** out, int T, const int64_t* sizes,
                         float* const* w, const float* const* g, float* const* m, float* const* pub)
{
    if (!out)
        return WAGMA_EINVAL;
    *out = nullptr;
    if (!ctx || T < 1 || T > (1 << 20) || !sizes || !w || !g || !m || !pub)
        return WAGMA_EINVAL;
    const size_t slots = (size_t)ctx->P * (size_t)T;
    for (size_t i = 0; i < slots; ++i) {
        if (!w[i] || !g[i] || !m[i] || !pub[i])
            return WAGMA_EINVAL;
        if ((((uintptr_t)w[i]) | ((uintptr_t)g[i]) | ((uintptr_t)m[i]) | ((uintptr_t)pub[i])) & 15u)
            return WAGMA_EINVAL;
    }
    int64_t total = 0;
    for (int k = 0; k < T; ++k) {
        if (sizes[k] < 1 || sizes[k] > kMaxN)
            return WAGMA_EINVAL;
        total += sizes[k];
    }
    if (total != ctx->n)
        return WAGMA_EINVAL;
    if (ctx->opt_tensor_tables)
        return create_plan(ctx, out, T, sizes, w, g, m, pub);
    // The step works element by element and knows no tensor boundaries: tensors that follow one
    // another without a gap, in every array of every process (views into one buffer per process),
    // are one tensor to it.  Fewer, longer tensors leave fewer short ends outside the mapped blocks.
    try {
        const void* const* arrays[4] = {(const void* const*)w, (const void* const*)g, (const void* const*)m,
                                        (const void* const*)pub};
        std::vector<int> first_of;
        std::vector<int64_t> joined_sizes;
        wagma_detail::join_tensors(ctx->P, T, sizes, arrays, first_of, joined_sizes);
        const int J = (int)first_of.size();
        if (J == T)
            return create_plan(ctx, out, T, sizes, w, g, m, pub);
        std::vector<const void*> joined[4];
        for (int a = 0; a < 4; ++a) {
            joined[a].resize((size_t)ctx->P * J);
            for (int r = 0; r < ctx->P; ++r)
                for (int j = 0; j < J; ++j)
                    joined[a][(size_t)r * J + j] = arrays[a][(size_t)r * T + first_of[(size_t)j]];
        }
        return create_plan(ctx, out, J, joined_sizes.data(), (float* const*)joined[0].data(),
                           (const float* const*)joined[1].data(), (float* const*)joined[2].data(),
                           (float* const*)joined[3].data());
    } catch (const std::bad_alloc&) {
        return WAGMA_ENOMEM;
    }
}

int wagma_tensors_destroy(wagma_tensors* plan)
{
    if (!plan)
        return WAGMA_OK;
    int rc = WAGMA_OK;
    const hipError_t e = hipFree(plan->d_blob);
    if (e != hipSuccess)
        rc = hip_failed(e);
    delete plan;
    return rc;
}

int wagma_step_tensors(wagma_ctx* ctx, const wagma_tensors* plan, const uint64_t* stale_mask, float lr,
                       float mu, int64_t iter, void* stream)
{
    return wagma_step_tensors_lag(ctx, plan, stale_mask, nullptr, lr, mu, iter, stream);
}

int wagma_step_tensors_lag(wagma_ctx* ctx, const wagma_tensors* plan, const uint64_t* late_mask,
                           const uint64_t* busy_mask, float lr, float mu, int64_t iter, void* stream)
{
    const int global = wagma_is_global_iteration(ctx, iter);
    if (global < 0)
        return global;
    if (!plan || plan->ctx != ctx)
        return WAGMA_EINVAL;
    int device = -1;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess)
        return hip_failed(e);
    if (device != ctx->device)
        return WAGMA_EINVAL;

    StepParams p;
    const bool lag = fill_common(ctx, p, global != 0, late_mask, busy_mask, lr, mu, iter);
    p.tile_ref = plan->tile_ref;
    p.affine_tile = plan->affine_tile;
    // this iteration's row of the schedule table, and the pointers laid out by its places
    p.slot_ptrs = plan->slot_ptrs ? plan->slot_ptrs + (p.table - ctx->d_table) / ctx->P * plan->units * ctx->P : nullptr;
    p.mapped_tiles = plan->mapped_tiles;
    p.map = plan->map;
    p.num_ranks = ctx->P;
    p.tiles = plan->tiles;  // a multiple of 8 (whole XCD rounds)
    p.blocks = (int64_t)(ctx->P / p.members) * p.tiles;
    // Measured (bench.py --tensors --S k --tau 0): with 2 wavefronts per group the cooperative kernel
    // beats the row-streaming one (6093 against 5916 GB/s through the pointer tables); with 4 and 8
    // it loses, through the pointer tables (5157 against 5689, 4539 against 5617) and also where
    // the tile's entry names the tensor's place (5944 against 6058, 5680 against 6100): on arrays
    // that the library did not place the flat layout, too, takes the row-streaming kernel there.
    const bool cooperative = p.members == 2 * kRegisterRows && !ctx->opt_force_stream;
    if (cooperative)
        p.blocks *= 4;  // one workgroup per quarter tile
    if (p.blocks > 0x7fffffff)
        return WAGMA_EINVAL;
    p.log2_chunks = p.members > kRegisterRows && !cooperative ? exact_log2(p.members / streamed_chunk(lag)) : 0;
    const hipStream_t on = (hipStream_t)stream;
    if (ctx->opt_nontemporal) {
        if (lag)
            launch_tensors<true, true>(p, cooperative, (unsigned)p.blocks, on);
        else
            launch_tensors<true, false>(p, cooperative, (unsigned)p.blocks, on);
    } else {
        if (lag)
            launch_tensors<false, true>(p, cooperative, (unsigned)p.blocks, on);
        else
            launch_tensors<false, false>(p, cooperative, (unsigned)p.blocks, on);
    }
    e = hipGetLastError();
    if (e != hipSuccess)
        return hip_failed(e);
    return WAGMA_OK;
}

int wagma_stale_mask(const wagma_ctx* ctx, uint64_t seed, int64_t iter, uint32_t threshold,
                     uint64_t* mask_words)
{
    if (!ctx || iter < 0 || !mask_words)
        return WAGMA_EINVAL;
    wagma_masks::bernoulli(ctx->P, seed, iter, threshold, mask_words);
    return WAGMA_OK;
}

int wagma_straggler_mask(const wagma_ctx* ctx, uint64_t seed, int64_t iter, int count,
                         uint64_t* mask_words)
{
    if (!ctx || iter < 0 || count < 0 || count > ctx->P || !mask_words)
        return WAGMA_EINVAL;
    wagma_masks::stragglers(ctx->P, ctx->G, seed, iter, count, mask_words);
    return WAGMA_OK;
}

int wagma_clock_mask(const wagma_ctx* ctx, uint64_t seed, int64_t iter, uint32_t tolerance_ms,
                     uint64_t* mask_words, uint32_t* step_ms)
{
    if (!ctx || iter < 0 || !mask_words)
        return WAGMA_EINVAL;
    try {
        wagma_masks::clock(ctx->P, seed, iter, tolerance_ms, mask_words, step_ms);
    } catch (const std::bad_alloc&) {
        return WAGMA_ENOMEM;
    }
    return WAGMA_OK;
}

int wagma_lag_masks(const wagma_ctx* ctx, uint64_t seed, int64_t iter, int window, uint32_t tolerance_ms,
                    uint64_t* late_words, uint64_t* busy_words)
{
    if (!ctx || iter < 0 || iter > INT64_MAX - 4 || !late_words || !busy_words ||
        tolerance_ms >= wagma_masks::kShortestStepMs || (ctx->tau == 0 && window < 1))
        return WAGMA_EINVAL;
    try {
        wagma_masks::lag(ctx->P, ctx->tau, window, seed, iter, tolerance_ms, late_words, busy_words);
    } catch (const std::bad_alloc&) {
        return WAGMA_ENOMEM;
    }
    return WAGMA_OK;
}

int wagma_set_option(wagma_ctx* ctx, int option, int64_t value)
{
    if (!ctx)
        return WAGMA_EINVAL;
    switch (option) {
    case WAGMA_OPT_NONTEMPORAL:
        ctx->opt_nontemporal = value != 0;
        return WAGMA_OK;
    case WAGMA_OPT_PLACEMENT:
        if (value < WAGMA_PLACE_PLAIN || value > WAGMA_PLACE_SEARCH)
            return WAGMA_EINVAL;
        ctx->opt_placement = (int)value;
        return WAGMA_OK;
    default:
        return WAGMA_EINVAL;
    }
}

// Not part of include/wagma.h: launch-shape switches for the tests and for measurements
// (declared in wagma_internal.h).  Results never depend on them.
int wagma_debug_set_option(wagma_ctx* ctx, int option, int64_t value)
{
    if (!ctx)
        return WAGMA_EINVAL;
    switch (option) {
    case WAGMA_DEBUG_FORCE_STREAM:
        ctx->opt_force_stream = value != 0;
        return WAGMA_OK;
    case WAGMA_DEBUG_STRIPE_LOG2:
        if (value < 0 || value > 16)
            return WAGMA_EINVAL;
        ctx->opt_stripe_log2 = (int)value;
        ctx->stripe_forced = 1;
        return WAGMA_OK;
    case WAGMA_DEBUG_XCD_CHUNK_LOG2:
        if (value < -1 || value > 13)
            return WAGMA_EINVAL;
        ctx->opt_xcd_chunk_log2 = (int)value;
        return WAGMA_OK;
    case WAGMA_DEBUG_PLACED_SHAPE:
        if (value < 0 || value >= wagma_detail::kNumLaunchShapes)
            return WAGMA_EINVAL;
        ctx->placed_shape = (int)value;
        return WAGMA_OK;
    case WAGMA_DEBUG_PLACED_COOP_SHAPE:
        if (value < 0 || value >= wagma_detail::kNumCoopShapes)
            return WAGMA_EINVAL;
        ctx->placed_coop_shape = (int)value;
        return WAGMA_OK;
    case WAGMA_DEBUG_TENSOR_TABLES:
        if (value != 0 && value != 1)
            return WAGMA_EINVAL;
        ctx->opt_tensor_tables = (int)value;
        return WAGMA_OK;
    case WAGMA_DEBUG_MAP:
        if (value < 0 || !wagma_detail::valid_map((uint64_t)value))
            return WAGMA_EINVAL;
        ctx->opt_map = (uint64_t)value;
        return WAGMA_OK;
    default:
        return wagma_set_option(ctx, option, value);
    }
}

int wagma_debug_get_option(const wagma_ctx* ctx, int option, int64_t* value)
{
    if (!ctx || !value)
        return WAGMA_EINVAL;
    switch (option) {
    case WAGMA_OPT_NONTEMPORAL: *value = ctx->opt_nontemporal; return WAGMA_OK;
    case WAGMA_OPT_PLACEMENT: *value = ctx->opt_placement; return WAGMA_OK;
    case WAGMA_DEBUG_FORCE_STREAM: *value = ctx->opt_force_stream; return WAGMA_OK;
    case WAGMA_DEBUG_STRIPE_LOG2: *value = ctx->opt_stripe_log2; return WAGMA_OK;
    case WAGMA_DEBUG_XCD_CHUNK_LOG2: *value = ctx->opt_xcd_chunk_log2; return WAGMA_OK;
    case WAGMA_DEBUG_PLACED_SHAPE: *value = ctx->placed_shape; return WAGMA_OK;
    case WAGMA_DEBUG_PLACED_COOP_SHAPE: *value = ctx->placed_coop_shape; return WAGMA_OK;
    case WAGMA_DEBUG_MAP: *value = (int64_t)ctx->opt_map; return WAGMA_OK;
    case WAGMA_DEBUG_TENSOR_TABLES: *value = ctx->opt_tensor_tables; return WAGMA_OK;
    default: return WAGMA_EINVAL;
    }
}

const char* wagma_strerror(int code)
{
    switch (code) {
    case WAGMA_OK: return "success";
    case WAGMA_EINVAL: return "invalid argument";
    case WAGMA_EHIP: return "HIP runtime error (see wagma_last_hip_error)";
    case WAGMA_ENOMEM: return "out of memory";
    default: return "unknown libwagma error";
    }
}

int wagma_last_hip_error(void)
{
    return g_last_hip_error;
}

}  // extern "C"
