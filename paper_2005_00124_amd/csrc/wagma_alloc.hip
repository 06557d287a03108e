// libwagma, the optional allocator: wagma_alloc_buffers places the four P x ld arrays in HBM so
// that the step runs fast (what is measured and why it matters is told in wagma_placement.h and
// wagma_chunks.h, whose searches run here against the real memory).  Nothing in the step
// depends on this file: a caller may always bring its own buffers.  gfx950 only.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <new>

#include "wagma.h"
#include "wagma_internal.h"
#include "wagma_placement.h"
#include "wagma_chunks.h"

using wagma_detail::hip_failed;
using wagma_detail::step_flat;

// (global scope: the context holds a pointer to it)
// Arrays built from 1 GiB physical chunks through the HIP virtual memory API (wagma_chunks.h).
struct VmmArrays {
    char* va[4] = {nullptr, nullptr, nullptr, nullptr};  // w, g, m, pub
    size_t va_bytes = 0;                                  // per array: chunks * 1 GiB
    int chunks = 0;                                       // per array
    hipMemGenericAllocationHandle_t* handle[4] = {nullptr, nullptr, nullptr, nullptr};
};

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
constexpr int kMaskWords = WAGMA_MAX_P / 64;

// ---- the HIP side of the region search (wagma_placement.h) ---------------------------------

// Writes four streams through `a` and four through `b`; fast exactly when a and b lie in
// different HBM regions.
__global__ void __launch_bounds__(256) placement_probe(float* a, float* b, uint32_t vec_per_stream)
{
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i >= vec_per_stream)
        return;
    const v4f zero = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (uint32_t k = 0; k < 4; ++k) {
        __builtin_nontemporal_store(zero, reinterpret_cast<v4f*>(a) + (size_t)k * vec_per_stream + i);
        __builtin_nontemporal_store(zero, reinterpret_cast<v4f*>(b) + (size_t)k * vec_per_stream + i);
    }
}

struct HipMemory {
    hipEvent_t start = nullptr, stop = nullptr;
    size_t reserve = 0;  // free memory to leave untouched

    bool init()
    {
        return hipEventCreate(&start) == hipSuccess && hipEventCreate(&stop) == hipSuccess;
    }
    ~HipMemory()
    {
        if (start)
            (void)hipEventDestroy(start);
        if (stop)
            (void)hipEventDestroy(stop);
    }
    char* allocate(size_t bytes)
    {
        size_t free_b = 0, total_b = 0;
        if (hipMemGetInfo(&free_b, &total_b) != hipSuccess || free_b < bytes + reserve)
            return nullptr;
        char* c = nullptr;
        if (hipMalloc((void**)&c, bytes) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        return c;
    }
    void release(char* c) { (void)hipFree(c); }
    // GB/s of the probe writing side_bytes through a and through b; best of three timed runs.
    double rate(char* a, char* b, size_t side_bytes)
    {
        const uint32_t vec = (uint32_t)(side_bytes / 4 / 16);
        const unsigned grid = (vec + 255) / 256;
        float best_ms = 1e30f;
        for (int rep = 0; rep < 4; ++rep) {
            if (hipEventRecord(start, nullptr) != hipSuccess)
                return -1.0;
            hipLaunchKernelGGL(placement_probe, dim3(grid), dim3(256), 0, (hipStream_t) nullptr, (float*)a,
                               (float*)b, vec);
            if (hipEventRecord(stop, nullptr) != hipSuccess || hipEventSynchronize(stop) != hipSuccess)
                return -1.0;
            float ms = 0.0f;
            if (hipEventElapsedTime(&ms, start, stop) != hipSuccess)
                return -1.0;
            if (rep > 0 && ms < best_ms)
                best_ms = ms;
        }
        return 2.0 * 4.0 * 16.0 * (double)vec / (best_ms * 1e-3) / 1e9;
    }
};

void free_vmm_arrays(VmmArrays* arrays)
{
    if (!arrays)
        return;
    for (int a = 0; a < 4; ++a) {
        if (arrays->va[a]) {
            for (int j = 0; j < arrays->chunks; ++j) {  // each chunk exactly as it was mapped
                (void)hipMemUnmap(arrays->va[a] + (size_t)j * wagma_placement::kChunkBytes,
                                  wagma_placement::kChunkBytes);
                (void)hipMemRelease(arrays->handle[a][j]);
            }
            (void)hipMemAddressFree(arrays->va[a], arrays->va_bytes);
        }
        delete[] arrays->handle[a];
    }
    delete arrays;
}

// The Memory of wagma_placement::ChunkSearch: chunks are created one by one and mapped side by
// side into one scratch window of virtual addresses, where the probe can reach them.
struct VmmMemory {
    static constexpr size_t kChunk = wagma_placement::kChunkBytes;
    static constexpr size_t kVaAlign = size_t(1) << 21;
    int device = 0;
    HipMemory prober;     // events + the probe kernel
    char* scratch = nullptr;
    size_t scratch_bytes = 0;
    hipMemGenericAllocationHandle_t handle[wagma_placement::kMaxChunks];
    bool mapped[wagma_placement::kMaxChunks];
    int n = 0;
    void* spacer[64];
    int n_spacers = 0;
    size_t reserve = 0;  // free memory to leave to the caller

    hipMemAllocationProp prop() const
    {
        hipMemAllocationProp p = {};
        p.type = hipMemAllocationTypePinned;
        p.location.type = hipMemLocationTypeDevice;
        p.location.id = device;
        return p;
    }
    hipMemAccessDesc access() const
    {
        hipMemAccessDesc d = {};
        d.location.type = hipMemLocationTypeDevice;
        d.location.id = device;
        d.flags = hipMemAccessFlagsProtReadWrite;
        return d;
    }
    bool init(int dev)
    {
        device = dev;
        int supported = 0;
        if (hipDeviceGetAttribute(&supported, hipDeviceAttributeVirtualMemoryManagementSupported, dev) != hipSuccess ||
            !supported)
            return false;
        const hipMemAllocationProp p = prop();
        size_t granularity = 0;
        if (hipMemGetAllocationGranularity(&granularity, &p, hipMemAllocationGranularityRecommended) != hipSuccess ||
            granularity == 0 || kChunk % granularity != 0)
            return false;
        if (!prober.init())
            return false;
        scratch_bytes = (size_t)wagma_placement::kMaxChunks * kChunk;
        void* va = nullptr;
        if (hipMemAddressReserve(&va, scratch_bytes, kVaAlign, nullptr, 0) != hipSuccess) {
            (void)hipGetLastError();
            return false;
        }
        scratch = (char*)va;
        return true;
    }
    char* new_chunk()
    {
        if (n >= wagma_placement::kMaxChunks)
            return nullptr;
        size_t free_b = 0, total_b = 0;
        if (hipMemGetInfo(&free_b, &total_b) != hipSuccess || free_b < kChunk + reserve)
            return nullptr;
        const hipMemAllocationProp p = prop();
        if (hipMemCreate(&handle[n], kChunk, &p, 0) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        char* at = scratch + (size_t)n * kChunk;
        const hipMemAccessDesc d = access();
        if (hipMemMap(at, kChunk, 0, handle[n], 0) != hipSuccess) {
            (void)hipGetLastError();
            (void)hipMemRelease(handle[n]);
            return nullptr;
        }
        if (hipMemSetAccess(at, kChunk, &d, 1) != hipSuccess) {
            (void)hipGetLastError();
            (void)hipMemUnmap(at, kChunk);
            (void)hipMemRelease(handle[n]);
            return nullptr;
        }
        mapped[n] = true;
        ++n;
        return at;
    }
    bool skip(size_t bytes, size_t keep)
    {
        size_t free_b = 0, total_b = 0;
        if (n_spacers >= 64 || hipMemGetInfo(&free_b, &total_b) != hipSuccess || free_b < bytes + keep + reserve)
            return false;
        if (hipMalloc(&spacer[n_spacers], bytes) != hipSuccess) {
            (void)hipGetLastError();
            return false;
        }
        ++n_spacers;
        return true;
    }
    double rate(char* a, char* b, size_t side) { return prober.rate(a, b, side); }

    // Moves the chunks of `plan` out of the scratch window into four arrays of their own.
    VmmArrays* build(const wagma_placement::ChunkPlan& plan)
    {
        VmmArrays* out = new (std::nothrow) VmmArrays();
        if (!out)
            return nullptr;
        out->chunks = plan.per_array;
        out->va_bytes = (size_t)plan.per_array * kChunk;
        const int* index[4] = {plan.w, plan.g, plan.m, plan.pub};
        const hipMemAccessDesc d = access();
        bool ok = (hipDeviceSynchronize() == hipSuccess);
        for (int a = 0; a < 4 && ok; ++a) {
            out->handle[a] = new (std::nothrow) hipMemGenericAllocationHandle_t[plan.per_array];
            void* va = nullptr;
            ok = out->handle[a] && hipMemAddressReserve(&va, out->va_bytes, kVaAlign, nullptr, 0) == hipSuccess;
            if (!ok)
                break;
            int done = 0;  // chunks of this array that are mapped at their new place
            while (done < plan.per_array) {
                const int i = index[a][done];
                if (hipMemUnmap(scratch + (size_t)i * kChunk, kChunk) != hipSuccess) {
                    ok = false;  // chunk i stays where it was; the destructor returns it
                    break;
                }
                mapped[i] = false;
                if (hipMemMap((char*)va + (size_t)done * kChunk, kChunk, 0, handle[i], 0) != hipSuccess) {
                    (void)hipMemRelease(handle[i]);
                    taken[i] = true;
                    ok = false;
                    break;
                }
                out->handle[a][done] = handle[i];
                taken[i] = true;
                ++done;
            }
            if (ok)
                ok = hipMemSetAccess(va, out->va_bytes, &d, 1) == hipSuccess;
            if (ok) {
                out->va[a] = (char*)va;
            } else {
                // undo this array: unmap and release what was moved, free its addresses
                for (int j = 0; j < done; ++j) {
                    (void)hipMemUnmap((char*)va + (size_t)j * kChunk, kChunk);
                    (void)hipMemRelease(out->handle[a][j]);
                }
                (void)hipMemAddressFree(va, out->va_bytes);
            }
        }
        if (!ok) {
            (void)hipGetLastError();
            free_vmm_arrays(out);
            return nullptr;
        }
        return out;
    }
    bool taken[wagma_placement::kMaxChunks] = {};

    ~VmmMemory()
    {
        // everything that did not go into an array goes back
        for (int i = 0; i < n; ++i) {
            if (taken[i])
                continue;
            if (mapped[i])
                (void)hipMemUnmap(scratch + (size_t)i * kChunk, kChunk);
            (void)hipMemRelease(handle[i]);
        }
        for (int k = 0; k < n_spacers; ++k)
            (void)hipFree(spacer[k]);
        if (scratch)
            (void)hipMemAddressFree(scratch, scratch_bytes);
    }
};

void report_search(const wagma_placement::RegionSearch<HipMemory>& rs)
{
    std::fprintf(stderr, "wagma placement: %d candidates, threshold %.0f GB/s, w=%d g=%d m=%d pub=%d\n",
                 rs.count(), rs.threshold(), rs.role_w(), rs.role_g(), rs.role_m(), rs.role_pub());
    for (int i = 0; i < rs.count(); ++i) {
        std::fprintf(stderr, "  cand %2d %p inner %.0f cross:", i, (void*)rs.candidate(i), rs.inner_rate(i));
        for (int j = 0; j < rs.count(); ++j)
            if (rs.cross_rate(i, j) != 0.0)
                std::fprintf(stderr, " %d:%.0f", j, rs.cross_rate(i, j));
        std::fprintf(stderr, "\n");
    }
}

// ---- candidate placements of the four arrays -----------------------------------------------

struct ArraySet {
    float* ptr[4] = {nullptr, nullptr, nullptr, nullptr};  // w, g, m, pub
    VmmArrays* vmm = nullptr;  // not NULL: chunk-mapped arrays
    int mode = WAGMA_PLACE_PLAIN;
    int examined = 0, regions = 1, g_with_w = 0;
    double slow_gbs = 0.0, fast_gbs = 0.0;
    double step_ms = 0.0;  // measured time of a group step on these arrays (0 = not measured)
};

void release(ArraySet& set)
{
    if (set.vmm) {
        (void)hipDeviceSynchronize();
        free_vmm_arrays(set.vmm);
    } else {
        for (float* p : set.ptr)
            if (p)
                (void)hipFree(p);
    }
    set = ArraySet();
}

// arrays built chunk by chunk (wagma_chunks.h) after one of its patterns
bool place_chunks(int device, size_t bytes, bool debug, wagma_placement::ChunkPattern pattern, ArraySet& out)
{
    using wagma_placement::ChunkPattern;
    const int per_array = (int)((bytes + wagma_placement::kChunkBytes - 1) / wagma_placement::kChunkBytes);
    if (4 * per_array > wagma_placement::kMaxChunks)
        return false;
    VmmMemory* memory = new (std::nothrow) VmmMemory();
    int* index = new (std::nothrow) int[4 * (size_t)per_array];
    VmmArrays* arrays = nullptr;
    if (memory && index && memory->init(device)) {
        memory->reserve = size_t(2) << 30;
        auto* search = new (std::nothrow) wagma_placement::ChunkSearch<VmmMemory>(*memory, per_array, pattern);
        wagma_placement::ChunkPlan plan;
        plan.w = index;
        plan.g = index + per_array;
        plan.m = index + 2 * per_array;
        plan.pub = index + 3 * per_array;
        if (search && search->run(plan)) {
            if (debug) {
                std::fprintf(stderr, "wagma placement (chunks, %s): %d examined, %d classes, %d of %d in pattern, "
                                     "slow %.0f fast %.0f GB/s\n  classes:",
                             pattern == ChunkPattern::one_region  ? "one region"
                             : pattern == ChunkPattern::pub_apart ? "pub apart"
                                                                  : "three regions",
                             plan.examined, plan.classes, plan.in_pattern, 4 * per_array, plan.slow_gbs, plan.fast_gbs);
                for (int i = 0; i < search->chunks(); ++i)
                    std::fprintf(stderr, " %d", search->chunk_class(i));
                std::fprintf(stderr, "\n");
            }
            arrays = memory->build(plan);
            out.examined = plan.examined;
            const int wanted = pattern == ChunkPattern::one_region ? 1 : pattern == ChunkPattern::pub_apart ? 2 : 3;
            out.regions = plan.classes < wanted ? (plan.classes < 1 ? 1 : plan.classes) : wanted;
            out.g_with_w = 1;
            out.slow_gbs = plan.slow_gbs;
            out.fast_gbs = plan.fast_gbs;
        }
        delete search;
    }
    delete memory;  // returns the chunks that were not used, the spacers, the scratch window
    delete[] index;
    if (!arrays)
        return false;
    out.vmm = arrays;
    out.mode = WAGMA_PLACE_CHUNKS;
    for (int a = 0; a < 4; ++a)
        out.ptr[a] = (float*)arrays->va[a];
    return true;
}

// whole arrays in different regions (wagma_placement.h)
bool place_arrays(size_t bytes, bool debug, ArraySet& out)
{
    wagma_placement::Result found;
    {
        HipMemory memory;
        memory.reserve = 2 * bytes;  // keep room for the caller while candidates are held
        auto* search = new (std::nothrow) wagma_placement::RegionSearch<HipMemory>(memory, bytes);
        if (search && memory.init()) {
            found = search->run();
            if (debug)
                report_search(*search);
        }
        delete search;
    }
    char* arrays[4] = {found.w, found.g, found.m, found.pub};
    const bool useful = found.regions >= 2;
    bool ok = useful;
    for (char*& a : arrays)
        if (ok && !a && hipMalloc((void**)&a, bytes) != hipSuccess) {
            a = nullptr;
            ok = false;
        }
    if (!ok) {  // nothing gained over plain allocations, or out of memory
        for (char* a : arrays)
            if (a)
                (void)hipFree(a);
        return false;
    }
    out.mode = WAGMA_PLACE_ARRAYS;
    out.examined = found.candidates;
    out.regions = found.regions;
    out.g_with_w = found.g_with_w;
    out.slow_gbs = found.slow_gbs;
    out.fast_gbs = found.fast_gbs;
    for (int a = 0; a < 4; ++a)
        out.ptr[a] = (float*)arrays[a];
    return true;
}

bool place_plain(size_t bytes, ArraySet& out)
{
    for (int a = 0; a < 4; ++a) {
        if (hipMalloc((void**)&out.ptr[a], bytes) != hipSuccess) {
            out.ptr[a] = nullptr;
            release(out);
            return false;
        }
    }
    out.mode = WAGMA_PLACE_PLAIN;
    return true;
}

// Milliseconds per group step of `ctx` on the (uninitialised) arrays of `set`: every distinct
// group schedule equally often, six steps or a few more, after one untimed pass of as many; with
// `global`, of a global iteration (three, after three untimed ones).  0 on failure.
double time_steps(wagma_ctx* ctx, const ArraySet& set, bool global = false)
{
    hipEvent_t start = nullptr, stop = nullptr;
    if (hipEventCreate(&start) != hipSuccess || hipEventCreate(&stop) != hipSuccess) {
        if (start)
            (void)hipEventDestroy(start);
        return 0.0;
    }
    // every fourth process late, so that the send-buffer reads of late members are part of
    // what is timed
    uint64_t late[kMaskWords];
    for (int k = 0; k < kMaskWords; ++k)
        late[k] = UINT64_C(0x2222222222222222);
    double ms_per_step = 0.0;
    bool ok = true;
    for (int pass = 0; pass < 2 && ok; ++pass) {
        const int steps = global ? 3 : ctx->period * ((6 + ctx->period - 1) / ctx->period);
        ok = hipEventRecord(start, nullptr) == hipSuccess;
        for (int t = 0; t < steps && ok; ++t)
            ok = step_flat(ctx, set.ptr[0], set.ptr[1], set.ptr[2], set.ptr[3], late, nullptr, 0.0f, 0.0f, t, nullptr,
                           global ? wagma_detail::Force::global : wagma_detail::Force::group) == WAGMA_OK;
        ok = ok && hipEventRecord(stop, nullptr) == hipSuccess && hipEventSynchronize(stop) == hipSuccess;
        float ms = 0.0f;
        if (ok && pass == 1 && hipEventElapsedTime(&ms, start, stop) == hipSuccess)
            ms_per_step = ms / steps;
    }
    (void)hipEventDestroy(start);
    (void)hipEventDestroy(stop);
    return ok ? ms_per_step : 0.0;
}

// Which launch-shape setting of the context a group (or global) iteration uses: placed_shape for
// the kernel that holds a group in registers, placed_coop_shape for the one that deals a group's
// rows out to the wavefronts of a workgroup, none (nullptr) for the row-streaming kernel.
int* shape_setting(wagma_ctx* ctx, bool global, int* count)
{
    const int members = global ? ctx->P : ctx->S;
    if (members <= 8) {
        *count = wagma_detail::kNumLaunchShapes;
        return &ctx->placed_shape;
    }
    if (members <= 64) {
        *count = wagma_detail::kNumCoopShapes;
        return &ctx->placed_coop_shape;
    }
    *count = 0;
    return nullptr;
}

// What a placement is judged by: milliseconds per iteration over a period of tau iterations,
// the kernel that holds a group in registers with the better of its first and of its caller-array
// launch shape, the one for larger groups with the best of its three (which wins depends on the
// placement, so a placement is not judged with one of them alone).
// 0 on failure.
double time_placement(wagma_ctx* ctx, const ArraySet& set)
{
    const int kept = ctx->placed_shape, kept_coop = ctx->placed_coop_shape;
    auto better_of_two = [&](bool global) {
        int count = 0;
        int* setting = shape_setting(ctx, global, &count);
        if (!setting)
            return time_steps(ctx, set, global);
        double best = 0.0;
        const bool in_registers = setting == &ctx->placed_shape;
        for (int shape : {0, in_registers ? wagma_detail::kForeignShape : 1, in_registers ? -1 : 2}) {
            if (shape < 0)
                break;
            *setting = shape;
            const double t = time_steps(ctx, set, global);
            if (t > 0.0 && (best == 0.0 || t < best))
                best = t;
        }
        return best;
    };
    const double group_ms = ctx->tau != 1 ? better_of_two(false) : 0.0;
    const double global_ms = ctx->tau >= 1 ? better_of_two(true) : 0.0;
    ctx->placed_shape = kept;
    ctx->placed_coop_shape = kept_coop;
    if (ctx->tau == 0)
        return group_ms;
    if (ctx->tau == 1)
        return global_ms;
    if (group_ms == 0.0 || global_ms == 0.0)
        return 0.0;
    return ((ctx->tau - 1) * group_ms + global_ms) / ctx->tau;
}

// Placement by measurement alone: candidate arrays spread over the free memory, then a
// coordinate descent over which candidate plays which role (w, g, m, pub), judged by the time
// of the step kernel itself.  No assumption about regions is needed; on a GPU with clean
// memory it ends with w, m and pub in three regions and g next to w.
bool place_search(wagma_ctx* ctx, size_t bytes, bool debug, ArraySet& out)
{
    constexpr int kMaxCand = 8;
    const size_t reserve = size_t(4) << 30;
    size_t free_b = 0, total_b = 0;
    if (hipMemGetInfo(&free_b, &total_b) != hipSuccess || free_b < 5 * bytes + reserve)
        return false;  // fewer than five candidates: nothing to choose from
    int n = (int)((free_b - reserve) / bytes);
    if (n > kMaxCand)
        n = kMaxCand;
    size_t gap = (free_b - reserve - (size_t)n * bytes) / n;  // spread the candidates evenly
    if (gap > (size_t(24) << 30))
        gap = size_t(24) << 30;
    float* cand[kMaxCand] = {};
    void* spacer[kMaxCand] = {};
    int got = 0;
    for (; got < n; ++got) {
        if (hipMalloc((void**)&cand[got], bytes) != hipSuccess) {
            cand[got] = nullptr;
            break;
        }
        if (gap >= (size_t(1) << 30) && hipMalloc(&spacer[got], gap) != hipSuccess)
            spacer[got] = nullptr;
    }
    (void)hipGetLastError();
    for (void* sp : spacer)
        if (sp)
            (void)hipFree(sp);
    bool ok = got >= 5;
    int role[4] = {0, 1, 2, 3};  // candidate index of w, g, m, pub
    double best = 0.0;
    int trials = 0;
    if (ok) {
        ArraySet trial;
        auto time_roles = [&](const int r[4]) {
            for (int a = 0; a < 4; ++a)
                trial.ptr[a] = cand[r[a]];
            ++trials;
            return time_steps(ctx, trial);
        };
        best = time_roles(role);
        ok = best > 0.0;
        const int visit[4] = {0, 2, 3, 1};  // w, m, pub, then g
        for (int round = 0; round < 2 && ok; ++round) {
            bool moved = false;
            for (int which : visit) {
                for (int c = 0; c < got && ok; ++c) {
                    if (c == role[0] || c == role[1] || c == role[2] || c == role[3])
                        continue;
                    int r[4] = {role[0], role[1], role[2], role[3]};
                    r[which] = c;
                    const double ms = time_roles(r);
                    if (ms > 0.0 && ms < 0.995 * best) {
                        best = ms;
                        role[which] = c;
                        moved = true;
                    }
                }
            }
            if (!moved)
                break;
        }
    }
    if (debug)
        std::fprintf(stderr, "wagma placement (search): %d candidates, %d timings, roles w=%d g=%d m=%d pub=%d, "
                             "%.3f ms per group step\n", got, trials, role[0], role[1], role[2], role[3], best);
    for (int c = 0; c < got; ++c) {
        const bool used = ok && (c == role[0] || c == role[1] || c == role[2] || c == role[3]);
        if (!used)
            (void)hipFree(cand[c]);
    }
    if (!ok)
        return false;
    out.mode = WAGMA_PLACE_SEARCH;
    out.regions = 0;  // not known: the search does not look at regions
    out.examined = got;
    out.step_ms = best;
    for (int a = 0; a < 4; ++a)
        out.ptr[a] = cand[role[a]];
    return true;
}

}  // namespace

extern "C" {

int wagma_alloc_buffers(wagma_ctx* ctx, float** w, float** g, float** m, float** pub)
{
    if (!ctx || !w || !g || !m || !pub || ctx->placed[0])
        return WAGMA_EINVAL;
    int device = -1;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess)
        return hip_failed(e);
    if (device != ctx->device)
        return WAGMA_EINVAL;
    const size_t bytes = (size_t)ctx->P * (size_t)ctx->ld * sizeof(float);
    const bool debug = std::getenv("WAGMA_DEBUG_PLACEMENT") != nullptr;

    // With WAGMA_PLACE_AUTO: four ordinary allocations first, while the memory is as the caller
    // left it (on a GPU with untouched memory they lie in one HBM region, which the kernel that
    // holds a group in registers likes); then arrays built from chunks: w, g and m from one region
    // and pub, which is written and hardly ever read, from another (measured best for that kernel
    // and good for the one for larger groups: 0.814 -> 0.822 of peak, global iteration 6130 -> 6400
    // GB/s); all from one region (what brings the ordinary allocations' rate back on a GPU whose
    // memory has been in use); from all three regions in turn (which the kernel for larger groups
    // likes best).  Each is judged with the step kernels themselves and must be 0.5 % faster than
    // what is kept to replace it; at most two sets of arrays exist at a time.  WAGMA_PLACE_CHUNKS
    // compares the three chunk patterns in the same manner; another fixed mode takes that mode if
    // it can be had (the timed search and the placement by whole arrays are no longer part of
    // AUTO: the chunk patterns cover what they find).  Ordinary allocations are what remains when
    // nothing else could be had.
    using wagma_placement::ChunkPattern;
    constexpr int kChunksOneRegion = 100, kChunksPubApart = 101;  // candidates, not modes: reported as WAGMA_PLACE_CHUNKS
    const int mode = bytes >= wagma_placement::kPlacementMinBytes ? ctx->opt_placement : WAGMA_PLACE_PLAIN;
    const int auto_order[4] = {WAGMA_PLACE_PLAIN, kChunksPubApart, kChunksOneRegion, WAGMA_PLACE_CHUNKS};
    const int chunks_order[4] = {kChunksPubApart, kChunksOneRegion, WAGMA_PLACE_CHUNKS, WAGMA_PLACE_PLAIN};
    const int fixed_order[4] = {mode, WAGMA_PLACE_PLAIN, -1, -1};
    const bool compare = mode == WAGMA_PLACE_AUTO || mode == WAGMA_PLACE_CHUNKS;
    ArraySet best;
    for (int candidate : (mode == WAGMA_PLACE_AUTO ? auto_order : mode == WAGMA_PLACE_CHUNKS ? chunks_order : fixed_order)) {
        if (candidate < 0 || (best.ptr[0] && (!compare || (mode == WAGMA_PLACE_CHUNKS && candidate == WAGMA_PLACE_PLAIN))))
            break;  // a fixed mode: the first placement that worked; ordinary allocations only if none did
        size_t free_b = 0, total_b = 0;
        if (best.ptr[0] && (hipMemGetInfo(&free_b, &total_b) != hipSuccess || free_b < 4 * bytes + (size_t(4) << 30)))
            break;  // no room for a second set to compare with
        ArraySet trial;
        bool ok = false;
        if (candidate == WAGMA_PLACE_SEARCH)
            ok = place_search(ctx, bytes, debug, trial);
        else if (candidate == WAGMA_PLACE_CHUNKS || candidate == kChunksOneRegion || candidate == kChunksPubApart)
            ok = place_chunks(device, bytes, debug,
                              candidate == kChunksOneRegion  ? ChunkPattern::one_region
                              : candidate == kChunksPubApart ? ChunkPattern::pub_apart
                                                             : ChunkPattern::rotate,
                              trial);
        else if (candidate == WAGMA_PLACE_ARRAYS)
            ok = place_arrays(bytes, debug, trial);
        else
            ok = place_plain(bytes, trial);
        if (!ok) {
            (void)hipGetLastError();
            continue;
        }
        if (compare)
            trial.step_ms = time_placement(ctx, trial);
        if (debug)
            std::fprintf(stderr, "wagma placement: mode %d regions %d: %.3f ms per iteration\n", trial.mode,
                         trial.regions, trial.step_ms);
        // step_ms == 0: the timing failed, the placement's speed is unknown; any placement with
        // a known time replaces such a one, and a later one must be 0.5 % faster to replace a known one
        const bool better = trial.step_ms > 0.0 && (best.step_ms == 0.0 || trial.step_ms < 0.995 * best.step_ms);
        if (!best.ptr[0] || better) {
            release(best);
            best = trial;
        } else {
            release(trial);
        }
    }
    if (!best.ptr[0]) {
        wagma_detail::set_last_hip_error(hipErrorOutOfMemory);
        return WAGMA_ENOMEM;
    }
    if ((e = hipDeviceSynchronize()) != hipSuccess) {
        release(best);
        return hip_failed(e);
    }
    ctx->vmm = best.vmm;
    ctx->place_mode = best.mode;
    ctx->place_candidates = best.examined;
    ctx->place_regions = best.regions;
    ctx->place_g_with_w = best.g_with_w;
    ctx->place_same_gbs = best.slow_gbs;
    ctx->place_split_gbs = best.fast_gbs;
    ctx->placed_ld = ctx->ld;
    ctx->placed[0] = *w = best.ptr[0];
    ctx->placed[1] = *g = best.ptr[1];
    ctx->placed[2] = *m = best.ptr[2];
    ctx->placed[3] = *pub = best.ptr[3];
    // The launch shapes are measured on the chosen arrays as well (step_flat says what is known
    // about them): every shape once, the two fastest once more; the group iterations first, then
    // the global one if it runs another kernel.
    ctx->placed_shape = 0;
    ctx->placed_coop_shape = 0;
    if (bytes >= wagma_placement::kPlacementMinBytes) {
        auto keep_fastest = [&](bool global) {
            int count = 0;
            int* setting = shape_setting(ctx, global, &count);
            if (!setting)
                return;
            double ms[8] = {};
            int first = 0, second = -1;
            for (int c = 0; c < count; ++c) {
                *setting = c;
                ms[c] = time_steps(ctx, best, global);
            }
            for (int c = 1; c < count; ++c) {
                if (ms[c] > 0.0 && (ms[first] == 0.0 || ms[c] < ms[first])) {
                    second = first;
                    first = c;
                } else if (ms[c] > 0.0 && (second < 0 || ms[second] == 0.0 || ms[c] < ms[second])) {
                    second = c;
                }
            }
            for (int c : {first, second}) {
                if (c < 0)
                    continue;
                *setting = c;
                const double again = time_steps(ctx, best, global);
                if (again > 0.0 && (ms[c] == 0.0 || again < ms[c]))
                    ms[c] = again;
            }
            if (second >= 0 && ms[second] > 0.0 && (ms[first] == 0.0 || ms[second] < ms[first]))
                first = second;
            *setting = first;
            if (debug)
                for (int c = 0; c < count; ++c)
                    std::fprintf(stderr, "wagma placement: %s step, launch shape %d: %.3f ms%s\n", global ? "global" : "group", c,
                                 ms[c], c == first ? " (kept)" : "");
        };
        static_assert(wagma_detail::kNumLaunchShapes <= 8 && wagma_detail::kNumCoopShapes <= 8, "ms[] above");
        int count = 0;
        const bool has_group = ctx->tau != 1, has_global = ctx->tau >= 1;
        if (has_group)
            keep_fastest(false);
        if (has_global && !(has_group && shape_setting(ctx, true, &count) == shape_setting(ctx, false, &count)))
            keep_fastest(true);
        (void)hipGetLastError();
    }
    return WAGMA_OK;
}

int wagma_free_buffers(wagma_ctx* ctx)
{
    if (!ctx)
        return WAGMA_EINVAL;
    int rc = WAGMA_OK;
    if (ctx->vmm) {
        const hipError_t e = hipDeviceSynchronize();
        if (e != hipSuccess)
            rc = hip_failed(e);
        free_vmm_arrays(ctx->vmm);
        ctx->vmm = nullptr;
        for (int k = 0; k < 4; ++k)
            ctx->placed[k] = nullptr;
        return rc;
    }
    for (int k = 0; k < 4; ++k) {
        if (ctx->placed[k]) {
            const hipError_t e = hipFree(ctx->placed[k]);
            if (e != hipSuccess)
                rc = hip_failed(e);
            ctx->placed[k] = nullptr;
        }
    }
    return rc;
}

int wagma_placement_info(const wagma_ctx* ctx, int* mode, int* candidates, int* regions, int* g_with_w,
                         double* same_gbs, double* split_gbs)
{
    if (!ctx)
        return WAGMA_EINVAL;
    if (mode)
        *mode = ctx->place_mode;
    if (g_with_w)
        *g_with_w = ctx->place_g_with_w;
    if (candidates)
        *candidates = ctx->place_candidates;
    if (regions)
        *regions = ctx->place_regions;
    if (same_gbs)
        *same_gbs = ctx->place_same_gbs;
    if (split_gbs)
        *split_gbs = ctx->place_split_gbs;
    return WAGMA_OK;
}

}  // extern "C"
