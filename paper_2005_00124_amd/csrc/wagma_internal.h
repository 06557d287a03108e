// What the two translation units of libwagma share: the context and a few helpers.
// wagma.hip holds the step (kernels, launches, schedule, masks, per-tensor plans);
// wagma_alloc.hip holds the optional allocator (wagma_alloc_buffers and what it needs).
#ifndef WAGMA_INTERNAL_H
#define WAGMA_INTERNAL_H

#include <hip/hip_runtime.h>

#include <cstdint>

#include "wagma.h"

struct VmmArrays;  // arrays built from 1 GiB physical chunks (wagma_alloc.hip)

struct wagma_ctx {
    int P, S, G, g, tau, period, device;
    int fixed_groups;  // 1: every group iteration uses the groups of iteration 0
    int64_t n, ld;
    int32_t* d_table;  // (period + 1) * P, device
    int32_t* h_table;  // host mirror
    int opt_block, opt_nontemporal, opt_force_stream, opt_swizzle, opt_tile_major, opt_waves, opt_stripe_log2, opt_xcd_chunk_log2;
    float* placed[4];        // w, g, m, pub handed out by wagma_alloc_buffers (or all NULL)
    int64_t placed_ld;       // the row stride those arrays were sized for
    VmmArrays* vmm;          // not NULL: the four arrays are chunk-mapped, not hipMalloc'ed
    int opt_placement;       // WAGMA_PLACE_*
    int place_mode;          // the WAGMA_PLACE_* that the last wagma_alloc_buffers ended with
    int place_candidates;    // allocations tried by the last wagma_alloc_buffers
    int place_regions;       // how many of w, m, pub lie in pairwise different regions (1..3)
    int place_g_with_w;      // 1 if g was found a place in the region of w
    double place_same_gbs;   // probe rate inside one region
    double place_split_gbs;  // probe rate between the regions of w and m (0 if not separated)
};

namespace wagma_detail {

// Records a failed HIP call for wagma_last_hip_error (per thread) and returns WAGMA_EHIP.
int hip_failed(hipError_t e);
void set_last_hip_error(hipError_t e);

// wagma_step_lag; with group_only the iteration is treated as a group iteration whatever tau
// says (the allocator times group steps with it).
int step_flat(wagma_ctx* ctx, float* w, const float* g, float* m, float* pub, const uint64_t* stale_mask,
              const uint64_t* busy_mask, float lr, float mu, int64_t iter, void* stream, bool group_only);

}  // namespace wagma_detail

#endif  // WAGMA_INTERNAL_H
