// What the two translation units of libwagma share: the context and a few helpers.
// wagma.hip holds the step (kernels, launches, schedule, masks, per-tensor plans);
// wagma_alloc.hip holds the optional allocator (wagma_alloc_buffers and what it needs).
#ifndef WAGMA_INTERNAL_H
#define WAGMA_INTERNAL_H

#include <hip/hip_runtime.h>

#include <cstdint>

#include "wagma.h"
#include "wagma_shapes.h"

struct VmmArrays;  // arrays built from 1 GiB physical chunks (wagma_alloc.hip)

struct wagma_ctx {
    int P, S, G, g, tau, period, device;
    int fixed_groups;  // 1: every group iteration uses the groups of iteration 0
    int64_t n, ld;
    int32_t* d_table;  // (period + 1) * P, device
    int32_t* h_table;  // host mirror
    int opt_nontemporal, opt_force_stream, opt_stripe_log2;
    int stripe_forced;       // 1: opt_stripe_log2 was set through wagma_debug_set_option
    int opt_xcd_chunk_log2;  // -1: chosen per launch (see step_flat); >= 0: this value for every launch
    uint64_t opt_map;        // not 0: this tile-to-address map for every launch (see slice_of)
    int opt_tensor_tables;   // 1: per-tensor plans take the tensor list as it is and find every tensor through
                             // the pointers by place, also where the tensors are spaced alike in every array
    float* placed[4];        // w, g, m, pub handed out by wagma_alloc_buffers (or all NULL)
    int placed_shape;        // index into wagma_detail::kLaunchShapes: what wagma_alloc_buffers measured as
                             // best for steps on those arrays with the kernel that holds a group in registers
    int placed_coop_shape;   // likewise, index into kCoopShapes, for the kernel that deals a group's rows out
                             // to the wavefronts of a workgroup (measured on the global iteration)
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

// Launch-shape switches that are not part of the public header: exported for the tests and for
// measurements only.  wagma_debug_set_option also accepts the public WAGMA_OPT_* values.
#define WAGMA_DEBUG_FORCE_STREAM 3   /* 0/1: the row-streaming kernel for every S >= 8 */
#define WAGMA_DEBUG_STRIPE_LOG2 7    /* 0..16: the wavefronts of a workgroup work 2^v KiB apart in every row */
#define WAGMA_DEBUG_XCD_CHUNK_LOG2 8 /* 0..13: each XCD works on runs of 2^v consecutive column tiles of a row;
                                        -1 (the default): chosen per launch, by kernel and by whose arrays they
                                        are.  A per-tensor plan takes the value at wagma_tensors_create (-1
                                        counts as 2) and uses runs twice as long: 2^(v+1), at most 256, tiles */
#define WAGMA_DEBUG_PLACED_SHAPE 10  /* 0..kNumLaunchShapes-1: which of the launch shapes below the kernel that
                                        holds a group in registers uses on the arrays of wagma_alloc_buffers,
                                        which measures them all; read it back after that call */
#define WAGMA_DEBUG_PLACED_COOP_SHAPE 12 /* 0..kNumCoopShapes-1: likewise for the kernel for groups of 16 to 64 rows */
#define WAGMA_DEBUG_MAP 11           /* ten 4-bit fields, a permutation of 0..9: bit k of ((tile << 2 | wavefront) << 2
                                        | lane >> 4) becomes bit 4 + field[k] of the number of the 16-byte slice
                                        of a row; 0 (the default): no forced map */
#define WAGMA_DEBUG_TENSOR_TABLES 13 /* 0/1: a per-tensor plan made after this takes the tensor list as it is given
                                        (tensors that follow one another without a gap are not joined) and finds
                                        its tensors through the pointers laid out by place even if they are
                                        spaced alike */
extern "C" int wagma_debug_set_option(wagma_ctx* ctx, int option, int64_t value);
extern "C" int wagma_debug_get_option(const wagma_ctx* ctx, int option, int64_t* value);

namespace wagma_detail {

// Records a failed HIP call for wagma_last_hip_error (per thread) and returns WAGMA_EHIP.
int hip_failed(hipError_t e);
void set_last_hip_error(hipError_t e);

// wagma_step_lag; `force` makes the iteration a group or a global iteration whatever tau says
// (the allocator times both with it, on arrays that count as the library's own).
enum class Force { none, group, global };
// says (the allocator times group steps with it).
int step_flat(wagma_ctx* ctx, float* w, const float* g, float* m, float* pub, const uint64_t* stale_mask,
              const uint64_t* busy_mask, float lr, float mu, int64_t iter, void* stream, Force force);

}  // namespace wagma_detail

#endif  // WAGMA_INTERNAL_H
