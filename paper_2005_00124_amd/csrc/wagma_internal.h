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
    int opt_nontemporal, opt_force_stream, opt_stripe_log2;
    int stripe_forced;       // 1: opt_stripe_log2 was set through wagma_debug_set_option
    int opt_xcd_chunk_log2;  // -1: chosen per launch (see step_flat); >= 0: this value for every launch
    uint64_t opt_map;        // not 0: this tile-to-address map for every launch (see slice_of)
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
extern "C" int wagma_debug_set_option(wagma_ctx* ctx, int option, int64_t value);
extern "C" int wagma_debug_get_option(const wagma_ctx* ctx, int option, int64_t* value);

namespace wagma_detail {

// How the column tiles of a row are dealt out to workgroups (hence XCDs) and wavefronts: either
// a map (slice_of in wagma_kernels.h) or, with map == 0, stripe and XCD run length.
struct LaunchShape {
    uint64_t map;
    int stripe_log2, xcd_chunk_log2;
    bool row_streaming = false;  // kCoopShapes only: run the row-streaming kernel instead
};
// The shapes wagma_alloc_buffers times on its arrays.  Bits of the slice number from bit 4 up
// (l = bits 4, 5 of the lane, w = wavefront, x = XCD, t = later tile bits):
//   0  l4 l5 t3 t4 w0 w1 x0 x1 x2 t5   a wavefront takes 1 KiB, the wavefronts of a workgroup 4 KiB
//                                      apart, runs of 4 tiles per XCD
//   1  l4 l5 x0 x1 w0 w1 x2 t3 t4 t5   as 0, tile by tile round the XCDs
//   2  l4 l5 t3 t4 w0 w1 x0 t5 x2 x1   as 0 with the upper XCD bits further up
//   3  l5 t3 x0 x1 t5 w0 x2 l4 w1 t4   a wavefront takes 512 B and the 512 B that lie 32 KiB further on,
//                                      the wavefronts of a workgroup 8 KiB and 64 KiB apart
//   4  l5 x0 x1 t3 w0 t5 x2 l4 w1 t4   as 3, other places for the XCD bits
//   5  l4 x0 t3 t4 w0 t5 x1 l5 w1 x2   as 3, the other lane bit chooses the piece; other places for the rest
constexpr int kNumLaunchShapes = 6;
constexpr LaunchShape kLaunchShapes[kNumLaunchShapes] = {
    {0u, 2, 2}, {0u, 2, 0}, {0x7328965410ull, 0, 0}, {0x4916328507ull, 0, 0}, {0x5936218407ull, 0, 0},
    {0x5329618470ull, 0, 0}};
constexpr int kForeignShape = 3;  // for arrays the library did not place
// Groups of 16 to 64 rows (and the global iteration of 16 to 64 processes):
//   0  l4 l5 t3 t4 w0 w1 t5 x0 x1 x2   1 KiB per wavefront, 4 KiB stripe, runs of 8 tiles per XCD
//   1  l4 x0 x1 t4 w0 t5 t3 l5 w1 x2   a wavefront takes 512 B and the 512 B that lie 32 KiB further on
//   2  the row-streaming kernel with shape 3 of the list above
constexpr int kNumCoopShapes = 3;
constexpr LaunchShape kCoopShapes[kNumCoopShapes] = {
    {0u, 2, 3}, {0x5369218470ull, 0, 0}, {0x4916328507ull, 0, 0, true}};


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
