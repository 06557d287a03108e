// Launch shapes of libwagma: which 16-byte column slice of a row each lane of each wavefront of
// each workgroup takes.  No HIP in here beyond the function qualifiers, so that the arithmetic also
// runs on the CPU (tests/shapes_host.cpp).
#ifndef WAGMA_SHAPES_H
#define WAGMA_SHAPES_H

#include <cstdint>

#if defined(__HIPCC__)
#define WAGMA_SHAPES_FN __host__ __device__ __forceinline__
#else
#define WAGMA_SHAPES_FN inline
#endif

namespace wagma_detail {

// Workgroup b of a launch runs on XCD b mod 8, so bits [0,3) of a workgroup's column tile number
// are its XCD.  A workgroup is four wavefronts of 64 lanes and takes 256 slices (4 KiB) of a row.

// With a map: ten 4-bit fields, a permutation of 0..9.  With y = (tile << 2 | wave) << 2 | lane >> 4,
// bit k of y becomes bit 4 + field[k] of the slice number and the higher bits of y stay; 16
// lanes always take 16 consecutive slices (256 B).  A field of the two lane bits that is not 0
// or 1 splits a wavefront's 1 KiB into pieces that lie apart.
WAGMA_SHAPES_FN int64_t mapped_slice(uint64_t map, int64_t tile, int64_t wave, int64_t lane)
{
    const int64_t y = (((tile << 2) | wave) << 2) | (lane >> 4);
    int64_t upper = y & ~int64_t(0x3ff);
#if defined(__HIPCC__)
#pragma unroll
#endif
    for (int k = 0; k < 10; ++k)
        upper |= ((y >> k) & 1) << ((map >> (4 * k)) & 15u);
    return (upper << 4) | (lane & 15);
}

// Without a map: a wavefront takes 64 consecutive slices (1 KiB); each XCD takes runs of
// 2^xcd_chunk_log2 consecutive tiles (the XCD number moves from tile bits [0,3) up to bits
// [j, j+3)), and the four wavefronts of a workgroup work 2^stripe_log2 KiB apart inside
// 4 << stripe_log2 KiB.
WAGMA_SHAPES_FN int64_t striped_slice(int stripe_log2, int xcd_chunk_log2, int64_t tile, int64_t wave, int64_t lane)
{
    if (xcd_chunk_log2 > 0) {
        const int j = xcd_chunk_log2;
        const int64_t xcd = tile & 7;
        const int64_t hi = tile >> 3;
        tile = ((hi >> j) << (j + 3)) | (xcd << j) | (hi & ((int64_t(1) << j) - 1));
    }
    const int64_t super = tile >> stripe_log2;
    const int64_t within = tile & ((int64_t(1) << stripe_log2) - 1);
    return ((((super * 4 + wave) << stripe_log2) + within) << 6) | lane;
}

// 0, or ten fields that are a permutation of 0..9
inline bool valid_map(uint64_t map)
{
    if (map == 0)
        return true;
    if (map >> 40)
        return false;
    unsigned seen = 0;
    for (int k = 0; k < 10; ++k) {
        const unsigned field = (unsigned)(map >> (4 * k)) & 15u;
        if (field > 9u)
            return false;
        seen |= 1u << field;
    }
    return seen == 0x3ffu;
}

// The number of column tiles of a row is rounded up to a multiple of 2^this, so that a shape
// deals the slices of whole rounds among themselves (the surplus lanes find their slice beyond
// the row's end).
inline int round_log2_of(uint64_t map, int stripe_log2, int xcd_chunk_log2)
{
    if (map != 0)
        return 6;  // a map permutes the slices of 64 tiles among themselves
    int round_log2 = stripe_log2;
    if (xcd_chunk_log2 > 0 && xcd_chunk_log2 + 3 > round_log2)
        round_log2 = xcd_chunk_log2 + 3;
    return round_log2;
}

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

}  // namespace wagma_detail

#endif  // WAGMA_SHAPES_H
