// The tile table of the per-tensor layout of libwagma: which workgroup takes which slices of which
// tensor.  No HIP in here beyond the function qualifiers, so that the construction also runs on
// the CPU (tests/tiles_host.cpp).
#ifndef WAGMA_TILES_H
#define WAGMA_TILES_H

#include <cstddef>
#include <cstdint>
#include <vector>

#include "wagma_shapes.h"

namespace wagma_detail {

constexpr int kTileSlices = 256;                   // 16-byte slices of a contiguous tile: 4 KiB, four wavefronts of 64 lanes
constexpr int64_t kBlockSlices = 64 * kTileSlices; // slices of a mapped block: 256 KiB, what a map permutes

struct TileRef {
    int32_t tensor;         // which tensor a tile of the per-tensor layout belongs to
    uint32_t size;          // floats in that tensor (0: an empty tile that pads the table)
    uint32_t first_slice;   // first 16-byte slice of the tile inside that tensor, or of the block below
    uint32_t tile_in_block; // 0: the tile is 256 consecutive slices.  k + 1: tile k of a block of 64 tiles
                            // (256 KiB, whole slices only) whose slices are dealt out by the plan's map
};

// A tile together with where its tensor lies, for plans whose tensors are spaced alike in every
// array: tensor k of process r begins `stride` floats behind that of process r - 1 (a stack of the
// P replicas of a parameter, or views into P rows).  One 64-byte entry per tile, so that a
// workgroup knows its addresses after a single look-up.
struct AffineTile {
    TileRef ref;
    int64_t stride;  // floats from the tensor of one process to that of the next, in all four arrays
    float* w;        // the tensor of process 0
    const float* g;
    float* m;
    float* pub;
    int64_t unused;
};
static_assert(sizeof(AffineTile) == 64, "one entry is one 64-byte line");

// For plans whose tensors lie anywhere: the four pointers of one tensor of one process.  The plan
// holds them by unit and by place: a unit is a mapped block (64 tiles of one tensor), or a tensor
// (for its tiles outside the blocks); a place is a position in a row of the schedule table.
struct SlotPointers {
    float* w;
    const float* g;
    float* m;
    float* pub;
};
static_assert(sizeof(SlotPointers) == 32, "four pointers");

// The tile table begins with mapped_tiles tiles that belong to blocks of 64: such a tile knows its
// unit from its number alone, the others from the tensor their entry names.
WAGMA_SHAPES_FN int64_t unit_of_tile(int64_t tile, int64_t mapped_tiles, int tensor)
{
    return tile < mapped_tiles ? tile >> 6 : (mapped_tiles >> 6) + tensor;
}

// The 16-byte slice, inside its tensor, that lane `lane` of wavefront (or quarter) `wave` of a tile
// takes.
WAGMA_SHAPES_FN int64_t tensor_slice(uint64_t map, const TileRef& ref, int64_t wave, int64_t lane)
{
    if (ref.tile_in_block == 0)
        return (int64_t)ref.first_slice + wave * 64 + lane;
    return (int64_t)ref.first_slice + mapped_slice(map, ref.tile_in_block - 1, wave, lane);
}

// Where the mapped blocks of a tensor of `size` floats lie: `lead` slices into the tensor (the
// slices before it are contiguous tiles), `blocks` of them.  `phase` is the tensor's address
// modulo 64 KiB if that is the same in every process and array, else -1: the launch shapes pair
// pieces whose addresses differ in bit 15 only, so the blocks begin on a 64 KiB boundary of the
// address space where the tensor crosses one at the same place everywhere, else at its first
// element.
inline void blocks_of(int64_t size, int phase, uint64_t block_map, int64_t& lead, int64_t& blocks)
{
    lead = 0;
    blocks = 0;
    if (block_map == 0)
        return;
    const int64_t whole = size / 4;
    if (phase >= 0)
        lead = (int64_t)((65536 - phase) & 65535) / 16;
    if (whole - lead < kBlockSlices)
        lead = 0;
    blocks = (whole - lead) / kBlockSlices;
}

// The table for T tensors.  Every whole 256 KiB of a tensor is a mapped block of 64 tiles; they
// come first (64 slots each, so that the low three bits of a tile's number in its block are its
// XCD: workgroup b of a launch runs on XCD b mod 8).  What is left of a tensor is cut into
// contiguous 4 KiB tiles; of these each XCD gets runs of 2^run_log2 consecutive ones: that part of
// the table is padded with empty tiles to whole rounds of 8 runs and permuted.  The tiles before a
// tensor's first block end where it begins: to them the tensor is that short.  Returns the number
// of mapped tiles (a multiple of 64); refs.size() is the number of tiles.
inline int64_t build_tile_table(int T, const int64_t* sizes, const int* phase, uint64_t block_map, int run_log2,
                                std::vector<TileRef>& refs)
{
    std::vector<TileRef> in_order;  // the contiguous tiles, tensor by tensor
    refs.clear();
    for (int k = 0; k < T; ++k) {
        const int64_t slices = (sizes[k] + 3) / 4;
        int64_t lead, blocks;
        blocks_of(sizes[k], phase ? phase[k] : -1, block_map, lead, blocks);
        for (int64_t first = 0; first < lead; first += kTileSlices)
            in_order.push_back(TileRef{k, (uint32_t)(lead * 4), (uint32_t)first, 0u});
        for (int64_t b = 0; b < blocks; ++b)
            for (uint32_t j = 0; j < 64; ++j)
                refs.push_back(TileRef{k, (uint32_t)sizes[k], (uint32_t)(lead + b * kBlockSlices), j + 1});
        for (int64_t first = lead + blocks * kBlockSlices; first < slices; first += kTileSlices)
            in_order.push_back(TileRef{k, (uint32_t)sizes[k], (uint32_t)first, 0u});
    }
    const int64_t mapped_tiles = (int64_t)refs.size();
    const int64_t round_tiles = int64_t(8) << run_log2;
    const int64_t plain_tiles = ((int64_t)in_order.size() + round_tiles - 1) / round_tiles * round_tiles;
    // an empty tile has size 0: every lane of it returns at once
    while ((int64_t)in_order.size() < plain_tiles)
        in_order.push_back(TileRef{0, 0u, 0u, 0u});
    // slot i of this part holds tile number `linear` of the walk: the XCD number i mod 8 moves
    // from bits [0,3) of the tile number up to bits [run_log2, run_log2 + 3)
    refs.resize((size_t)(mapped_tiles + plain_tiles));
    for (int64_t i = 0; i < plain_tiles; ++i) {
        const int64_t xcd = i & 7, hi = i >> 3;
        const int64_t linear =
            ((hi >> run_log2) << (run_log2 + 3)) | (xcd << run_log2) | (hi & ((int64_t(1) << run_log2) - 1));
        refs[(size_t)(mapped_tiles + i)] = in_order[(size_t)linear];
    }
    return mapped_tiles;
}

// The step works element by element and knows no tensor boundaries: tensors that follow one
// another without a gap, in every array of every process (views into one buffer per process), are
// one tensor to it.  arrays[a][r * T + k] is tensor k of process r in array a (w, g, m, pub).
// Joined tensor j begins with tensor first_of[j] and has joined_sizes[j] floats.
inline void join_tensors(int P, int T, const int64_t* sizes, const void* const* const arrays[4],
                         std::vector<int>& first_of, std::vector<int64_t>& joined_sizes)
{
    first_of.clear();
    joined_sizes.clear();
    for (int k = 0; k < T; ++k) {
        bool joins = k > 0;
        for (int a = 0; a < 4 && joins; ++a)
            for (int r = 0; r < P && joins; ++r) {
                const size_t i = (size_t)r * T + k;
                joins = (uintptr_t)arrays[a][i] == (uintptr_t)arrays[a][i - 1] + (uintptr_t)sizes[k - 1] * sizeof(float);
            }
        if (joins) {
            joined_sizes.back() += sizes[k];
        } else {
            first_of.push_back(k);
            joined_sizes.push_back(sizes[k]);
        }
    }
}

// Are the tensors spaced alike in every array: tensor k of process r a fixed number of bytes, the
// same in all four arrays, behind that of process r - 1?  (A stack of the P replicas of a
// parameter, or views into P rows.)  step_bytes[k] is that distance (0 with one process).
inline bool spaced_alike(int P, int T, const void* const* const arrays[4], std::vector<int64_t>& step_bytes)
{
    step_bytes.assign((size_t)T, 0);
    for (int k = 0; k < T && P > 1; ++k) {
        const intptr_t step = (intptr_t)arrays[0][(size_t)T + k] - (intptr_t)arrays[0][k];
        for (int a = 0; a < 4; ++a)
            for (int r = 1; r < P; ++r)
                if ((intptr_t)arrays[a][(size_t)r * T + k] - (intptr_t)arrays[a][(size_t)(r - 1) * T + k] != step)
                    return false;
        step_bytes[(size_t)k] = (int64_t)step;
    }
    return true;
}

// The pointers by place: out[(row * units + unit) * P + place] holds the four pointers of the
// unit's tensor for the process that stands at `place` in row `row` of the schedule table
// (`schedule`: rows x P ranks).  Returns the number of units: the mapped blocks, then the T tensors.
inline int64_t build_slot_pointers(int P, int T, int rows, const int32_t* schedule, const std::vector<TileRef>& refs,
                                   int64_t mapped_tiles, const void* const* const arrays[4],
                                   std::vector<SlotPointers>& out)
{
    const int64_t blocks = mapped_tiles >> 6;
    const int64_t units = blocks + T;
    out.resize((size_t)rows * (size_t)units * (size_t)P);
    for (int row = 0; row < rows; ++row)
        for (int64_t unit = 0; unit < units; ++unit) {
            const size_t k = unit < blocks ? (size_t)refs[(size_t)unit * 64].tensor : (size_t)(unit - blocks);
            SlotPointers* to = out.data() + ((size_t)row * (size_t)units + (size_t)unit) * (size_t)P;
            for (int place = 0; place < P; ++place) {
                const size_t i = (size_t)schedule[(size_t)row * P + place] * (size_t)T + k;
                to[place] = SlotPointers{(float*)arrays[0][i], (const float*)arrays[1][i], (float*)arrays[2][i],
                                         (float*)arrays[3][i]};
            }
        }
    return units;
}

}  // namespace wagma_detail

#endif  // WAGMA_TILES_H
