// CPU check of the tile table of libwagma's per-tensor layout (csrc/wagma_tiles.h, no HIP in it):
// for lists of tensor sizes, address phases, maps and XCD run lengths, the lanes of the table's
// tiles, taken the way the kernels take them (a lane owns the four floats of its slice, cut off at
// the size its tile names), must touch every element of every tensor exactly once and nothing else.
// Also: which tensors a plan joins, and when it counts the replicas of the tensors as spaced alike.
#include <cstdint>
#include <cstdio>
#include <vector>

#include "wagma_tiles.h"

using namespace wagma_detail;

static int failures = 0;

static void check(const char* what, const std::vector<int64_t>& sizes, const std::vector<int>& phase, uint64_t map,
                  int run_log2)
{
    const int T = (int)sizes.size();
    std::vector<TileRef> refs;
    const int64_t mapped = build_tile_table(T, sizes.data(), phase.empty() ? nullptr : phase.data(), map, run_log2, refs);
    const int64_t tiles = (int64_t)refs.size();
    bool ok = mapped % 64 == 0 && (tiles - mapped) % (int64_t(8) << run_log2) == 0 && (map != 0 || mapped == 0);
    std::vector<std::vector<unsigned char>> seen((size_t)T);
    for (int k = 0; k < T; ++k)
        seen[(size_t)k].assign((size_t)sizes[k], 0);
    int64_t empty = 0;
    for (int64_t t = 0; t < tiles && ok; ++t) {
        const TileRef& ref = refs[(size_t)t];
        if (ref.tensor < 0 || ref.tensor >= T || (int64_t)ref.size > sizes[(size_t)ref.tensor]) {
            ok = false;
            break;
        }
        if (ref.size == 0)
            ++empty;
        if (t < mapped) {
            // tile j of a block sits in a slot that is j modulo 64, and a block begins on a 64 KiB
            // boundary of the address space when the tensor's phase is known ...
            ok = ok && ref.tile_in_block == (uint32_t)(t % 64) + 1 && (int64_t)ref.size == sizes[(size_t)ref.tensor] &&
                 ((int64_t)ref.first_slice + kBlockSlices) * 4 <= (int64_t)ref.size;
            if (!phase.empty() && phase[(size_t)ref.tensor] >= 0) {
                // ... unless the tensor has no room for a block behind its first boundary: then its
                // blocks begin at its first element
                const int64_t lead = (int64_t)((65536 - phase[(size_t)ref.tensor]) & 65535) / 16;
                if (sizes[(size_t)ref.tensor] / 4 - lead >= kBlockSlices)
                    ok = ok && ((int64_t)phase[(size_t)ref.tensor] + (int64_t)ref.first_slice * 16) % 65536 == 0;
                else
                    ok = ok && (int64_t)ref.first_slice % kBlockSlices == 0;
            }
        } else {
            ok = ok && ref.tile_in_block == 0;
        }
        for (int wave = 0; wave < 4 && ok; ++wave) {
            for (int lane = 0; lane < 64; ++lane) {
                const int64_t first = tensor_slice(map, ref, wave, lane) * 4;
                if (first >= (int64_t)ref.size)
                    continue;
                for (int64_t e = first; e < first + 4 && e < (int64_t)ref.size; ++e) {
                    if (seen[(size_t)ref.tensor][(size_t)e]++) {
                        ok = false;
                        break;
                    }
                }
            }
        }
    }
    for (int k = 0; k < T && ok; ++k)
        for (int64_t e = 0; e < sizes[(size_t)k]; ++e)
            if (seen[(size_t)k][(size_t)e] != 1) {
                ok = false;
                break;
            }
    // padding never exceeds one round of the XCD walk
    ok = ok && empty < (int64_t(8) << run_log2);
    if (!ok) {
        std::printf("FAILED: %s (map %010llx run_log2 %d, %d tensors, first size %lld)\n", what, (unsigned long long)map,
                    run_log2, T, (long long)sizes[0]);
        ++failures;
    }
}

// Pointer sets made of plain numbers: array a of process r begins at base[a] + r * row_bytes, and
// tensor k lies offset[k] bytes into it.
struct Pointers {
    std::vector<const void*> at[4];
    const void* const* arrays[4];
    Pointers(int P, const std::vector<int64_t>& offset, int64_t row_bytes)
    {
        const int T = (int)offset.size();
        for (int a = 0; a < 4; ++a) {
            at[a].resize((size_t)P * T);
            for (int r = 0; r < P; ++r)
                for (int k = 0; k < T; ++k)
                    at[a][(size_t)r * T + k] = (const void*)(uintptr_t)(0x100000000ull * (a + 1) + r * row_bytes + offset[(size_t)k]);
            arrays[a] = at[a].data();
        }
    }
};

static void expect(bool ok, const char* what)
{
    if (!ok) {
        std::printf("FAILED: %s\n", what);
        ++failures;
    }
}

static void check_joining()
{
    const int P = 3;
    const std::vector<int64_t> sizes = {100, 64, 7, 8, 12, 4};
    // 100 and 64 back to back; 7 follows 64 at once but leaves a gap (its 28 bytes are padded to 32);
    // 8 and 12 back to back; 4 after a gap of one slice
    const std::vector<int64_t> offset = {0, 400, 656, 688, 720, 784};
    std::vector<int> first_of;
    std::vector<int64_t> joined;
    {
        Pointers p(P, offset, 4096);
        join_tensors(P, (int)sizes.size(), sizes.data(), p.arrays, first_of, joined);
        expect(first_of == std::vector<int>({0, 3, 5}) && joined == std::vector<int64_t>({171, 20, 4}), "joining back-to-back tensors");
        std::vector<int64_t> step;
        expect(spaced_alike(P, (int)sizes.size(), p.arrays, step) && step == std::vector<int64_t>(6, 4096), "rows spaced alike");
        // one process of one array holds tensor 1 elsewhere: nothing joins it, and the spacing is gone
        p.at[2][(size_t)1 * sizes.size() + 1] = (const void*)((uintptr_t)p.at[2][(size_t)1 * sizes.size() + 1] + 16);
        join_tensors(P, (int)sizes.size(), sizes.data(), p.arrays, first_of, joined);
        expect(first_of == std::vector<int>({0, 1, 2, 3, 5}) && joined == std::vector<int64_t>({100, 64, 7, 20, 4}),
               "a gap in one process of one array");
        expect(!spaced_alike(P, (int)sizes.size(), p.arrays, step), "spacing broken in one array");
    }
    {
        // the same distance within every array, but another one in g: not alike
        Pointers p(P, offset, 4096);
        for (int r = 0; r < P; ++r)
            for (size_t k = 0; k < sizes.size(); ++k)
                p.at[1][(size_t)r * sizes.size() + k] = (const void*)(uintptr_t)(0x900000000ull + r * 8192 + offset[k]);
        std::vector<int64_t> step;
        expect(!spaced_alike(P, (int)sizes.size(), p.arrays, step), "another distance in one array");
        join_tensors(P, (int)sizes.size(), sizes.data(), p.arrays, first_of, joined);
        expect(first_of == std::vector<int>({0, 3, 5}), "joining does not need equal distances");
    }
    {
        // one process: always spaced alike, distance 0; a negative distance is a distance too
        Pointers one(1, offset, 4096);
        std::vector<int64_t> step;
        expect(spaced_alike(1, (int)sizes.size(), one.arrays, step) && step == std::vector<int64_t>(6, 0), "one process");
        Pointers back(P, offset, -8192);
        expect(spaced_alike(P, (int)sizes.size(), back.arrays, step) && step == std::vector<int64_t>(6, -8192), "rows in descending order");
    }
    {
        // stacked parameters: every tensor its own distance
        const int T = 3;
        Pointers p(2, {0, 0, 0}, 0);
        const int64_t bases[T] = {0x1000, 0x20000, 0x300000}, dist[T] = {400, 4096, 65536};
        for (int a = 0; a < 4; ++a)
            for (int r = 0; r < 2; ++r)
                for (int k = 0; k < T; ++k)
                    p.at[a][(size_t)r * T + k] = (const void*)(uintptr_t)(0x100000000ull * (a + 1) + bases[k] + r * dist[k]);
        std::vector<int64_t> step;
        expect(spaced_alike(2, T, p.arrays, step) && step == std::vector<int64_t>({400, 4096, 65536}), "stacked parameters");
    }
}

// The pointers by place must name, for every row of a schedule, every tile and every place, the
// tensor of the tile's entry in the process that stands at that place.
static void check_by_place()
{
    const int P = 8, rows = 3;
    const std::vector<int64_t> sizes = {65536 + 40, 3, 2 * 65536, 5000, 70001};
    const int T = (int)sizes.size();
    std::vector<int64_t> offset(sizes.size());
    for (size_t k = 0; k < sizes.size(); ++k)
        offset[k] = 0x1000000 * (int64_t)k;
    Pointers p(P, offset, 0x100000);
    // three rows of a schedule: the identity, its reverse, and a shuffle
    std::vector<int32_t> schedule;
    for (int r = 0; r < P; ++r) schedule.push_back(r);
    for (int r = 0; r < P; ++r) schedule.push_back(P - 1 - r);
    for (int r = 0; r < P; ++r) schedule.push_back((r * 3 + 5) % P);
    for (uint64_t map : {uint64_t(0), kLaunchShapes[kForeignShape].map}) {
        std::vector<TileRef> refs;
        const int64_t mapped = build_tile_table(T, sizes.data(), nullptr, map, 3, refs);
        std::vector<SlotPointers> by_place;
        const int64_t units = build_slot_pointers(P, T, rows, schedule.data(), refs, mapped, p.arrays, by_place);
        bool ok = units == mapped / 64 + T && (int64_t)by_place.size() == rows * units * P;
        for (int row = 0; row < rows && ok; ++row)
            for (int64_t tile = 0; tile < (int64_t)refs.size() && ok; ++tile) {
                const int64_t unit = unit_of_tile(tile, mapped, refs[(size_t)tile].tensor);
                ok = unit >= 0 && unit < units;
                for (int place = 0; place < P && ok; ++place) {
                    const SlotPointers& have = by_place[(size_t)((row * units + unit) * P + place)];
                    const size_t i = (size_t)schedule[(size_t)row * P + place] * T + (size_t)refs[(size_t)tile].tensor;
                    ok = have.w == p.arrays[0][i] && have.g == p.arrays[1][i] && have.m == p.arrays[2][i] &&
                         have.pub == p.arrays[3][i];
                }
            }
        expect(ok, map ? "pointers by place, with mapped blocks" : "pointers by place, contiguous tiles only");
    }
}

int main()
{
    check_joining();
    check_by_place();
    const uint64_t maps[] = {0, kLaunchShapes[kForeignShape].map, 0x9876543210ull, 0x0123456789ull, 0x5329618470ull};
    const std::vector<std::vector<int64_t>> lists = {
        {1},
        {3, 1, 2},
        {1023, 1024, 1025, 4096, 5},
        {65536},                     // exactly one block
        {65535, 65537, 65536 + 283}, // just below, just above
        {262144 + 7, 64, 3 * 65536, 2 * 65536 - 1},
        {9408, 64, 64, 4096, 36864, 16384, 147456, 589824, 2359296, 2048000, 1000},  // a convolutional net's mix
    };
    uint64_t seed = 12345;
    for (const auto& sizes : lists) {
        for (uint64_t map : maps) {
            for (int run_log2 : {0, 1, 3, 5, 8}) {
                check("no phases", sizes, {}, map, run_log2);
                std::vector<int> phase(sizes.size());
                // slice-aligned phases, some unknown (-1), some zero
                for (size_t k = 0; k < sizes.size(); ++k) {
                    seed = seed * 6364136223846793005ull + 1442695040888963407ull;
                    const int pick = (int)(seed >> 60);
                    phase[k] = pick == 0 ? -1 : pick == 1 ? 0 : (int)((seed >> 33) % 4096) * 16;
                }
                check("random phases", sizes, phase, map, run_log2);
                std::fill(phase.begin(), phase.end(), 65536 - 16);
                check("one slice before a boundary", sizes, phase, map, run_log2);
                std::fill(phase.begin(), phase.end(), 16);
                check("one slice after a boundary", sizes, phase, map, run_log2);
            }
        }
    }
    std::printf("%s\n", failures ? "failures" : "ok");
    return failures ? 1 : 0;
}
