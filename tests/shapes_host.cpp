// CPU check of the launch shapes of libwagma (csrc/wagma_shapes.h, no HIP in it): every shape the
// library uses, and a range of forced stripes, runs and maps, must deal the slices of a padded
// row out to (workgroup, wavefront, lane) exactly once, 16 lanes on 16 consecutive slices.
#include <cstdint>
#include <cstdio>
#include <vector>

#include "wagma_shapes.h"

using namespace wagma_detail;

static int failures = 0;

static void check(const char* what, uint64_t map, int stripe_log2, int xcd_chunk_log2, int64_t tiles_wanted)
{
    const int round_log2 = round_log2_of(map, stripe_log2, xcd_chunk_log2) < 3 ? 3 : round_log2_of(map, stripe_log2, xcd_chunk_log2);
    const int64_t tiles = ((tiles_wanted + (int64_t(1) << round_log2) - 1) >> round_log2) << round_log2;
    std::vector<unsigned char> seen((size_t)tiles * 256, 0);
    bool ok = valid_map(map);
    for (int64_t tile = 0; tile < tiles && ok; ++tile) {
        for (int wave = 0; wave < 4 && ok; ++wave) {
            for (int lane = 0; lane < 64; ++lane) {
                const int64_t slice = map != 0 ? mapped_slice(map, tile, wave, lane)
                                               : striped_slice(stripe_log2, xcd_chunk_log2, tile, wave, lane);
                if (slice < 0 || slice >= tiles * 256 || seen[(size_t)slice]) {
                    ok = false;
                    break;
                }
                seen[(size_t)slice] = 1;
                // 16 lanes take 16 consecutive slices
                if ((lane & 15) != 0) {
                    const int64_t first = map != 0 ? mapped_slice(map, tile, wave, lane & ~15)
                                                   : striped_slice(stripe_log2, xcd_chunk_log2, tile, wave, lane & ~15);
                    if (slice != first + (lane & 15))
                        ok = false;
                }
            }
        }
    }
    if (!ok) {
        std::printf("FAILED: %s (map %010llx stripe %d run %d, %lld tiles)\n", what, (unsigned long long)map, stripe_log2,
                    xcd_chunk_log2, (long long)tiles);
        ++failures;
    }
}

int main()
{
    for (int64_t tiles : {1, 8, 63, 64, 65, 1000, 24959}) {
        for (int k = 0; k < kNumLaunchShapes; ++k)
            check("launch shape", kLaunchShapes[k].map, kLaunchShapes[k].stripe_log2, kLaunchShapes[k].xcd_chunk_log2, tiles);
        for (int k = 0; k < kNumCoopShapes; ++k)
            check("shape for large groups", kCoopShapes[k].map, kCoopShapes[k].stripe_log2, kCoopShapes[k].xcd_chunk_log2, tiles);
        for (int stripe = 0; stripe <= 9; ++stripe)
            for (int run = 0; run <= 9; ++run)
                check("stripe and run", 0, stripe, run, tiles);
        check("identity map", 0x9876543210ull, 0, 0, tiles);
        check("reversed map", 0x0123456789ull, 0, 0, tiles);
    }
    // what must be refused
    const uint64_t bad[] = {0x9876543211ull, 0xa876543210ull, 0x876543210ull, 0x19876543210ull, 0x9876543200ull};
    for (uint64_t map : bad) {
        if (valid_map(map)) {
            std::printf("FAILED: map %llx accepted\n", (unsigned long long)map);
            ++failures;
        }
    }
    if (!valid_map(0))
        ++failures;
    std::printf("%s\n", failures ? "failures" : "ok");
    return failures ? 1 : 0;
}
