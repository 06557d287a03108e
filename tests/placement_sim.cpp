// CPU simulation of the HBM-region search (csrc/wagma_placement.h): a fake memory with
// regions, sequential or scattered physical placement, noisy probe rates with slow outliers.
// Prints one line per scenario and exits non-zero if an invariant of the search is violated.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <set>
#include <utility>
#include <vector>

#include "wagma_placement.h"

namespace {

constexpr double kGiB = 1024.0 * 1024.0 * 1024.0;
constexpr uintptr_t kBase = uintptr_t(1) << 44;  // fake addresses, never dereferenced

struct SimMemory {
    std::vector<double> boundaries_gib;  // region k = [boundaries[k], boundaries[k+1])
    double capacity_gib = 288.0;
    // fragmented memory: the middle third of every allocation whose index is in this set lies
    // `detour_gib` further on (in another region), although both of its ends do not
    std::set<size_t> pieced;
    double detour_gib = 0.0;
    std::vector<std::pair<double, double>> detours;  // [start, end) in GiB of detoured ranges
    double next_gib = 0.0;               // bump pointer (sequential placement)
    std::vector<double> scattered_gib;   // if not empty: start of the i-th allocation
    size_t allocations = 0;
    double slow = 5900.0, fast = 7000.0, noise = 0.03, outlier_every = 0.0;
    uint64_t rng = 88172645463325252ull;
    std::set<char*> live;
    long probes = 0;
    bool double_free = false;

    double uniform()
    {
        rng ^= rng << 13;
        rng ^= rng >> 7;
        rng ^= rng << 17;
        return (double)(rng >> 11) / 9007199254740992.0;
    }
    int region_of(double gib) const
    {
        for (const auto& d : detours)
            if (gib >= d.first && gib < d.second)
                gib += detour_gib;
        for (size_t k = 0; k + 1 < boundaries_gib.size(); ++k)
            if (gib >= boundaries_gib[k] && gib < boundaries_gib[k + 1])
                return (int)k;
        return (int)boundaries_gib.size();
    }
    char* allocate(size_t bytes)
    {
        const double size = bytes / kGiB;
        double at;
        if (!scattered_gib.empty()) {
            if (allocations >= scattered_gib.size())
                return nullptr;
            at = scattered_gib[allocations];
        } else {
            at = next_gib;
            if (at + size > capacity_gib)
                return nullptr;
            next_gib += size;
        }
        if (pieced.count(allocations))
            detours.push_back({at + size / 3, at + 2 * size / 3});
        ++allocations;
        char* p = (char*)(kBase + (uintptr_t)(at * kGiB));
        live.insert(p);
        return p;
    }
    void release(char* p)
    {
        if (!live.erase(p))
            double_free = true;
    }
    // fraction of the bytes of [p, p+side) that lie in each region
    std::vector<double> shares(char* p, size_t side) const
    {
        std::vector<double> out(boundaries_gib.size() + 1, 0.0);
        const double lo = ((uintptr_t)p - kBase) / kGiB, len = side / kGiB;
        const int steps = 64;
        for (int i = 0; i < steps; ++i)
            out[region_of(lo + len * (i + 0.5) / steps)] += 1.0 / steps;
        return out;
    }
    double rate(char* a, char* b, size_t side)
    {
        ++probes;
        const std::vector<double> sa = shares(a, side), sb = shares(b, side);
        // writes are fast to the extent that they are spread over more than one region
        double largest = 0.0;
        for (size_t k = 0; k < sa.size(); ++k)
            if (0.5 * (sa[k] + sb[k]) > largest)
                largest = 0.5 * (sa[k] + sb[k]);
        const double spread = 2.0 * (1.0 - largest);  // 0: one region, 1: half and half
        double r = slow + (fast - slow) * (spread > 1.0 ? 1.0 : spread);
        r *= 1.0 + noise * (2.0 * uniform() - 1.0);
        if (outlier_every > 0.0 && uniform() < 1.0 / outlier_every)
            r *= 0.87;
        return r;
    }
};

int failures = 0;

void check(bool ok, const char* scenario, const char* what)
{
    if (!ok) {
        std::printf("FAIL %s: %s\n", scenario, what);
        ++failures;
    }
}

wagma_placement::Result run(const char* name, SimMemory& mem, double array_gib, int want_regions,
                            bool want_g_with_w)
{
    const size_t bytes = (size_t)(array_gib * kGiB);
    wagma_placement::RegionSearch<SimMemory> search(mem, bytes);
    const wagma_placement::Result r = search.run();
    // the region that holds most of an array, and whether it holds at least 90% of it
    auto region = [&](char* p) {
        if (!p)
            return -1;
        const std::vector<double> sh = mem.shares(p, bytes);
        int best = 0;
        for (size_t k = 1; k < sh.size(); ++k)
            if (sh[k] > sh[best])
                best = (int)k;
        return best;
    };
    auto whole = [&](char* p) { return p && mem.shares(p, bytes)[region(p)] >= 0.9; };
    std::printf("%-34s candidates %2d regions %d g_with_w %d  w:%d m:%d pub:%d g:%d  probes %ld  slow %.0f fast %.0f\n",
                name, r.candidates, r.regions, (int)r.g_with_w, region(r.w), region(r.m), region(r.pub),
                region(r.g), mem.probes, r.slow_gbs, r.fast_gbs);
    check(r.regions == want_regions, name, "number of regions found");
    check(!mem.double_free, name, "a candidate was released twice");
    // every live allocation is one of the returned arrays
    std::set<char*> kept;
    for (char* p : {r.w, r.m, r.pub, r.g})
        if (p)
            kept.insert(p);
    check(kept == mem.live, name, "candidates leaked or returned arrays released");
    if (want_regions >= 2) {
        check(region(r.w) != region(r.m), name, "w and m share a region");
        check(whole(r.w) && whole(r.m), name, "a chosen array straddles");
    }
    if (want_regions == 3) {
        check(region(r.pub) != region(r.w) && region(r.pub) != region(r.m), name, "pub shares a region");
        check(whole(r.pub), name, "pub straddles");
    }
    if (want_regions == 3 && r.g)
        check(region(r.g) != region(r.pub), name, "g lies in the region of pub");
    if (want_g_with_w) {
        check(r.g_with_w && region(r.g) == region(r.w) && whole(r.g), name,
              "g is not in the region of w");
    }
    return r;
}

}  // namespace

int main()
{
    const std::vector<double> three = {0.0, 96.0, 192.0, 288.0};
    {
        SimMemory mem;
        mem.boundaries_gib = three;
        run("fresh memory", mem, 6.09, 3, true);
    }
    {
        SimMemory mem;
        mem.boundaries_gib = {0.0, 3.0, 99.0, 195.0, 288.0};  // the first candidate straddles
        run("first candidate straddles", mem, 6.09, 3, true);
    }
    for (int seed = 1; seed <= 12; ++seed) {
        SimMemory mem;
        mem.boundaries_gib = three;
        mem.noise = 0.04;
        mem.outlier_every = 12.0;
        mem.rng ^= (uint64_t)seed * 0x9E3779B97F4A7C15ull;
        mem.next_gib = 7.3 * seed;
        char name[64];
        std::snprintf(name, sizeof name, "noise and slow outliers, seed %d", seed);
        // where the first region holds one whole candidate only, g goes next to m instead
        const bool room_for_g = 96.0 - mem.next_gib >= 2 * 6.09;
        run(name, mem, 6.09, 3, room_for_g);
    }
    {
        SimMemory mem;
        mem.boundaries_gib = {0.0, 288.0};
        mem.outlier_every = 10.0;
        const wagma_placement::Result r = run("one region only", mem, 6.09, 1, false);
        check(r.w && r.m && r.pub && r.g, "one region only", "left-over candidates were not used");
    }
    {
        SimMemory mem;
        mem.boundaries_gib = three;
        mem.capacity_gib = 40.0;  // never leaves the first region
        const wagma_placement::Result r = run("little memory", mem, 6.09, 1, false);
        check(r.w && r.m && r.pub && r.g, "little memory", "left-over candidates were not used");
    }
    {
        SimMemory mem;
        mem.boundaries_gib = three;
        mem.capacity_gib = 15.0;  // room for two candidates only
        const wagma_placement::Result r = run("two candidates fit", mem, 6.09, 1, false);
        check((r.w != nullptr) + (r.m != nullptr) + (r.pub != nullptr) + (r.g != nullptr) == 2,
              "two candidates fit", "roles beyond the candidates");
    }
    {
        SimMemory mem;
        mem.boundaries_gib = three;
        run("arrays of 25.4 GiB", mem, 25.4, 3, false);
    }
    {
        SimMemory mem;
        mem.boundaries_gib = three;
        mem.scattered_gib = {100, 10, 130, 200, 20, 250, 40, 150, 60, 220};  // a used, fragmented GPU
        run("scattered placement", mem, 6.09, 3, true);
    }
    {
        SimMemory mem;
        mem.boundaries_gib = three;
        mem.pieced = {0, 2, 3, 17, 18, 33};  // arrays whose middle lies in another region
        mem.detour_gib = 100.0;
        run("arrays pieced from two regions", mem, 6.09, 3, true);
    }
    {
        SimMemory mem;
        mem.boundaries_gib = {0.0, 64.0, 128.0, 160.0, 192.0, 288.0};  // narrower, uneven regions
        mem.noise = 0.03;
        run("five uneven regions", mem, 6.09, 3, true);
    }
    {
        SimMemory mem;
        mem.boundaries_gib = three;
        run("arrays of 1.5 GiB (half-array probes)", mem, 1.52, 3, true);
    }
    std::printf(failures ? "%d FAILURES\n" : "all scenarios hold\n", failures);
    return failures ? 1 : 0;
}
