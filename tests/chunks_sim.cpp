// CPU simulation of the chunk-wise region placement (csrc/wagma_chunks.h): a fake memory that
// hands out 1 GiB chunks in physical order or scattered, with noisy probe rates and slow
// stragglers.  Exits non-zero if an invariant of the plan is violated.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <set>
#include <vector>

#include "wagma_chunks.h"

namespace {

constexpr double kGiB = 1024.0 * 1024.0 * 1024.0;
constexpr uintptr_t kBase = uintptr_t(1) << 44;

struct SimMemory {
    std::vector<double> boundaries_gib;
    double capacity_gib = 288.0, next_gib = 0.0;
    std::vector<double> scattered_gib;  // if not empty: where the i-th chunk lies
    std::set<int> mixed;                // chunks whose second half lies in the next region
    int chunks = 0;
    double slow = 5900.0, fast = 7000.0, noise = 0.03, straggler_every = 0.0;
    uint64_t rng = 88172645463325252ull;
    long probes = 0;
    double skipped_gib = 0.0;

    double uniform()
    {
        rng ^= rng << 13;
        rng ^= rng >> 7;
        rng ^= rng << 17;
        return (double)(rng >> 11) / 9007199254740992.0;
    }
    int region_at(double gib) const
    {
        for (size_t k = 0; k + 1 < boundaries_gib.size(); ++k)
            if (gib >= boundaries_gib[k] && gib < boundaries_gib[k + 1])
                return (int)k;
        return (int)boundaries_gib.size();
    }
    std::vector<std::pair<double, int>> where;  // chunk -> (start GiB, index)
    int region_of_half(char* p) const
    {
        const double off = ((uintptr_t)p - kBase) / kGiB;  // position in the scratch window
        const int idx = (int)off;
        const bool second = off - idx >= 0.5;
        int r = region_at(where[idx].first + (second ? 0.5 : 0.0));
        if (second && mixed.count(idx))
            r = (r + 1) % 3;
        return r;
    }
    char* new_chunk()
    {
        double at;
        if (!scattered_gib.empty()) {
            if ((size_t)chunks >= scattered_gib.size())
                return nullptr;
            at = scattered_gib[chunks];
        } else {
            if (next_gib + 1.0 > capacity_gib)
                return nullptr;
            at = next_gib;
            next_gib += 1.0;
        }
        where.push_back({at, chunks});
        return (char*)(kBase + (uintptr_t)(chunks++ * kGiB));
    }
    bool skip(size_t bytes, size_t keep)
    {
        if (!scattered_gib.empty())
            return true;
        if (next_gib + (bytes + keep) / kGiB > capacity_gib)
            return false;
        next_gib += bytes / kGiB;
        skipped_gib += bytes / kGiB;
        return true;
    }
    double rate(char* a, char* b, size_t)
    {
        ++probes;
        double r = region_of_half(a) == region_of_half(b) ? slow : fast;
        r *= 1.0 + noise * (2.0 * uniform() - 1.0);
        if (straggler_every > 0.0 && uniform() < 1.0 / straggler_every)
            r *= 0.87;
        return r;
    }
    int region_of_chunk(int idx) const { return region_at(where[idx].first + 0.25); }
};

int failures = 0;
void check(bool ok, const char* scenario, const char* what)
{
    if (!ok) {
        std::printf("FAIL %s: %s\n", scenario, what);
        ++failures;
    }
}

void run(const char* name, SimMemory& mem, int k, bool expect_plan, int min_in_pattern_percent)
{
    std::vector<int> w(k), g(k), m(k), pub(k);
    wagma_placement::ChunkPlan plan;
    plan.w = w.data();
    plan.g = g.data();
    plan.m = m.data();
    plan.pub = pub.data();
    auto* search = new wagma_placement::ChunkSearch<SimMemory>(mem, k);
    const bool ok = search->run(plan);
    std::printf("%-34s plan %d  examined %3d  classes %d  in pattern %3d/%3d  probes %4ld  skipped %3.0f GiB\n", name,
                (int)ok, plan.examined, plan.classes, plan.in_pattern, 4 * k, mem.probes, mem.skipped_gib);
    check(ok == expect_plan, name, "plan / no plan");
    if (ok) {
        std::set<int> seen;
        int good = 0;
        for (int j = 0; j < k; ++j) {
            for (int idx : {w[j], g[j], m[j], pub[j]}) {
                check(idx >= 0 && idx < plan.examined, name, "a slot without a chunk");
                check(seen.insert(idx).second, name, "a chunk used twice");
            }
            if (w[j] < 0 || g[j] < 0 || m[j] < 0 || pub[j] < 0)
                continue;
            const int rw = mem.region_of_chunk(w[j]), rg = mem.region_of_chunk(g[j]);
            const int rm = mem.region_of_chunk(m[j]), rp = mem.region_of_chunk(pub[j]);
            const bool clean = !mem.mixed.count(w[j]) && !mem.mixed.count(m[j]) && !mem.mixed.count(pub[j]);
            if (rw != rm && rw != rp && rm != rp && rg == rw && clean)
                ++good;
        }
        check(100 * good >= min_in_pattern_percent * k, name, "too few columns with w, m, pub in three regions and g with w");
    }
    delete search;
}

// The other pattern: all chunks of all four arrays from one region.
void run_one_region(const char* name, SimMemory& mem, int k, bool expect_plan, int min_same_percent)
{
    std::vector<int> w(k), g(k), m(k), pub(k);
    wagma_placement::ChunkPlan plan;
    plan.w = w.data();
    plan.g = g.data();
    plan.m = m.data();
    plan.pub = pub.data();
    auto* search = new wagma_placement::ChunkSearch<SimMemory>(mem, k, wagma_placement::ChunkPattern::one_region);
    const bool ok = search->run(plan);
    std::printf("%-44s plan %d  examined %3d  classes %d  in pattern %3d/%3d  probes %4ld  skipped %3.0f GiB\n", name,
                (int)ok, plan.examined, plan.classes, plan.in_pattern, 4 * k, mem.probes, mem.skipped_gib);
    check(ok == expect_plan, name, "plan / no plan");
    if (ok) {
        std::set<int> seen;
        int in_region[8] = {0, 0, 0, 0, 0, 0, 0, 0}, mixed = 0;
        for (int j = 0; j < k; ++j)
            for (int idx : {w[j], g[j], m[j], pub[j]}) {
                check(idx >= 0 && idx < plan.examined, name, "a slot without a chunk");
                check(seen.insert(idx).second, name, "a chunk used twice");
                if (idx >= 0) {
                    ++in_region[mem.region_of_chunk(idx) & 7];
                    mixed += (int)mem.mixed.count(idx);
                }
            }
        int most = 0, second = 0;
        for (int c : in_region) {
            if (c > most) {
                second = most;
                most = c;
            } else if (c > second) {
                second = c;
            }
        }
        check(100 * (most - mixed) >= min_same_percent * 4 * k, name, "too few chunks from one region");
        // what the one region could not give comes from one other region, if that one has enough
        if (min_same_percent < 100 && mem.noise < 0.035)
            check(most + second == 4 * k, name, "the rest is spread over more than one other region");
    }
    delete search;
}

// The third pattern: w, g and m from one region, pub from another.
void run_pub_apart(const char* name, SimMemory& mem, int k, int min_right_percent)
{
    std::vector<int> w(k), g(k), m(k), pub(k);
    wagma_placement::ChunkPlan plan;
    plan.w = w.data();
    plan.g = g.data();
    plan.m = m.data();
    plan.pub = pub.data();
    auto* search = new wagma_placement::ChunkSearch<SimMemory>(mem, k, wagma_placement::ChunkPattern::pub_apart);
    const bool ok = search->run(plan);
    std::printf("%-44s plan %d  examined %3d  classes %d  in pattern %3d/%3d  probes %4ld  skipped %3.0f GiB\n", name,
                (int)ok, plan.examined, plan.classes, plan.in_pattern, 4 * k, mem.probes, mem.skipped_gib);
    check(ok, name, "no plan");
    if (ok) {
        std::set<int> seen;
        int main_region[8] = {0, 0, 0, 0, 0, 0, 0, 0}, pub_region[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int j = 0; j < k; ++j) {
            for (int idx : {w[j], g[j], m[j], pub[j]}) {
                check(idx >= 0 && idx < plan.examined, name, "a slot without a chunk");
                check(seen.insert(idx).second, name, "a chunk used twice");
            }
            for (int idx : {w[j], g[j], m[j]})
                if (idx >= 0 && !mem.mixed.count(idx))
                    ++main_region[mem.region_of_chunk(idx) & 7];
            if (pub[j] >= 0 && !mem.mixed.count(pub[j]))
                ++pub_region[mem.region_of_chunk(pub[j]) & 7];
        }
        int a = 0, b = 0;
        for (int r = 1; r < 8; ++r) {
            a = main_region[r] > main_region[a] ? r : a;
            b = pub_region[r] > pub_region[b] ? r : b;
        }
        check(a != b, name, "pub lies where w, g and m lie");
        check(100 * (main_region[a] + pub_region[b]) >= min_right_percent * 4 * k, name, "too few chunks where the pattern wants them");
    }
    delete search;
}

}  // namespace

int main()
{
    {
        const std::vector<double> three = {0.0, 96.0, 192.0, 288.0};
        for (int k : {2, 7, 27}) {
            SimMemory mem;
            mem.boundaries_gib = three;
            char name[64];
            std::snprintf(name, sizeof name, "pub apart: fresh memory, %d chunks per array", k);
            run_pub_apart(name, mem, k, 100);
        }
        for (int seed = 1; seed <= 6; ++seed) {
            SimMemory mem;
            mem.boundaries_gib = three;
            mem.noise = 0.04;
            mem.straggler_every = 12.0;
            mem.rng ^= (uint64_t)seed * 0x9E3779B97F4A7C15ull;
            for (int i = 0; i < 200; ++i)
                mem.scattered_gib.push_back((double)((i * (31 + 2 * seed)) % 280));
            char name[64];
            std::snprintf(name, sizeof name, "pub apart: scattered, noise, seed %d", seed);
            run_pub_apart(name, mem, 7, 90);
        }
        {
            SimMemory mem;
            mem.boundaries_gib = three;
            for (int i = 0; i < 160; ++i)
                mem.scattered_gib.push_back((double)((i * 37) % 280));
            mem.mixed = {0, 3, 4, 11, 30};
            run_pub_apart("pub apart: scattered, some chunks mixed", mem, 7, 100);
        }
        {
            // arrays of 35 chunks: w, g, m need 105, a region has 96; the rest comes from the third region
            SimMemory mem;
            mem.boundaries_gib = three;
            for (int i = 0; i < 280; ++i)
                mem.scattered_gib.push_back((double)((i * 37) % 280));
            run_pub_apart("pub apart: 105 + 35 chunks needed", mem, 35, 85);
        }
    }
    {
        const std::vector<double> three = {0.0, 96.0, 192.0, 288.0};
        for (int k : {2, 7, 20}) {
            SimMemory mem;
            mem.boundaries_gib = three;
            char name[64];
            std::snprintf(name, sizeof name, "one region: fresh memory, %d chunks per array", k);
            run_one_region(name, mem, k, true, 100);
        }
        for (int seed = 1; seed <= 6; ++seed) {
            SimMemory mem;
            mem.boundaries_gib = three;
            mem.noise = 0.04;
            mem.straggler_every = 12.0;
            mem.rng ^= (uint64_t)seed * 0x9E3779B97F4A7C15ull;
            for (int i = 0; i < 200; ++i)
                mem.scattered_gib.push_back((double)((i * (31 + 2 * seed)) % 280));
            char name[64];
            std::snprintf(name, sizeof name, "one region: scattered, noise, seed %d", seed);
            run_one_region(name, mem, 7, true, 90);
        }
        {
            SimMemory mem;
            mem.boundaries_gib = three;
            for (int i = 0; i < 160; ++i)
                mem.scattered_gib.push_back((double)((i * 37) % 280));
            mem.mixed = {0, 3, 4, 11, 30};
            run_one_region("one region: scattered, some chunks mixed", mem, 7, true, 100);
        }
        {
            SimMemory mem;
            mem.boundaries_gib = {0.0, 288.0};
            mem.straggler_every = 10.0;
            run_one_region("one region: one region only", mem, 7, true, 100);
        }
        {
            SimMemory mem;
            mem.boundaries_gib = three;
            mem.capacity_gib = 20.0;
            run_one_region("one region: memory for 20 chunks, 28 needed", mem, 7, false, 0);
        }
        {
            // arrays larger than a region (workload 5: 27 chunks per array): the search ends once a
            // region has given what a region has, the rest comes from one other region
            SimMemory mem;
            mem.boundaries_gib = three;
            for (int i = 0; i < 280; ++i)
                mem.scattered_gib.push_back((double)((i * 37) % 280));
            run_one_region("one region: 108 chunks needed, regions of 96", mem, 27, true, 80);
        }
        {
            // a region too small to give all the chunks: the plan is filled up from the others
            SimMemory mem;
            mem.boundaries_gib = {0.0, 20.0, 40.0, 60.0};
            mem.capacity_gib = 60.0;
            run_one_region("one region: three regions of 20 chunks, 28 needed", mem, 7, true, 60);
        }
    }
    const std::vector<double> three = {0.0, 96.0, 192.0, 288.0};
    for (int k : {2, 7, 15, 26}) {
        SimMemory mem;
        mem.boundaries_gib = three;
        char name[64];
        std::snprintf(name, sizeof name, "fresh memory, %d chunks per array", k);
        run(name, mem, k, true, 100);
    }
    for (int seed = 1; seed <= 10; ++seed) {
        SimMemory mem;
        mem.boundaries_gib = three;
        mem.noise = 0.04;
        mem.straggler_every = 12.0;
        mem.rng ^= (uint64_t)seed * 0x9E3779B97F4A7C15ull;
        mem.next_gib = 9.5 * seed;
        char name[64];
        std::snprintf(name, sizeof name, "noise and stragglers, seed %d", seed);
        run(name, mem, 7, true, seed <= 6 ? 100 : 0);   // late starts may not reach three regions
    }
    {
        SimMemory mem;
        mem.boundaries_gib = three;
        for (int i = 0; i < 120; ++i)  // a used GPU: free memory scattered over the regions
            mem.scattered_gib.push_back((double)((i * 37) % 280));
        run("scattered chunks", mem, 7, true, 100);
    }
    {
        SimMemory mem;
        mem.boundaries_gib = three;
        for (int i = 0; i < 120; ++i)
            mem.scattered_gib.push_back((double)((i * 37) % 280));
        mem.mixed = {0, 3, 4, 11, 30};  // chunks that are themselves pieced from two regions
        run("scattered, some chunks mixed", mem, 7, true, 100);
    }
    {
        SimMemory mem;
        mem.boundaries_gib = {0.0, 288.0};
        mem.straggler_every = 10.0;
        run("one region only", mem, 7, true, 0);
    }
    {
        SimMemory mem;
        mem.boundaries_gib = three;
        mem.capacity_gib = 20.0;
        run("memory for 20 chunks, 28 needed", mem, 7, false, 0);
    }
    {
        SimMemory mem;
        mem.boundaries_gib = three;
        mem.capacity_gib = 60.0;
        run("memory inside the first region", mem, 7, true, 0);
    }
    {
        SimMemory mem;
        mem.boundaries_gib = {0.0, 64.0, 128.0, 160.0, 192.0, 288.0};
        run("five uneven regions", mem, 7, true, 100);
    }
    std::printf(failures ? "%d FAILURES\n" : "all scenarios hold\n", failures);
    return failures ? 1 : 0;
}
