// Chunk-wise HBM-region placement for wagma_alloc_buffers: plain host C++ with no HIP in it
// (tests/chunks_sim.cpp exercises it on a CPU against a simulated memory).
//
// What is measured on MI355X and why regions matter is told in wagma_placement.h.  Here the
// four arrays are not taken from whole-array allocations but built, through the HIP virtual
// memory API, from physical chunks of 1 GiB whose region has been found by timing:
//   chunk j of w and of g   lies in region (j    ) mod 3
//   chunk j of m            lies in region (j + 1) mod 3
//   chunk j of pub          lies in region (j + 2) mod 3
// so that at every column the three arrays that are written (w, m, pub) lie in three regions
// and g lies with w, whatever the size of the arrays, and every region carries a third of
// the load.  This also works where whole arrays cannot be had cleanly: arrays of tens of
// GiB, or a GPU whose free memory is scattered over the regions.
// A second pattern takes every chunk of every array from ONE region (the class with the most
// chunks; arrays larger than a region go on with the next largest): what ordinary allocations
// look like on a GPU with untouched memory, rebuilt where the memory has been in use.  A third
// takes w, g and m from one region and pub, the array that is written and hardly ever read, from
// another.  Which of them the step runs fastest on depends on its kernel and on the GPU's
// memory (wagma_alloc_buffers times them).
//
// A Memory object provides
//   char*  new_chunk()                   maps one more physical chunk, nullptr when out of room
//   bool   skip(size_t bytes, size_t keep)   takes `bytes` of physical memory out of the way,
//                                        unless fewer than `keep` bytes would remain free
//   double rate(char* a, char* b, size_t side)   probe rate in GB/s, <= 0 on failure
// Chunks come in physical address order on a fresh GPU (about 96 of one region, then 96 of
// the next ...), so once a region has given enough chunks the search skips ahead.
#ifndef WAGMA_CHUNKS_H
#define WAGMA_CHUNKS_H

#include <cstddef>

namespace wagma_placement {

constexpr size_t kChunkBytes = size_t(1) << 30;
constexpr int kMaxChunks = 768;    // chunks examined at most
constexpr int kMaxClasses = 6;     // regions told apart at most (three are used)
constexpr int kRegionChunks = 88;  // chunks one region gives for certain (it holds about 96 GiB)
constexpr size_t kSkipBytes = size_t(8) << 30;
constexpr double kChunkMinSpread = 1.10;  // class means closer than this: only one cluster seen
constexpr int kChunkWarmupProbes = 40;

// Two clusters of probe rates and the threshold between them (see wagma_placement.h).
class RateClusters {
public:
    static constexpr int kMaxVals = 4096;
    static constexpr double kNone = 1e30;
    void see(double v)
    {
        if (n_ < kMaxVals)
            vals_[n_++] = v;
        // insertion into the sorted copy
        int j = n_sorted_;
        while (j > 0 && sorted_[j - 1] > v) {
            sorted_[j] = sorted_[j - 1];
            --j;
        }
        sorted_[j] = v;
        ++n_sorted_;
        double total = 0.0;
        for (int i = 0; i < n_sorted_; ++i)
            total += sorted_[i];
        slow_mean = total / n_sorted_;
        fast_mean = 0.0;
        threshold = kNone;
        double best = -1.0, low_sum = 0.0, split_at = kNone, lo_best = slow_mean, hi_best = 0.0;
        int k_best = 0;
        for (int k = 1; k < n_sorted_; ++k) {
            low_sum += sorted_[k - 1];
            const double lo = low_sum / k, hi = (total - low_sum) / (n_sorted_ - k);
            const double score = (double)k * (n_sorted_ - k) * (hi - lo) * (hi - lo);
            if (score > best) {
                best = score;
                split_at = 0.5 * (sorted_[k - 1] + sorted_[k]);
                lo_best = lo;
                hi_best = hi;
                k_best = k;
            }
        }
        // Two real clusters are about 18% apart and the slow one holds the larger part of the
        // readings (every chunk is probed against itself); a slow straggler or two do not make
        // a cluster.
        if (hi_best >= kChunkMinSpread * lo_best && k_best >= 2 && 4 * k_best >= n_sorted_) {
            threshold = split_at;
            slow_mean = lo_best;
            fast_mean = hi_best;
        }
    }
    bool full() const { return n_sorted_ >= kMaxVals; }
    double threshold = kNone;  // rates below: same region; at or above: different regions
    double slow_mean = 0.0, fast_mean = 0.0;

private:
    double vals_[kMaxVals];
    double sorted_[kMaxVals];
    int n_ = 0, n_sorted_ = 0;
};

struct ChunkPlan {
    // chunk index (order of Memory::new_chunk calls) for chunk j of each array, -1 = none
    int* w = nullptr;
    int* g = nullptr;
    int* m = nullptr;
    int* pub = nullptr;
    int per_array = 0;     // chunks per array
    int examined = 0;      // chunks mapped during the search
    int classes = 0;       // regions told apart
    int in_pattern = 0;    // array chunks that got a chunk of the region the pattern asks for
    double slow_gbs = 0.0, fast_gbs = 0.0;
};

// which region chunk j of each array comes from (region slots 0, 1, 2 are served by the classes with
// the most, second and third most chunks, the slot with the largest need by the largest class)
enum class ChunkPattern {
    rotate,      // w and g: j mod 3, m: (j + 1) mod 3, pub: (j + 2) mod 3
    one_region,  // everything from one
    pub_apart    // w, g, m from one, pub from another
};

template <typename Memory>
class ChunkSearch {
public:
    ChunkSearch(Memory& memory, int chunks_per_array, ChunkPattern pattern = ChunkPattern::rotate)
        : mem_(memory), k_(chunks_per_array), pattern_(pattern)
    {
    }

    // Fills plan.w/g/m/pub (arrays of chunks_per_array ints owned by the caller).  Returns
    // false if fewer than 4 * chunks_per_array chunks could be had at all.
    bool run(ChunkPlan& plan)
    {
        int need[3] = {0, 0, 0};
        for (int j = 0; j < k_; ++j)
            for (int a = 0; a < 4; ++a)
                need[slot(j, a)] += 1;
        const size_t side = kChunkBytes / 2;
        while (n_ < kMaxChunks && !failed_ && !clusters_.full()) {
            // the three regions with the most chunks so far are the ones that will be used
            int top[3];
            top_classes(top);
            const int classes_wanted = pattern_ == ChunkPattern::one_region ? 1 : pattern_ == ChunkPattern::pub_apart ? 2 : 3;
            bool enough = n_classes_ >= classes_wanted;
            for (int r = 0; r < 3 && enough; ++r) {
                int wanted = need_sorted(need, r);
                // arrays that a region cannot hold: once it has given what a region has, the
                // rest comes from the others
                if (pattern_ != ChunkPattern::rotate && wanted > kRegionChunks)
                    wanted = kRegionChunks;
                enough = count_[top[r]] >= wanted;
            }
            enough = enough && n_ >= 4 * k_;
            if (enough)
                break;
            char* c = mem_.new_chunk();
            if (!c)
                break;
            if (n_ == 0)
                for (int rep = 0; rep < kChunkWarmupProbes; ++rep)
                    (void)mem_.rate(c, c + side, side);
            chunk_[n_] = c;
            class_[n_] = classify(c, side);
            if (class_[n_] >= 0)
                ++count_[class_[n_]];
            ++n_;
            // with the threshold known by now, a chunk that looked uniform earlier may turn out
            // to be spread over two regions
            for (int i = 0; i < n_; ++i) {
                if (class_[i] >= 0 && inner_[i] >= clusters_.threshold) {
                    --count_[class_[i]];
                    class_[i] = -1;
                }
            }
            // a region that has already given more than any array pattern can use: move on
            // faster, as long as enough memory stays free for the chunks still to come
            const int cls = class_[n_ - 1];
            if (cls >= 0 && count_[cls] > need_sorted(need, 0) + 2 && !skip_failed_) {
                const size_t still = (size_t)(4 * k_ > n_ ? 4 * k_ - n_ : 0) + 4;
                skip_failed_ = !mem_.skip(kSkipBytes, still * kChunkBytes);
            }
        }
        plan.per_array = k_;
        plan.examined = n_;
        plan.classes = n_classes_;
        plan.slow_gbs = clusters_.slow_mean;
        plan.fast_gbs = clusters_.fast_mean;
        if (n_ < 4 * k_)
            return false;
        // hand out: region slot r of the pattern is served by the r-th most populated class
        int top[3];
        top_classes(top);
        // the class with the most chunks serves the slot with the largest need
        int slot_order[3] = {0, 1, 2};
        for (int a = 0; a < 3; ++a)
            for (int b = a + 1; b < 3; ++b)
                if (need[slot_order[b]] > need[slot_order[a]]) {
                    const int t = slot_order[a];
                    slot_order[a] = slot_order[b];
                    slot_order[b] = t;
                }
        int class_of_slot[3] = {-1, -1, -1};
        for (int r = 0; r < 3; ++r)
            class_of_slot[slot_order[r]] = r < n_classes_ ? top[r] : -1;
        for (int i = 0; i < n_; ++i)
            used_[i] = false;
        plan.in_pattern = 0;
        int* arrays[4] = {plan.w, plan.g, plan.m, plan.pub};
        for (int pass = 0; pass < 2; ++pass) {  // first the chunks the pattern asks for, then any
            for (int a = 0; a < 4; ++a) {
                for (int j = 0; j < k_; ++j) {
                    if (pass == 0)
                        arrays[a][j] = -1;
                    if (arrays[a][j] >= 0)
                        continue;
                    const int want = class_of_slot[slot(j, a)];
                    int got = -1;
                    if (pass == 0)
                        got = take(want);
                    // what a region cannot give comes from a region the pattern does not use, from
                    // as few as possible (ordinary allocations in untouched memory look like that)
                    for (int r = 0; r < 2 && pass == 1 && pattern_ != ChunkPattern::rotate && got < 0; ++r) {
                        const int next = pattern_ == ChunkPattern::one_region ? 1 + r : 2 - r;
                        if (next < n_classes_)
                            got = take(top[next]);
                    }
                    if (pass == 1 && got < 0)
                        got = take(-2);
                    arrays[a][j] = got;
                    if (pass == 0 && got >= 0)
                        ++plan.in_pattern;
                }
            }
        }
        return true;
    }

    int chunks() const { return n_; }
    char* chunk(int i) const { return chunk_[i]; }
    int chunk_class(int i) const { return class_[i]; }
    bool chunk_used(int i) const { return used_[i]; }

private:
    // which of the three region slots chunk j of array a (w, g, m, pub) asks for
    int slot(int j, int a) const
    {
        const int shift[4] = {0, 0, 1, 2};
        switch (pattern_) {
        case ChunkPattern::one_region: return 0;
        case ChunkPattern::pub_apart: return a == 3 ? 1 : 0;
        default: return (j + shift[a]) % 3;
        }
    }
    static int need_sorted(const int need[3], int rank)
    {
        int s[3] = {need[0], need[1], need[2]};
        for (int a = 0; a < 3; ++a)
            for (int b = a + 1; b < 3; ++b)
                if (s[b] > s[a]) {
                    const int t = s[a];
                    s[a] = s[b];
                    s[b] = t;
                }
        return s[rank];
    }
    void top_classes(int top[3]) const
    {
        top[0] = top[1] = top[2] = -1;
        for (int r = 0; r < 3; ++r) {
            int best = -1;
            for (int c = 0; c < n_classes_; ++c) {
                if (c == top[0] || c == top[1])
                    continue;
                if (best < 0 || count_[c] > count_[best])
                    best = c;
            }
            top[r] = best;
        }
        for (int r = 0; r < 3; ++r)
            if (top[r] < 0)
                top[r] = 0;
    }
    double measure(char* a, char* b, size_t side)
    {
        double v = mem_.rate(a, b, side);
        if (v > 0.0 && v < clusters_.threshold) {  // a slow reading is confirmed (see wagma_placement.h)
            const double again = mem_.rate(a, b, side);
            if (again <= 0.0 || again > v)
                v = again;
        }
        if (v <= 0.0)
            failed_ = true;
        else
            clusters_.see(v);
        return v;
    }
    // The region class of a new chunk: the first reference chunk it is "slow" with; a chunk
    // that is fast with every reference founds a new class.  -1: the chunk is itself spread
    // over regions (its two halves are fast with each other), or there are too many classes.
    int classify(char* c, size_t side)
    {
        const double inner = measure(c, c + side, side);
        inner_[n_] = inner;
        if (failed_)
            return -1;
        int cls = -1;
        for (int r = 0; r < n_classes_ && cls < 0 && !failed_; ++r)
            if (measure(ref_[r], c, side) < clusters_.threshold)
                cls = r;
        if (failed_ || inner >= clusters_.threshold)
            return -1;
        if (cls < 0 && n_classes_ < kMaxClasses) {
            ref_[n_classes_] = c;
            count_[n_classes_] = 0;
            cls = n_classes_++;
        }
        return cls;
    }
    // an unused chunk of class `want` (-2: of any class, classified ones last), or -1
    int take(int want)
    {
        if (want == -1)
            return -1;
        for (int pass = 0; pass < 2; ++pass) {
            for (int i = 0; i < n_; ++i) {
                if (used_[i])
                    continue;
                const bool ok = want >= 0 ? class_[i] == want : (pass == 0 ? class_[i] < 0 : true);
                if (ok) {
                    used_[i] = true;
                    return i;
                }
            }
            if (want >= 0)
                break;
        }
        return -1;
    }

    Memory& mem_;
    int k_;
    ChunkPattern pattern_;
    RateClusters clusters_;
    char* chunk_[kMaxChunks];
    int class_[kMaxChunks];
    double inner_[kMaxChunks];  // probe rate between the two halves of a chunk
    bool used_[kMaxChunks];
    char* ref_[kMaxClasses];
    int count_[kMaxClasses] = {0, 0, 0, 0, 0, 0};
    int n_ = 0, n_classes_ = 0;
    bool failed_ = false, skip_failed_ = false;
};

}  // namespace wagma_placement

#endif  // WAGMA_CHUNKS_H
