// HBM-region search of wagma_alloc_buffers: plain host C++ with no HIP in it, so that the
// logic can also be exercised on a CPU against a simulated memory (tests/placement_sim.cpp).
//
// Measured on MI355X: the HBM is split, by the top physical address bits, into a few regions
// of tens of GiB (three of about 96 GiB on the 288 GiB part, by all appearance the ranks of
// the 12-high stacks).  Write streams that all fall into one region sustain about 5.9 TB/s,
// write streams spread over two regions about 7.1 TB/s; reads do not care.  The step writes
// W, the momentum and the send buffer of every member row at once, so it runs about 15%
// faster when these three arrays lie in three regions, and the read-only gradient array is
// best placed in the region of W (and worst in that of the send buffer).
//
// Regions cannot be queried; they are found by timing.  A Memory object provides
//   char*  allocate(size_t bytes)      a new candidate array, or nullptr when there is no room
//   void   release(char*)
//   double rate(char* a, char* b, size_t side)   GB/s of a probe that writes `side` bytes
//                                       through a and through b; <= 0 on failure
// and the search allocates candidates one after another (the driver hands out physical memory
// in address order, so later candidates lie further on).  Probe rates fall into two clusters
// about 18% apart: both pointers in one region (slow) or in two regions (fast).  The
// threshold between them is re-estimated from all rates measured so far (the split of the
// sorted rates that maximises the between-class variance, accepted only if the class means
// are 10% apart), and the roles are re-derived from the stored measurements after every new
// candidate, so that an unlucky first candidate or a noisy probe cannot mislead the search.
#ifndef WAGMA_PLACEMENT_H
#define WAGMA_PLACEMENT_H

#include <cstddef>

namespace wagma_placement {

constexpr int kMaxCandidates = 64;
constexpr size_t kProbeSideMax = size_t(1) << 30;       // bytes written through each pointer: well
                                                        // beyond the 256 MB Infinity Cache
constexpr size_t kPlacementMinBytes = size_t(1) << 30;  // smaller arrays are not placed
constexpr double kMinSpread = 1.10;  // class means closer than this: only one cluster was seen
constexpr int kWarmupProbes = 40;    // an idle GPU needs a while to bring its clocks up
constexpr int kWindows = 6;          // places inside a candidate that are compared with its start
constexpr size_t kMinStride = size_t(4) << 30;  // candidates of small arrays are spaced this far
                                                // apart, so that 64 of them span the memory

struct Result {
    char* w = nullptr;    // arrays in pairwise different regions ...
    char* m = nullptr;
    char* pub = nullptr;
    char* g = nullptr;    // ... and one in the region of w
    int candidates = 0;   // allocations tried
    int regions = 1;      // how many of w, m, pub are known to lie in different regions (1..3)
    bool g_with_w = false;
    double slow_gbs = 0.0, fast_gbs = 0.0;  // means of the two clusters of probe rates
};

template <typename Memory>
class RegionSearch {
public:
    RegionSearch(Memory& memory, size_t array_bytes) : mem_(memory), bytes_(array_bytes)
    {
        side_ = bytes_ / 2 < kProbeSideMax ? bytes_ / 2 : kProbeSideMax;  // at most half an array
        side_ = side_ / 1024 * 1024;
        // windows of `side_` bytes spread evenly from behind the first one to the end of the array
        windows_ = (int)(bytes_ / side_) - 1;
        if (windows_ > kWindows)
            windows_ = kWindows;
        if (windows_ < 1)
            windows_ = 1;
    }

    // Allocates candidates until w, m, pub and g have their places or memory runs out; every
    // candidate without a role is released again.  Roles that could not be filled stay nullptr.
    Result run()
    {
        while (!complete() && !failed_ && n_ < kMaxCandidates) {
            char* c = mem_.allocate(bytes_);
            if (!c)
                break;
            add(c);
            assign();
            // w and g sit side by side; after that, small arrays move on in larger steps
            if (!complete() && w_ >= 0 && (g_ >= 0 || m_ >= 0) && bytes_ < kMinStride && n_spacers_ < kMaxCandidates) {
                char* spacer = mem_.allocate(kMinStride - bytes_);
                if (spacer)
                    spacers_[n_spacers_++] = spacer;
            }
        }
        for (int k = 0; k < n_spacers_; ++k)
            mem_.release(spacers_[k]);
        Result r;
        r.candidates = n_;
        r.slow_gbs = slow_mean_;
        r.fast_gbs = fast_mean_;
        r.regions = (w_ >= 0) + (m_ >= 0) + (pub_ >= 0);
        if (r.regions == 0)
            r.regions = 1;
        r.g_with_w = g_ >= 0;
        for (int i = 0; i < n_; ++i) {
            if (i == w_)
                r.w = cand_[i];
            else if (i == m_)
                r.m = cand_[i];
            else if (i == pub_)
                r.pub = cand_[i];
            else if (i == g_ || (g_ < 0 && i == g_alt_))
                r.g = cand_[i];
            else
                spare_[n_spare_++] = cand_[i];
        }
        // a role without a place takes any left-over candidate; the others go back
        char** roles[4] = {&r.w, &r.m, &r.pub, &r.g};
        for (char** role : roles)
            if (!*role && n_spare_ > 0)
                *role = spare_[--n_spare_];
        for (int k = 0; k < n_spare_; ++k)
            mem_.release(spare_[k]);
        return r;
    }

    // for the debug report
    int count() const { return n_; }
    double threshold() const { return threshold_; }
    double inner_rate(int i) const { return inner_[i]; }
    double cross_rate(int i, int j) const { return cross_[i][j]; }
    char* candidate(int i) const { return cand_[i]; }
    int role_w() const { return w_; }
    int role_m() const { return m_; }
    int role_pub() const { return pub_; }
    int role_g() const { return g_; }

private:
    void see(double v)
    {
        if (v <= 0.0) {
            failed_ = true;
            return;
        }
        if (n_vals_ < kMaxVals)
            vals_[n_vals_++] = v;
        double sorted[kMaxVals];
        for (int i = 0; i < n_vals_; ++i)
            sorted[i] = vals_[i];
        for (int i = 1; i < n_vals_; ++i) {  // insertion sort: a few hundred values at most
            const double x = sorted[i];
            int j = i - 1;
            while (j >= 0 && sorted[j] > x) {
                sorted[j + 1] = sorted[j];
                --j;
            }
            sorted[j + 1] = x;
        }
        double total = 0.0;
        for (int i = 0; i < n_vals_; ++i)
            total += sorted[i];
        slow_mean_ = total / n_vals_;
        fast_mean_ = 0.0;
        threshold_ = kNoThreshold;
        double best = -1.0, low_sum = 0.0, split_at = kNoThreshold, lo_best = slow_mean_, hi_best = 0.0;
        int k_best = 0;
        for (int k = 1; k < n_vals_; ++k) {  // k values in the slow class
            low_sum += sorted[k - 1];
            const double lo = low_sum / k, hi = (total - low_sum) / (n_vals_ - k);
            const double score = (double)k * (n_vals_ - k) * (hi - lo) * (hi - lo);
            if (score > best) {
                best = score;
                split_at = 0.5 * (sorted[k - 1] + sorted[k]);
                lo_best = lo;
                hi_best = hi;
                k_best = k;
            }
        }
        // Two real clusters are about 18% apart and the slow one holds a good part of the
        // readings (every candidate is probed against itself); a slow straggler or two do not
        // make a cluster, and a split of mere noise is none.
        if (hi_best >= kMinSpread * lo_best && k_best >= 2 && 4 * k_best >= n_vals_) {
            threshold_ = split_at;
            slow_mean_ = lo_best;
            fast_mean_ = hi_best;
        }
    }

    // A probe disturbed by something else reads slow, never fast, and a slow reading is what
    // lets two pointers pass for "same region": a reading in the slow class is taken twice
    // and the larger value counts.
    double measure(char* a, char* b)
    {
        double v = mem_.rate(a, b, side_);
        if (v > 0.0 && v < threshold_) {
            const double again = mem_.rate(a, b, side_);
            if (again <= 0.0 || again > v)
                v = again;
        }
        return v;
    }

    void add(char* c)
    {
        cand_[n_] = c;
        for (int k = 0; k <= n_; ++k)
            cross_[n_][k] = cross_[k][n_] = 0.0;
        if (n_ == 0)
            for (int rep = 0; rep < kWarmupProbes; ++rep)
                (void)mem_.rate(c, c + side_, side_);
        // A candidate may straddle two regions, or be pieced together from several (a GPU whose
        // memory is fragmented): its start is compared with windows all along it, and the
        // fastest of these readings tells.
        inner_[n_] = 0.0;
        for (int j = 1; j <= windows_; ++j) {
            const size_t at = (side_ + (bytes_ - 2 * side_) / windows_ * j) / 16 * 16;
            const double v = measure(c, c + at);
            see(v);
            if (v > inner_[n_])
                inner_[n_] = v;
        }
        ++n_;
        if (n_ > 1)
            (void)between(0, n_ - 1);  // one rate per candidate that does not depend on the roles
    }

    double between(int i, int j)
    {
        if (cross_[i][j] == 0.0) {
            cross_[i][j] = cross_[j][i] = measure(cand_[i], cand_[j]);
            see(cross_[i][j]);
        }
        return cross_[i][j];
    }

    // a candidate that does not lie in one region is of no use
    bool clean(int i) const { return inner_[i] < threshold_; }

    // Greedy roles in allocation order; repeated while new probes keep moving the threshold.
    void assign()
    {
        for (int round = 0; round < 8 && !failed_; ++round) {
            const double threshold_before = threshold_;
            w_ = m_ = pub_ = g_ = g_alt_ = -1;
            for (int i = 0; i < n_ && !failed_; ++i) {
                if (!clean(i))
                    continue;
                if (w_ < 0) {
                    w_ = i;
                    continue;
                }
                const int placed[3] = {w_, m_, pub_};
                bool apart = true, with_w = false, with_m = false;
                for (int k = 0; k < 3 && placed[k] >= 0; ++k) {
                    if (between(placed[k], i) < threshold_) {
                        apart = false;
                        if (k == 0)
                            with_w = true;
                        if (k == 1)
                            with_m = true;
                    }
                }
                if (apart && m_ < 0)
                    m_ = i;
                else if (apart && pub_ < 0)
                    pub_ = i;
                else if (with_w && g_ < 0)
                    g_ = i;
                else if (with_m && g_alt_ < 0)
                    g_alt_ = i;  // second best for g: next to m (anywhere but next to pub)
            }
            if (threshold_ == threshold_before)
                break;  // the yardstick did not move: the roles stand
        }
        if (threshold_ == kNoThreshold)
            m_ = pub_ = -1;  // only one cluster seen: nothing is known to be apart
    }

    bool complete() const { return w_ >= 0 && m_ >= 0 && pub_ >= 0 && (g_ >= 0 || g_alt_ >= 0); }

    static constexpr int kMaxVals = kMaxCandidates * 12;  // at most 10 readings per candidate
    static constexpr double kNoThreshold = 1e30;

    Memory& mem_;
    size_t bytes_, side_ = 0;
    int windows_ = 1;
    char* cand_[kMaxCandidates];
    char* spare_[kMaxCandidates];
    char* spacers_[kMaxCandidates];
    double inner_[kMaxCandidates];  // fastest reading between a candidate's start and its windows
    double cross_[kMaxCandidates][kMaxCandidates];  // 0 = not measured yet
    double vals_[kMaxVals];
    int n_ = 0, n_vals_ = 0, n_spare_ = 0, n_spacers_ = 0;
    double threshold_ = kNoThreshold;  // rates below: same region; at or above: different regions
    double slow_mean_ = 0.0, fast_mean_ = 0.0;
    int w_ = -1, m_ = -1, pub_ = -1, g_ = -1, g_alt_ = -1;  // indices into cand_
    bool failed_ = false;
};

}  // namespace wagma_placement

#endif  // WAGMA_PLACEMENT_H
