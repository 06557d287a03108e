// Who is late in which iteration: the host-side generators behind wagma_stale_mask,
// wagma_straggler_mask, wagma_clock_mask and wagma_lag_masks.  Plain host C++ with no HIP in
// it and integer arithmetic only, so that any two implementations agree bit for bit
// (tests/masks_host.cpp runs these on a CPU).  Arguments are checked by the callers.
//
// A mask is ceil(P/64) words; bit p of the mask = process p.
#ifndef WAGMA_MASKS_H
#define WAGMA_MASKS_H

#include <cstdint>
#include <functional>
#include <queue>
#include <vector>

namespace wagma_masks {

constexpr uint64_t kIterStride = UINT64_C(0x9E3779B97F4A7C15);
constexpr uint64_t kRankStride = UINT64_C(0xD1B54A32D192ED03);
constexpr uint64_t kStragglerTag = UINT64_C(0x5354524147474C52);  // keeps the models independent
constexpr uint64_t kClockTag = UINT64_C(0x434C4F434B4D534B);
constexpr uint32_t kShortestStepMs = 1700;

// Algorithm 2 line 8: iteration t ends in the global average iff (t+1) mod tau == 0.
inline bool is_global_iteration(int tau, int64_t iter)
{
    return tau > 0 && (iter + 1) % tau == 0;
}

// 64-bit finaliser of the public splitmix64 generator (Steele, Lea, Flood 2014).
inline uint64_t mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * UINT64_C(0xBF58476D1CE4E5B9);
    z = (z ^ (z >> 27)) * UINT64_C(0x94D049BB133111EB);
    return z ^ (z >> 31);
}

inline void clear(int P, uint64_t* words)
{
    for (int k = 0; k < (P + 63) / 64; ++k)
        words[k] = 0;
}

inline void set_bit(uint64_t* words, int rank)
{
    words[rank >> 6] |= UINT64_C(1) << (rank & 63);
}

// Process p is late iff the top 32 bits of a hash of (seed, iter, p) are below threshold.
inline void bernoulli(int P, uint64_t seed, int64_t iter, uint32_t threshold, uint64_t* words)
{
    clear(P, words);
    const uint64_t iter_key = mix64(seed + ((uint64_t)iter + 1) * kIterStride);
    for (int rank = 0; rank < P; ++rank) {
        const uint64_t h = mix64(iter_key + ((uint64_t)rank + 1) * kRankStride);
        if ((uint32_t)(h >> 32) < threshold)
            set_bit(words, rank);
    }
}

// Exactly `count` distinct processes of P = 2^G, drawn one after another (Section 6.2 delays
// two randomly selected processes per step).
inline void stragglers(int P, int G, uint64_t seed, int64_t iter, int count, uint64_t* words)
{
    clear(P, words);
    const uint64_t iter_key = mix64((seed ^ kStragglerTag) + ((uint64_t)iter + 1) * kIterStride);
    int picked = 0;
    for (uint64_t draw = 1; picked < count; ++draw) {
        const uint64_t h = mix64(iter_key + draw * kRankStride);
        const int rank = G == 0 ? 0 : (int)(h >> (64 - G));
        if ((words[rank >> 6] >> (rank & 63)) & 1u)
            continue;  // already selected: draw again
        set_bit(words, rank);
        ++picked;
    }
}

// The step times, in ms, that the P processes draw in iteration iter: nine in sixteen take
// 1.7 s to 2 s, the others one of 16 geometric steps from 2 s to 43.5 s (the range and the
// median of the reinforcement-learning workload of Section 6.4).
inline void clock_step_times(uint64_t seed, int64_t iter, int P, uint32_t* ms)
{
    static const uint32_t kTailMs[16] = {2000, 2456, 3016, 3703, 4548, 5585, 6858, 8422,
                                         10342, 12700, 15595, 19151, 23517, 28879, 35463, 43500};
    const uint64_t iter_key = mix64((seed ^ kClockTag) + ((uint64_t)iter + 1) * kIterStride);
    for (int rank = 0; rank < P; ++rank) {
        const uint64_t h = mix64(iter_key + ((uint64_t)rank + 1) * kRankStride);
        const bool in_tail = (h >> 60) >= 9;  // seven steps in sixteen
        ms[rank] = in_tail ? kTailMs[(h >> 56) & 15] : kShortestStepMs + (uint32_t)((h >> 32) & 0xFF) * 300u / 256u;
    }
}

// All processes start together; the first to finish is the activator of Section 3.2 and never
// late, anybody more than tolerance_ms behind it is.  step_ms (may be null) gets the P times.
inline void clock(int P, uint64_t seed, int64_t iter, uint32_t tolerance_ms, uint64_t* words, uint32_t* step_ms)
{
    std::vector<uint32_t> ms((size_t)P);
    clock_step_times(seed, iter, P, ms.data());
    uint32_t first_done = UINT32_MAX;
    for (int rank = 0; rank < P; ++rank)
        if (ms[(size_t)rank] < first_done)
            first_done = ms[(size_t)rank];
    clear(P, words);
    for (int rank = 0; rank < P; ++rank) {
        if ((uint64_t)ms[(size_t)rank] > (uint64_t)first_done + tolerance_ms)
            set_bit(words, rank);
        if (step_ms)
            step_ms[rank] = ms[(size_t)rank];
    }
}

// Steps that span iterations (wagma_lag_masks).  Between two global iterations nobody waits
// (Section 3.2): every process runs its steps back to back; the first to end a step begun for
// a group allreduce activates it, the allreduce reads the models tolerance_ms later and those
// who arrived by then go on together from that moment.  Ending a step between two reads makes a
// process late in the earlier iteration; still computing at the next read makes it busy.
// The clocks restart after every global iteration (every `window` iterations when tau == 0).
// tolerance_ms must be below kShortestStepMs.  May throw std::bad_alloc.
inline void lag(int P, int tau, int window, uint64_t seed, int64_t iter, uint32_t tolerance_ms,
                uint64_t* late_words, uint64_t* busy_words)
{
    clear(P, late_words);
    clear(P, busy_words);
    if (is_global_iteration(tau, iter))
        return;  // everybody waits for the global average
    const int64_t length = tau > 0 ? tau : window;
    const int64_t first_iter = iter / length * length;
    const int64_t target = iter - first_iter;  // number of this iteration's allreduce since the restart

    // Time-ordered events.  A step's end is seen by a read that happens at the same time.
    struct Event {
        int64_t at;
        int is_read;    // 0: a process ends a step, 1: the running allreduce reads the models
        int rank;
        int64_t begun;  // the allreduce the step was begun for
        bool operator>(const Event& o) const
        {
            if (at != o.at)
                return at > o.at;
            if (is_read != o.is_read)
                return is_read > o.is_read;
            return rank > o.rank;
        }
    };
    std::priority_queue<Event, std::vector<Event>, std::greater<Event>> events;
    std::vector<int> waiting;                      // arrived at the running allreduce, not yet read
    std::vector<uint8_t> went_on((size_t)P, 0);    // ended a step since the target allreduce read
    // times[k & 1]: the step times drawn for steps begun for allreduce k
    std::vector<uint32_t> times[2] = {std::vector<uint32_t>((size_t)P), std::vector<uint32_t>((size_t)P)};
    clock_step_times(seed, first_iter, P, times[0].data());
    clock_step_times(seed, first_iter + 1, P, times[1].data());
    for (int rank = 0; rank < P; ++rank)
        events.push(Event{(int64_t)times[0][(size_t)rank], 0, rank, 0});
    int64_t running = 0;  // the allreduce that will read next
    while (true) {
        const Event ev = events.top();
        events.pop();
        if (ev.is_read && running == target + 1)
            break;  // whoever ended a step since the target read was late in it
        if (ev.is_read) {
            // those who arrived in time take the average and go on together
            for (int rank : waiting)
                events.push(Event{ev.at + (int64_t)times[(running + 1) & 1][(size_t)rank], 0, rank, running + 1});
            if (running == target) {
                // everybody else contributes a send buffer; who also ends a step before the
                // next read is late, the rest is still computing
                for (int rank = 0; rank < P; ++rank)
                    set_bit(busy_words, rank);
                for (int rank : waiting)
                    busy_words[rank >> 6] &= ~(UINT64_C(1) << (rank & 63));
            }
            waiting.clear();
            ++running;
            clock_step_times(seed, first_iter + running + 1, P, times[(running + 1) & 1].data());
        } else if (ev.begun == running) {
            if (waiting.empty())  // the activator
                events.push(Event{ev.at + (int64_t)tolerance_ms, 1, -1, running});
            waiting.push_back(ev.rank);
        } else {
            // the allreduce this step was begun for has read already: the process averages the
            // sum it finds with its W' and begins the next step at once
            events.push(Event{ev.at + (int64_t)times[running & 1][(size_t)ev.rank], 0, ev.rank, running});
            if (running == target + 1)
                went_on[(size_t)ev.rank] = 1;
        }
    }
    for (int rank = 0; rank < P; ++rank) {
        const uint64_t bit = UINT64_C(1) << (rank & 63);
        if (went_on[(size_t)rank] && (busy_words[rank >> 6] & bit)) {
            busy_words[rank >> 6] &= ~bit;
            late_words[rank >> 6] |= bit;
        }
    }
}

}  // namespace wagma_masks

#endif  // WAGMA_MASKS_H
