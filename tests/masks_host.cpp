// Runs the library's host-side lateness generators (csrc/wagma_masks.h, no HIP in them) on the
// CPU and prints their masks, one line per request, for tests/test_masks_host.py to compare
// with the oracle.  Requests on stdin, one per line:
//   bernoulli P seed iter threshold
//   stragglers P seed iter count
//   clock P seed iter tolerance          (prints the mask words, then the P step times)
//   lag P tau window seed iter tolerance (prints the late words, then the busy words)
//   global tau iter
#include <cinttypes>
#include <cstdio>
#include <cstring>
#include <vector>

#include "wagma_masks.h"

static int log2_of(int P)
{
    int G = 0;
    while ((1 << G) < P)
        ++G;
    return G;
}

int main()
{
    char kind[32];
    while (std::scanf("%31s", kind) == 1) {
        if (!std::strcmp(kind, "global")) {
            int tau;
            int64_t iter;
            if (std::scanf("%d %" SCNd64, &tau, &iter) != 2)
                return 2;
            std::printf("%d\n", wagma_masks::is_global_iteration(tau, iter) ? 1 : 0);
            continue;
        }
        int P, tau = 0, window = 0;
        uint64_t seed, arg;
        int64_t iter;
        if (!std::strcmp(kind, "lag")) {
            if (std::scanf("%d %d %d %" SCNu64 " %" SCNd64 " %" SCNu64, &P, &tau, &window, &seed, &iter, &arg) != 6)
                return 2;
        } else if (std::scanf("%d %" SCNu64 " %" SCNd64 " %" SCNu64, &P, &seed, &iter, &arg) != 4) {
            return 2;
        }
        const int words = (P + 63) / 64;
        std::vector<uint64_t> a((size_t)words, ~UINT64_C(0)), b((size_t)words, ~UINT64_C(0));
        std::vector<uint32_t> ms((size_t)P);
        if (!std::strcmp(kind, "bernoulli"))
            wagma_masks::bernoulli(P, seed, iter, (uint32_t)arg, a.data());
        else if (!std::strcmp(kind, "stragglers") && arg > (uint64_t)P)
            return 2;  // the library refuses such a count before it gets here
        else if (!std::strcmp(kind, "stragglers"))
            wagma_masks::stragglers(P, log2_of(P), seed, iter, (int)arg, a.data());
        else if (!std::strcmp(kind, "clock"))
            wagma_masks::clock(P, seed, iter, (uint32_t)arg, a.data(), ms.data());
        else if (!std::strcmp(kind, "lag"))
            wagma_masks::lag(P, tau, window, seed, iter, (uint32_t)arg, a.data(), b.data());
        else
            return 2;
        for (int k = 0; k < words; ++k)
            std::printf("%" PRIu64 " ", a[(size_t)k]);
        if (!std::strcmp(kind, "lag"))
            for (int k = 0; k < words; ++k)
                std::printf("%" PRIu64 " ", b[(size_t)k]);
        if (!std::strcmp(kind, "clock"))
            for (int p = 0; p < P; ++p)
                std::printf("%u ", ms[(size_t)p]);
        std::printf("\n");
    }
    return 0;
}
