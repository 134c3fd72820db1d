// Host-side check of the chunked kernel's window bookkeeping (csrc/wkv6_windows.h): for every
// (units per workgroup, chunks per unit, producer group) of a grid, the producers' and the consumers'
// control flows execute the same number of workgroup barriers, and the three producer groups
// together start exactly one cycle for every chunk position (and a few drain cycles after the end).
#include <cstdio>
#include <vector>

#include "../../paper_2407_12077_amd/csrc/wkv6_windows.h"

int main() {
    long long cases = 0;
    for (int count = 1; count <= 40; ++count) {
        for (int nchunks = 1; nchunks <= 70; ++nchunks) {
            const int total = count * nchunks;
            const int nwin = wkv6::window_count(total);
            if (nwin % 3 != 0 || nwin < total + 4 || nwin > total + 6) {
                std::printf("FAIL window_count(%d) = %d\n", total, nwin);
                return 1;
            }
            const int want = wkv6::consumer_barriers(total);
            std::vector<int> seen(static_cast<size_t>(nwin) + 8, 0);
            for (int pg = 0; pg < wkv6::kWindowGroups; ++pg) {
                const wkv6::ProducerWalk w = wkv6::producer_walk(total, pg);
                if (w.barriers != want) {
                    std::printf("FAIL count=%d nchunks=%d pg=%d: producers %d barriers, consumers %d\n", count, nchunks,
                                pg, w.barriers, want);
                    return 1;
                }
                for (int c = 0, g = pg; c < w.cycles; ++c, g += 3) ++seen[static_cast<size_t>(g)];
                if (w.cycles > 0 && (w.first != pg || w.last != pg + 3 * (w.cycles - 1))) {
                    std::printf("FAIL cycle positions count=%d nchunks=%d pg=%d\n", count, nchunks, pg);
                    return 1;
                }
            }
            // every chunk position digested once; the stores of the last chunk leave in the score phase of
            // position total + 1, so cycles must exist up to there
            for (int g = 0; g < total + 2; ++g)
                if (seen[static_cast<size_t>(g)] != 1) {
                    std::printf("FAIL chunk position %d visited %d times (count=%d nchunks=%d)\n", g,
                                seen[static_cast<size_t>(g)], count, nchunks);
                    return 1;
                }
            ++cases;
        }
    }
    // a few very long sequences
    for (int total : {4096, 4097, 4098, 131072 / 32, 1000003}) {
        for (int pg = 0; pg < 3; ++pg)
            if (wkv6::producer_barriers(total, pg) != wkv6::consumer_barriers(total)) {
                std::printf("FAIL total=%d pg=%d\n", total, pg);
                return 1;
            }
        ++cases;
    }
    std::printf("ok %lld cases\n", cases);
    return 0;
}
