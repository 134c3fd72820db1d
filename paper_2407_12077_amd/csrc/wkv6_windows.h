// Window bookkeeping of the chunked kernel, shared by the producer and consumer code paths and by a
// host-side check.  A workgroup walks its chunk sequence (all chunks of all its units, `total` of
// them) in windows separated by one workgroup barrier each.  Every wave of the workgroup must
// execute the same number of barriers, whatever its role; the producer groups and the consumers
// reach theirs from differently shaped loops, so the loop conditions live here, and
// producer_barriers() / consumer_barriers() replay them on the host for any (total, group).
#pragma once

#if defined(__HIPCC__)
#define WKV6_HD __host__ __device__
#else
#define WKV6_HD
#endif

namespace wkv6 {

constexpr int kWindowGroups = 3;        // producer groups; group pg owns the chunks g = pg (mod 3)

// Windows a workgroup runs for `total` chunks: chunk g is digested in window g, its tiles are
// written in g + 1, its scores in g + 2, the state chain runs in g + 2 and its output rows leave in
// window g + 4 (the score phase of chunk g + 2); rounded up to whole cycles of three.
WKV6_HD inline int window_count(int total) { return (total + 6) / 3 * 3; }

// A producer group at window g (g = pg (mod 3)) still has two / one full three-window cycle to run.
WKV6_HD inline bool has_cycle_pair(int g, int nwin) { return g + 5 < nwin; }
WKV6_HD inline bool has_cycle(int g, int nwin) { return g + 2 < nwin; }

struct ProducerWalk {
    int barriers;        // barriers executed, the start barrier included
    int cycles;          // three-window cycles executed
    int first, last;     // first and last chunk position a cycle was started for (-1: none)
};

// The producer group's control flow with every barrier counted: the start barrier, `pg` idle
// windows, cycles two at a time, at most one more cycle, idle windows up to the end.
inline ProducerWalk producer_walk(int total, int pg) {
    const int nwin = window_count(total);
    ProducerWalk w = {1, 0, -1, -1};
    int done = 0;
    for (; done < pg; ++done) ++w.barriers;
    int g = pg;
    auto cycle = [&](int at) {
        w.barriers += 3;
        ++w.cycles;
        if (w.first < 0) w.first = at;
        w.last = at;
    };
    for (; has_cycle_pair(g, nwin); g += 6) {
        cycle(g);
        cycle(g + 3);
        done += 6;
    }
    if (has_cycle(g, nwin)) {
        cycle(g);
        done += 3;
    }
    for (; done < nwin; ++done) ++w.barriers;
    return w;
}

inline int producer_barriers(int total, int pg) { return producer_walk(total, pg).barriers; }

// The consumers: the start barrier and one barrier per window.
inline int consumer_barriers(int total) { return 1 + window_count(total); }

}  // namespace wkv6
