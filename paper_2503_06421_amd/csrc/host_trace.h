// Host-side timing for tuning builds of libtidal (-DTIDAL_TUNING_KNOBS): how long the calling thread
// spends in each kind of HIP call and at which offsets a call reaches its steps.  Switched on by the
// tuning knob TIDAL_TRACE_HOST; in the default build everything here is empty.
#ifndef TIDAL_HOST_TRACE_H_
#define TIDAL_HOST_TRACE_H_

#include <stddef.h>

#include "tidal_internal.h"

#ifdef TIDAL_TUNING_KNOBS
#include <stdio.h>
#include <string.h>

#include <chrono>

namespace tidal {

inline bool host_trace_on() { return tuning_knobs().trace_host == 1; }

struct HostCallStat { const char* what; double us; long n; };
inline HostCallStat* host_call_stats() {
    static HostCallStat stats[64];
    return stats;
}
inline int& host_call_count() {
    static int n = 0;
    return n;
}
inline void host_call_add(const char* what, double us) {
    size_t len = 0;
    while (what[len] && what[len] != '(') ++len;
    HostCallStat* st = host_call_stats();
    int& n = host_call_count();
    for (int i = 0; i < n; ++i)
        if (!strncmp(st[i].what, what, len) && (st[i].what[len] == '(' || st[i].what[len] == 0)) {
            st[i].us += us;
            st[i].n++;
            return;
        }
    if (n < 64) st[n++] = HostCallStat{what, us, 1};
}
// Print and reset the totals; every `every`-th call only (for entry points that run thousands of times).
inline void host_call_report(int every = 1) {
    static long calls = 0;
    if (!host_trace_on() || ++calls % every) return;
    HostCallStat* st = host_call_stats();
    int& n = host_call_count();
    for (int i = 0; i < n; ++i) {
        size_t len = 0;
        while (st[i].what[len] && st[i].what[len] != '(') ++len;
        fprintf(stderr, "[hostcalls] %-32.*s n=%5ld total %9.1f us\n", (int)len, st[i].what, st[i].n, st[i].us);
    }
    n = 0;
}
struct HostTrace {
    std::chrono::steady_clock::time_point origin = std::chrono::steady_clock::now();
    void mark(const char* what, size_t group) const {
        if (host_trace_on())
            fprintf(stderr, "[host] g%zu %-10s %8.1f us\n", group, what,
                    std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - origin).count());
    }
};

}  // namespace tidal

#define HIP_TIMED(expr)                                                                            \
    [&]() {                                                                                        \
        const auto t0_ = std::chrono::steady_clock::now();                                         \
        hipError_t r_ = (expr);                                                                    \
        ::tidal::host_call_add(#expr, std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - t0_).count()); \
        return r_;                                                                                 \
    }()

#else

namespace tidal {
inline bool host_trace_on() { return false; }
inline void host_call_report(int = 1) {}
struct HostTrace {
    void mark(const char*, size_t) const {}
};
}  // namespace tidal

#define HIP_TIMED(expr) (expr)

#endif
#endif
