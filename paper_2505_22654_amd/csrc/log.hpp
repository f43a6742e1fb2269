// Host-side debug log: with VSCAN_LOG=1 in the environment the library reports on stderr every
// error it returns (which check or HIP call failed, with the runtime's message) and every kernel
// it enqueues.  Read once per process; nothing is printed, and nothing on the device changes,
// when it is unset.
#pragma once
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>

namespace vscan {

inline bool log_on() {
    static const bool on = [] {
        const char *v = getenv("VSCAN_LOG");
        return v && v[0] && v[0] != '0';
    }();
    return on;
}

inline void logf(const char *fmt, ...) __attribute__((format(printf, 1, 2)));
inline void logf(const char *fmt, ...) {
    if (!log_on()) return;
    va_list ap;
    va_start(ap, fmt);
    fputs("[vscan] ", stderr);
    vfprintf(stderr, fmt, ap);
    fputc('\n', stderr);
    fflush(stderr);
    va_end(ap);
}

}  // namespace vscan
