// Status reporting shared by the library's translation units: a negative code plus a thread-local message that
// nexus_last_error() returns.
#pragma once
#include <cstdarg>
#include <cstdio>

namespace nexus {

inline thread_local char g_err[512] = "";

inline int fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

}  // namespace nexus
