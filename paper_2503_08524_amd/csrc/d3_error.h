// Thread-local error message behind d3_last_error().
#pragma once
#include <cstdarg>
#include <cstdio>

namespace d3 {

inline char* error_buffer() {
    static thread_local char buf[512] = "";
    return buf;
}

// Records the message and returns `status`, so call sites read `return fail(...)`.
inline int fail(int status, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
inline int fail(int status, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(error_buffer(), 512, fmt, ap);
    va_end(ap);
    return status;
}

}  // namespace d3
