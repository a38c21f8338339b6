// Error reporting of liblagom: one text buffer per thread, static names per code.
#include <cstdio>
#include "common.h"

namespace lagom {
static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    std::vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}
}  // namespace lagom

extern "C" const char* lagom_strerror(int code) {
    switch (code) {
        case LAGOM_OK: return "ok";
        case LAGOM_EINVAL: return "invalid argument";
        case LAGOM_EALIGN: return "device pointer not 16-byte aligned";
        case LAGOM_EHIP: return "HIP runtime error";
        case LAGOM_ECALLBACK: return "profile callback failed";
        default: return "unknown error code";
    }
}

extern "C" const char* lagom_last_error(void) { return lagom::g_err; }
