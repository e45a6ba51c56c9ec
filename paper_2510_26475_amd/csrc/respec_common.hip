// Host-side plumbing of librespec: status strings, thread-local error text, version.
#include "respec_common.hpp"

#include <cstdlib>
#include <cstring>

namespace respec {

namespace {
thread_local char g_last_error[512] = "";
}

respec_status_t fail(respec_status_t status, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_last_error, sizeof g_last_error, fmt, ap);
    va_end(ap);
    return status;
}

void clear_error() { g_last_error[0] = '\0'; }

long env_long(const char *name, long fallback) {
    const char *s = std::getenv(name);
    if (!s || !*s) return fallback;
    char *end = nullptr;
    const long v = std::strtol(s, &end, 10);
    return (end && *end == '\0') ? v : fallback;
}

}  // namespace respec

extern "C" {

const char *respec_status_string(respec_status_t status) {
    switch (status) {
        case RESPEC_OK: return "ok";
        case RESPEC_ERR_INVALID_ARG: return "invalid argument";
        case RESPEC_ERR_UNSUPPORTED: return "unsupported configuration";
        case RESPEC_ERR_WORKSPACE: return "workspace missing or too small";
        case RESPEC_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

const char *respec_last_error(void) { return respec::g_last_error; }

int respec_version(void) { return 100; /* 0.1.0 */ }

}  // extern "C"
