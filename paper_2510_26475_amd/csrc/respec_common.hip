// Host-side plumbing of librespec: status strings, thread-local error text, version.
#include "respec_common.hpp"

#include <cstdlib>
#include <cstring>
#include <mutex>

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

namespace {

long env_long(const char *name) {
    const char *s = std::getenv(name);
    if (!s || !*s) return Knobs::kUnset;
    char *end = nullptr;
    const long v = std::strtol(s, &end, 10);
    return (end && *end == '\0') ? v : Knobs::kUnset;
}

std::mutex g_knob_mutex;
bool g_knobs_read = false;
Knobs g_knobs;

void read_knobs_locked() {
    g_knobs.attn_wgs = env_long("RESPEC_ATTN_WGS");
    g_knobs.attn_head_major = env_long("RESPEC_ATTN_HEAD_MAJOR");
    g_knobs.attn_wide = env_long("RESPEC_ATTN_WIDE");
    g_knobs.attn_quad = env_long("RESPEC_ATTN_QUAD");
    g_knobs.attn_inline = env_long("RESPEC_ATTN_INLINE");
    g_knobs.sampler_split = env_long("RESPEC_SAMPLER_SPLIT");
    g_knobs.sampler_two_term = env_long("RESPEC_SAMPLER_TWO_TERM");
    g_knobs.sampler_guarded = env_long("RESPEC_SAMPLER_GUARDED");
    g_knobs.sampler_no_table = env_long("RESPEC_SAMPLER_NO_TABLE");
    g_knobs.sampler_two_items = env_long("RESPEC_SAMPLER_TWO_ITEMS");
    g_knobs.kd_wgs = env_long("RESPEC_KD_WGS");
    g_knobs_read = true;
}

}  // namespace

Knobs knobs() {
    std::lock_guard<std::mutex> lock(g_knob_mutex);
    if (!g_knobs_read) read_knobs_locked();
    return g_knobs;
}

void reload_knobs() {
    std::lock_guard<std::mutex> lock(g_knob_mutex);
    read_knobs_locked();
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

int respec_version(void) { return 200; /* 0.2.0 */ }

void respec_reload_knobs(void) { respec::reload_knobs(); }

}  // extern "C"
