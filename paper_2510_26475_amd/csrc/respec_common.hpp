// Shared host-side plumbing of librespec: status text, error slot, argument checks.
// Device code lives in the .hip files; nothing here is used by the CPU oracle.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "respec.h"

namespace respec {

// Thread-local text of the last failure; returns `status` so callers can `return fail(...)`.
respec_status_t fail(respec_status_t status, const char *fmt, ...);
void clear_error();

inline bool aligned_to(const void *p, size_t a) {
    return (reinterpret_cast<uintptr_t>(p) % a) == 0;
}

inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Integer environment knob (tuning sweeps); returns `fallback` when unset or malformed.
long env_long(const char *name, long fallback);

}  // namespace respec
