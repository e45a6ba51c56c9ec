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

// Knobs for tests and tuning sweeps, from RESPEC_* environment variables.  The environment is
// read once, at the library's first call (and again on respec_reload_knobs()): no entry point
// calls getenv on its way to a launch.  A field holds kUnset when its variable is absent or
// malformed; the entry points then use their own defaults.
struct Knobs {
    static constexpr long kUnset = -0x7fffffffL;
    long attn_wgs;          // RESPEC_ATTN_WGS: ranges the attention's tile lists are split over
    long attn_head_major;   // RESPEC_ATTN_HEAD_MAJOR: one head-major tile list
    long attn_wide;         // RESPEC_ATTN_WIDE: 0/1 one or two consumer waves per range (2-4 column tiles)
    long attn_quad;         // RESPEC_ATTN_QUAD: 0/1/2 four consumers per range never / by rule / also narrow blocks
    long attn_inline;       // RESPEC_ATTN_INLINE: 0 = the set-up kernel also for small batches
    long sampler_split;     // RESPEC_SAMPLER_SPLIT: work-groups per sequence (1, 2, 4, 8)
    long sampler_two_term;  // RESPEC_SAMPLER_TWO_TERM: never the one-fma exponent
    long sampler_guarded;   // RESPEC_SAMPLER_GUARDED: the guarded normaliser pass everywhere
    long sampler_no_table;  // RESPEC_SAMPLER_NO_TABLE: the final draw without its table of slot totals
    long sampler_two_items; // RESPEC_SAMPLER_TWO_ITEMS: 0/1 shared sequences walk one or two chain items per stage
    long kd_wgs;            // RESPEC_KD_WGS: work-groups of the distillation kernel
    long get(long Knobs::*field, long fallback) const { return this->*field == kUnset ? fallback : this->*field; }
};
Knobs knobs();
void reload_knobs();

}  // namespace respec
