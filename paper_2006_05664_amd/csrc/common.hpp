// Shared host-side declarations of the OpEvo library (not part of the C ABI).
#pragma once

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <string>
#include <vector>

#include "opevo.h"

namespace opevo {

// Thread-local text behind opevo_last_error().
void set_error(const char *fmt, ...);
const char *last_error();

inline int fail(int status, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
inline int fail(int status, const char *fmt, ...)
{
    char buf[2048];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    set_error("%s", buf);
    return status;
}

// SplitMix64 (Steele, Lea & Flood 2014): the only generator the library draws from.
struct Rng {
    uint64_t state;
    explicit Rng(uint64_t seed) : state(seed) {}
    uint64_t next_u64()
    {
        state += 0x9E3779B97F4A7C15ull;
        uint64_t z = state;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    double next_double() { return double(next_u64() >> 11) * (1.0 / 9007199254740992.0); }
    uint32_t next_below(uint32_t n) { return uint32_t(((next_u64() >> 32) * uint64_t(n)) >> 32); }
};

}  // namespace opevo

struct opevo_rng {
    opevo::Rng rng;
    explicit opevo_rng(uint64_t seed) : rng(seed) {}
};
