// Host-side helpers shared by the translation units of libintfa.so (not part of the C ABI).
#ifndef INTFA_INTERNAL_H
#define INTFA_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

// Stream set by ifa_set_stream(); the null stream until then.
hipStream_t ifa_current_stream();

static inline bool ifa_aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

#endif
