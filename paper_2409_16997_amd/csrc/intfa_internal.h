// Host-side helpers shared by the translation units of libintfa.so (not part of the C ABI).
#ifndef INTFA_INTERNAL_H
#define INTFA_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

// Stream set by ifa_set_stream(); the null stream until then.
hipStream_t ifa_current_stream();

// The few-query kernel of intfa_attention_fewq.hip (one workgroup per head and 32 queries), for the dispatcher of the
// entry points in intfa_attention.hip; arguments already validated.
int ifa_launch_narrow(const int8_t *Q, const int8_t *K, const int8_t *V, const float *sQ, const float *sK, const float *sV, int heads,
                      int Nq, int Nk, int d, int causal, int vblock, void *O, int o_dtype, hipStream_t st);

static inline bool ifa_aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

#endif
