// Tuning aid, compiled in only with -DGLOWQ_TRACE (never in the product build): per
// workgroup and stage, a 100 MHz real-time counter value or a caller's value, kept in a
// per-translation-unit device array and fetched by the glowq_debug_trace* exports that
// GLOWQ_TRACE_EXPORT defines.  Without the flag every macro here expands to nothing.
#pragma once
#include <hip/hip_runtime.h>

#ifdef GLOWQ_TRACE
namespace glowq {
static __device__ unsigned long long g_trace[8192][8];   // one copy per translation unit
}
#define GLOWQ_TRACE_VALUE(slot, value)                                            \
  do {                                                                            \
    const unsigned b_ = blockIdx.x + blockIdx.y * gridDim.x;                      \
    if (threadIdx.x == 0 && b_ < 8192)                                            \
      glowq::g_trace[b_][slot] = (unsigned long long)(value);                     \
  } while (0)
#define GLOWQ_STAMP(slot) GLOWQ_TRACE_VALUE(slot, __builtin_amdgcn_s_memrealtime())
// hardware id of the compute unit this workgroup runs on (XCC_ID in the high word, HW_ID low)
#define GLOWQ_TRACE_HWID(slot)                                                                    \
  GLOWQ_TRACE_VALUE(slot, ((unsigned long long)__builtin_amdgcn_s_getreg((20 << 0) | (31 << 11)) << 32) | \
                              __builtin_amdgcn_s_getreg((4 << 0) | (31 << 11)))
#define GLOWQ_TRACE_EXPORT(name)                                                                  \
  extern "C" int name(unsigned long long* host_out /* [8192][8] */) {                             \
    return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(glowq::g_trace), sizeof(glowq::g_trace)); \
  }
#else
#define GLOWQ_TRACE_VALUE(slot, value) do { } while (0)
#define GLOWQ_STAMP(slot) do { } while (0)
#define GLOWQ_TRACE_HWID(slot) do { } while (0)
#define GLOWQ_TRACE_EXPORT(name)
#endif
