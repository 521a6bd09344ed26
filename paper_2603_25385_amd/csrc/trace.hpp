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
#define GLOWQ_TRACE_VALUE_ANY(slot, value)                                        \
  do {                                                                            \
    const unsigned b_ = blockIdx.x + blockIdx.y * gridDim.x;                      \
    if (b_ < 8192) glowq::g_trace[b_][slot] = (unsigned long long)(value);        \
  } while (0)
#define GLOWQ_STAMP(slot) GLOWQ_TRACE_VALUE(slot, __builtin_amdgcn_s_memrealtime())
// the same from lane 0 of whichever wave gets there (the last one to do so stays)
#define GLOWQ_STAMP_WAVE(slot)                                                    \
  do {                                                                            \
    const unsigned b_ = blockIdx.x + blockIdx.y * gridDim.x;                      \
    if ((threadIdx.x & 63) == 0 && b_ < 8192)                                     \
      glowq::g_trace[b_][slot] = __builtin_amdgcn_s_memrealtime();                \
  } while (0)
// hardware id of the compute unit this workgroup runs on (XCC_ID in the high word, HW_ID low)
#define GLOWQ_TRACE_HWID(slot)                                                                    \
  GLOWQ_TRACE_VALUE(slot, ((unsigned long long)__builtin_amdgcn_s_getreg((20 << 0) | (31 << 11)) << 32) | \
                              __builtin_amdgcn_s_getreg((4 << 0) | (31 << 11)))
// per-wave stamps kept in registers and written out once, at the end (a store per stamp
// would join the wave's outstanding memory operations and be waited for with them)
namespace glowq {
static __device__ unsigned long long g_wtrace[2048][4][8];
}
#define GLOWQ_WTRACE_DECL unsigned long long glowq_wt_[8] = {0, 0, 0, 0, 0, 0, 0, 0}
#define GLOWQ_WSTAMP(slot) glowq_wt_[slot] = __builtin_amdgcn_s_memrealtime()
#define GLOWQ_WTRACE_HWID(slot)                                                                     \
  glowq_wt_[slot] = ((unsigned long long)__builtin_amdgcn_s_getreg((20 << 0) | (31 << 11)) << 32) | \
                    __builtin_amdgcn_s_getreg((4 << 0) | (31 << 11))
#define GLOWQ_WTRACE_FLUSH()                                                      \
  do {                                                                            \
    const unsigned b_ = blockIdx.x, w_ = threadIdx.x >> 6;                        \
    if ((threadIdx.x & 63) == 0 && b_ < 2048 && w_ < 4)                           \
      for (int i_ = 0; i_ < 8; ++i_) glowq::g_wtrace[b_][w_][i_] = glowq_wt_[i_]; \
  } while (0)
#define GLOWQ_WTRACE_EXPORT(name)                                                                 \
  extern "C" int name(unsigned long long* host_out /* [2048][4][8] */) {                          \
    return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(glowq::g_wtrace), sizeof(glowq::g_wtrace)); \
  }
#define GLOWQ_TRACE_EXPORT(name)                                                                  \
  extern "C" int name(unsigned long long* host_out /* [8192][8] */) {                             \
    return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(glowq::g_trace), sizeof(glowq::g_trace)); \
  }
#else
#define GLOWQ_TRACE_VALUE(slot, value) do { } while (0)
#define GLOWQ_TRACE_VALUE_ANY(slot, value) do { } while (0)
#define GLOWQ_STAMP(slot) do { } while (0)
#define GLOWQ_STAMP_WAVE(slot) do { } while (0)
#define GLOWQ_TRACE_HWID(slot) do { } while (0)
#define GLOWQ_TRACE_EXPORT(name)
#define GLOWQ_WTRACE_DECL
#define GLOWQ_WSTAMP(slot) do { } while (0)
#define GLOWQ_WTRACE_HWID(slot) do { } while (0)
#define GLOWQ_WTRACE_FLUSH() do { } while (0)
#define GLOWQ_WTRACE_EXPORT(name)
#endif
