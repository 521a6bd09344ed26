// Host-side launch entry points implemented by the .hip files (internal).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/glowq.h"

namespace glowq {

// Layout of one unit's slice of the caller's workspace.
struct UnitWorkspace {
  char* base;         // start of the slice (256-byte aligned)
  size_t bytes;       // size of the slice
  size_t off_counters;  // uint32 per 32-token block of the projection
  size_t off_rpart;   // fp32 [T][r][ksplit rounded up to 4]
  size_t off_r16;     // act dtype [T][r]
  size_t ctl_bytes;   // leading bytes that must be zero between calls
  int ksplit;         // K slices of the projection
  int kslice;         // channels per slice (multiple of 32)
  int kstride;        // elements between the slice arrays of two outputs in the partial-sum area
  int pf_parts;       // T > 32: K parts of a projection tile inside the GEMM launch
  int pf_part_stages; // 64-channel stages per such part
};

// decode path = one pass over the weights with all tokens in one matrix-core tile
static inline bool is_decode(int T) { return T <= 32; }

UnitWorkspace plan_unit_workspace(const glowq_unit& u, char* base);

hipError_t launch_prepare(const uint32_t* wq, const uint16_t* scales, const uint16_t* zeros,
                          int d_out, int d_in, int G, void* prepared, hipStream_t st);
hipError_t launch_debug_unpack(const void* prepared, int d_out, int d_in, int G, uint8_t* q_out,
                               hipStream_t st);
hipError_t launch_debug_dequant(const void* prepared, int d_out, int d_in, int G, int act,
                                void* w_out, hipStream_t st);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st);

struct ProjArgs;
ProjArgs make_proj_args(const glowq_unit& u, const UnitWorkspace& ws, float* R32, bool want_r16);

// R = X B^T: fp32 partial sums per K slice, reduced by the last workgroup of each
// 32-token block into R32 (optional) and R16 (optional).
hipError_t launch_proj(const glowq_unit& u, const UnitWorkspace& ws, float* R32, bool want_r16,
                       hipStream_t st);
// T <= 32: streaming pass over the prepared weights; when restore, the projection runs
// in the first workgroups of the same launch
bool decode_batch_compatible(const glowq_unit& a, const glowq_unit& b);
int decode_max_batch();
hipError_t launch_decode_multi(const glowq_unit* const* units, const UnitWorkspace* ws,
                               const bool* restore, int n, hipStream_t st);
// T > 32: tiled matrix-core GEMM, correction folded in as an extra K slab.  One launch
// covers several compatible units (same types, group size and token-tile size).
bool prefill_compatible(const glowq_unit& a, const glowq_unit& b);
int prefill_max_units();
int prefill_max_modules();
hipError_t launch_prefill_multi(const glowq_unit* const* units, const UnitWorkspace* ws,
                                const bool* restore, int n_units, hipStream_t st);

}  // namespace glowq
