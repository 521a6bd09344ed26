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
  size_t off_counters;  // T > 32: per token tile, a ready flag and an arrival counter of K parts
  size_t off_rpart;   // partial sums of the projection (T <= 32: 8-byte slots {fp32, launch tag},
                      // [T][ksplit][r]; T > 32 and glowq_shared_proj: fp32 [part][T][r])
  size_t off_r16;     // T > 32: R in the activation type, [T][r]
  size_t off_splitk;  // T > 64: fp32 slabs of a long contraction cut into K slices (0 bytes if not cut)
  size_t splitk_bytes;
  size_t ctl_bytes;   // leading bytes that must be zero between calls
  int ksplit;         // K slices of the projection
  int kslice;         // channels per slice (multiple of 32)
  int kstride;        // ksplit rounded up to a multiple of 4 (sizes the partial-sum area)
  int pf_parts;       // T > 32: K parts of a projection tile inside the GEMM launch
  int pf_part_stages; // 64-channel stages per such part
};

// decode path = one pass over the weights with all tokens in one matrix-core tile
static inline bool is_decode(int T) { return T <= 32; }

UnitWorkspace plan_unit_workspace(const glowq_unit& u, char* base);

hipError_t launch_prepare(const uint32_t* wq, const uint16_t* scales, const uint16_t* zeros,
                          int d_out, int d_in, int G, void* prepared, hipStream_t st);
hipError_t launch_quantize_rtn(const float* W, int d_out, int d_in, int G, uint32_t* wq, uint16_t* scales,
                               uint16_t* zeros, hipStream_t st);
hipError_t launch_debug_unpack(const void* prepared, int d_out, int d_in, int G, uint8_t* q_out,
                               hipStream_t st);
hipError_t launch_debug_dequant(const void* prepared, int d_out, int d_in, int G, int act,
                                void* w_out, hipStream_t st);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st);
hipError_t launch_importance(const glowq_unit& u, const float* const* W_modules, double* scratch,
                             double* scores, hipStream_t st);
// Workspace of the factorisation of one unit's stacked error (byte offsets, 256-aligned).
struct FactorizePlan {
  long long m;        // rows of the stack
  int d, l, l16, r16; // channels; sketch width r + p; both widths rounded up to 16
  int n_groups, rpw;  // row groups of the orthonormalisation and rows per group
  size_t off_ms, off_y, off_z, off_bs, off_ut, off_gram, off_lift, off_a64, off_slices, off_root,
      off_inv_root, off_c1, off_c2, off_norm, off_norm0, off_sig2, off_sigma, off_perm,
      off_counters;
  size_t bytes;
};
FactorizePlan plan_factorize(const glowq_unit& u, int r, int p);
hipError_t launch_factorize(const glowq_unit& u, const float* const* W_modules, const double* sigma_x,
                            int r, int p, int q, const double* Omega, char* ws, void* const* A_out,
                            void* B_out, double* sigma_out, hipStream_t st);
// Microscaling variant (MXFP4 weights, MXFP8 activations), up to 16 tokens.
struct MxWorkspace {
  size_t off_rpart;         // fp32 partial sums of the projection, [ks][16][r]
  size_t off_xcodes;        // E4M3 codes of the activations in fragment order, whole 16-token blocks
  size_t off_xscales;       // their E8M0 block scales, likewise
  size_t bytes;
  int ks, kslice;           // K slices of the projection and channels per slice
};
constexpr int MX_MAX_TOKENS = 16;
size_t mx_prepared_bytes(int d_out, int d_in);
MxWorkspace plan_mx_workspace(const glowq_unit& u);
hipError_t launch_mx_prepare(const uint32_t* codes, const uint8_t* scales, int d_out, int d_in, void* prepared,
                             hipStream_t st);
hipError_t launch_mx_quantize_x(const void* X, int T, int d_in, int act, uint8_t* codes, uint8_t* scales,
                                bool fragment_order, hipStream_t st);
hipError_t launch_mx_forward(const glowq_unit& u, bool restore, char* workspace, hipStream_t st);
// slices' start offsets in units of 256 bytes (every slice is 256-byte aligned)
constexpr int STATUS_BATCH = 256;
struct StatusBatch {
  uint32_t off256[STATUS_BATCH];
  int n;
};
hipError_t launch_status_count(const void* ws, const StatusBatch& b, bool first, uint32_t* out,
                               hipStream_t st);

struct ProjArgs;
ProjArgs make_proj_args(const glowq_unit& u, const UnitWorkspace& ws, float* R32, bool want_r16);

// R = X B^T, stand-alone: fp32 partial sums per K slice, then a second launch adds them in
// slice order into R32 (optional) and R16 (optional).
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
                                const bool* restore, int n_units, bool allow_split, hipStream_t st);
int prefill_k_slices(const glowq_unit& u);
size_t prefill_splitk_bytes(const glowq_unit& u);

}  // namespace glowq
