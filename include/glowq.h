/* glowq.h -- C ABI of the GlowQ group forward for AMD MI355X (gfx950).
 *
 * The library computes, for one input-sharing group of a decoder block (q/k/v;
 * gate/up) or one solo module (o_proj, down_proj), the cache-and-reuse forward
 * of GlowQ (paper Sec. 3.3):
 *
 *     R    = X B^T                          once per group          (Eq. 8)
 *     Y_i  = X dequant(W_q,i)^T + R A_i^T   every module i          (Eq. 9)
 *     Y_i  = X dequant(W_q,i)^T             unit not restored (GlowQ-S gating)
 *
 * Memory is token-major and dense: X[T][d_in], B[r][d_in], A_i[d_out][r],
 * R[T][r], Y_i[T][ldy].  W_q,i is W4A16 storage (paper Sec. 4.1: INT4 weights,
 * group size G along d_in, 16-bit activations): q in [0,15], one binary16 scale
 * s and one integer-valued binary16 zero-point z per (row, group), and
 * dequant = round_to_act((q - z) * s) with a single rounding.
 *
 * Conventions for every entry point
 *  - Pointers marked DEVICE are HIP device pointers owned by the caller and
 *    must stay valid until the stream has executed the call; pointers marked
 *    HOST are read during the call only.  The library allocates nothing and
 *    keeps no state between calls.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls enqueue work and return; they never synchronise the device.
 *  - Every function returns a glowq_status; on any error nothing is enqueued.
 *    Argument checking is host-side and touches no GPU.
 *  - All DEVICE pointers must be 16-byte aligned.
 *
 * How this boundary differs from the plainest possible statement of the problem
 * ("packed INT4 words, a scale array and a zero-point array per module"), and why:
 *  - Weights are handed over ONCE, through glowq_prepare_weights, which rewrites
 *    the canonical arrays into tile records in matrix-core operand order with each
 *    tile's (s, z) pairs folded in behind its weights (one DRAM page per tile).  A
 *    glowq_module therefore carries the single pointer w_prepared instead of
 *    wq / scales / zeros, and the inspection hooks read that prepared buffer.
 *  - Every forward call, glowq_shared_proj included, takes a caller-owned workspace,
 *    and glowq_workspace_init must have cleared it once before its first use: the
 *    projection R is produced inside the forward launch and handed over through it.
 *  - d_in must be a multiple of the 128-channel tile (not merely of the group size)
 *    and d_out, ldy multiples of 8; r a multiple of 8 up to GLOWQ_MAX_RANK.  A request
 *    that is well formed but outside these limits gets GLOWQ_ERR_UNSUPPORTED; sizes
 *    that contradict the storage format itself get GLOWQ_ERR_SHAPE.
 *  - binary16 activations with T <= 32: the kernels multiply X with the exact integers
 *    (q - z) and apply s to the fp32 sum of each quantisation group, i.e. they use
 *    (q - z) * s unrounded instead of its binary16 rounding (at most 2^-11 relative
 *    per term closer to the real weight).  Every other path multiplies with
 *    round_to_act((q - z) * s) bit for bit.
 */
#ifndef GLOWQ_H
#define GLOWQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GLOWQ_MAX_MODULES 8   /* modules per unit                               */
#define GLOWQ_MAX_RANK 128    /* r in {0} u {8k : k >= 1, 8k <= 128}           */

typedef enum {
  GLOWQ_OK = 0,
  GLOWQ_ERR_NULL = -1,        /* a required pointer is NULL                     */
  GLOWQ_ERR_SHAPE = -2,       /* a size is out of range or contradicts the
                                 storage format (d_in not a whole number of
                                 groups, group size not 64 / 128, T < 1, ...)   */
  GLOWQ_ERR_ALIGN = -3,       /* a device pointer or stride is misaligned       */
  GLOWQ_ERR_DTYPE = -4,       /* unsupported activation / output type           */
  GLOWQ_ERR_UNSUPPORTED = -5, /* well-formed request this build cannot serve:
                                 d_in not a multiple of 128, d_out or ldy not a
                                 multiple of 8, r not a multiple of 8 or > 128  */
  GLOWQ_ERR_WORKSPACE = -6,   /* workspace missing or too small                 */
  GLOWQ_ERR_HIP = -7          /* a HIP runtime call failed                      */
} glowq_status;

typedef enum { GLOWQ_F16 = 0, GLOWQ_BF16 = 1, GLOWQ_F32 = 2 } glowq_dtype;

/* One module (one linear map W_i of a unit). */
typedef struct {
  const void* w_prepared; /* DEVICE: output of glowq_prepare_weights for this module      */
  const void* A;          /* DEVICE: act dtype [d_out][r]; may be NULL if r == 0 or the
                             unit is not restored in this call                             */
  void* Y;                /* DEVICE: out dtype [T][ldy]                                    */
  int32_t d_out;          /* rows of W_i; multiple of 8                                    */
  int32_t ldy;            /* row stride of Y in elements; >= d_out, multiple of 8          */
} glowq_module;

/* One unit of the restore policy (Sec. 3.3): an input-sharing group
 * (n_modules > 1) or a solo module (n_modules == 1). */
typedef struct {
  const void* X;               /* DEVICE: act dtype [T][d_in]                              */
  const void* B;               /* DEVICE: act dtype [r][d_in], shared by all modules;
                                  may be NULL if r == 0 or the unit is not restored         */
  const glowq_module* modules; /* HOST: n_modules descriptors                               */
  int32_t n_modules;           /* 1 .. GLOWQ_MAX_MODULES                                    */
  int32_t T;                   /* tokens (batch x time flattened), >= 1                     */
  int32_t d_in;                /* shared input width; multiple of 128                       */
  int32_t r;                   /* rank of the correction; 0 or a multiple of 8, <= 128      */
  int32_t group_size;          /* G: 64 or 128                                              */
  int32_t act_dtype;           /* GLOWQ_F16 or GLOWQ_BF16: type of X, B, A and of the
                                  dequantised weight                                        */
  int32_t out_dtype;           /* act_dtype or GLOWQ_F32: type of Y                         */
} glowq_unit;

/* Human-readable name of a status code (static string). */
const char* glowq_status_string(glowq_status s);

/* Text of the HIP error behind the calling thread's most recent GLOWQ_ERR_HIP
 * ("no error" if there was none).  Static string owned by the HIP runtime. */
const char* glowq_last_hip_error(void);

/* Argument check of one unit exactly as the forward calls perform it for a
 * restored unit (HOST only, no GPU access).  check_pointers == 0 skips the NULL /
 * alignment tests so that shapes can be validated before buffers exist. */
glowq_status glowq_validate_unit(const glowq_unit* u, int32_t check_pointers);

/* ---- weight preparation (one-off, at load time) --------------------------
 * The kernels read weights from tile records of 16 rows x 128 input channels: one
 * contiguous 1 KiB wave load in which every lane's four words are already in
 * matrix-core operand order, followed by the tile's (s, z) pairs.  d_in must be a
 * multiple of 128, d_out a multiple of 8.
 * glowq_prepared_bytes gives the size of that buffer,
 * glowq_prepare_weights fills it from the canonical W4A16 arrays:
 *   wq      DEVICE uint32 [d_out][d_in/8], element 8j+e of a row in bits 4e..4e+3 of word j
 *   scales  DEVICE binary16 [d_out][d_in/G]
 *   zeros   DEVICE binary16 [d_out][d_in/G], integers in [0, 15]
 * Zero-points outside that set give unspecified values (never a fault). */
glowq_status glowq_prepared_bytes(int32_t d_out, int32_t d_in, int32_t group_size,
                                  size_t* bytes);
glowq_status glowq_prepare_weights(const uint32_t* wq, const uint16_t* scales,
                                   const uint16_t* zeros, int32_t d_out, int32_t d_in,
                                   int32_t group_size, void* w_prepared, void* stream);

/* ---- workspace ------------------------------------------------------------
 * Scratch for a call over `n_units` units (R in 16 bit, partial sums of the
 * projection, a few control and flag words).  glowq_workspace_init clears it; it must
 * be called once before the first forward call that uses the buffer.  After that one
 * buffer can serve any number of consecutive calls on one stream, eager or replayed
 * from a captured graph: a launch recognises its own projection by a tag that is
 * unique per kernel launch, so nothing in the buffer ever has to be reset.  Calls
 * that may overlap in time need separate workspaces.
 *
 * A unit of more than 64 tokens whose contraction is long (d_in >= 8192) on few tiles
 * (at most 128 tiles of 128 tokens x 256 rows, 192 rows for bfloat16) is multiplied in two
 * to four slices of K, so that its few workgroups do not each run the whole contraction
 * while the chip idles: every slice leaves an fp32 partial result in the unit's slice of
 * the workspace ([slice][T][d_out rounded up to 4] per module, counted by
 * glowq_workspace_bytes), and a second kernel adds them in slice order and writes Y.  The
 * rule reads T, d_in and the modules' d_out only: size the workspace from descriptors that
 * carry them (pointers may be NULL); a call whose workspace is smaller than what the unit's
 * shapes ask for is refused with GLOWQ_ERR_WORKSPACE.  Calls without a workspace
 * (no unit restored) and glowq_group_forward_static multiply such a unit in one piece.
 *
 * Unit i's slice starts at the sum of glowq_workspace_bytes of the units before it
 * (in the order of the forward call).  Word 3 of a slice (byte offset 12) is the
 * unit's status word: nonzero means that a bounded in-kernel wait for the projection
 * expired and the correction R A_i^T of that unit was LEFT OUT of Y (the output then
 * equals that of a unit that is not restored).  The producers of R lead their launch
 * and wait for nothing, so this happens only if workgroups of a launch are kept from
 * running; the bound is there so that nothing can ever hang.  Status words stay set
 * until glowq_workspace_init.  glowq_workspace_status counts them:
 * it enqueues one small kernel that writes to *failed_units (DEVICE, 4-byte aligned)
 * the number of the `n_units` units whose status word is nonzero; it allocates
 * nothing and does not synchronise (read the word after the stream has run). */
glowq_status glowq_workspace_bytes(const glowq_unit* units, int32_t n_units, size_t* bytes);
glowq_status glowq_workspace_init(void* workspace, size_t workspace_bytes, void* stream);
glowq_status glowq_workspace_status(const glowq_unit* units, int32_t n_units,
                                    const void* workspace, size_t workspace_bytes,
                                    uint32_t* failed_units, void* stream);

/* ---- the forward (Sec. 3.3) ------------------------------------------------
 * glowq_shared_proj: Eq. 8 alone.  R_out DEVICE fp32 [T][r] receives X B^T
 * (fp32 accumulation, K slices added in slice order).  Exists so that the cached
 * projection can be inspected; the group forward does not need it to be called
 * first (it computes R itself, inside its own launch for T <= 32).  r must be > 0. */
glowq_status glowq_shared_proj(const glowq_unit* u, float* R_out, void* workspace,
                               size_t workspace_bytes, void* stream);

/* glowq_group_forward: Eqs. 8-9 for one unit.  restore != 0: R is computed once
 * and every module adds R A_i^T.  restore == 0 (unit not selected by GlowQ-S) or
 * r == 0: Y_i = X dequant(W_q,i)^T and neither B nor any A_i is read. */
glowq_status glowq_group_forward(const glowq_unit* u, int32_t restore, void* workspace,
                                 size_t workspace_bytes, void* stream);

/* glowq_group_forward_static: glowq_group_forward for callers that cannot allocate
 * device memory or carry a workspace around (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc).  Same arguments without the
 * workspace: the scratch is a file-scope device array of GLOWQ_STATIC_SCRATCH_BYTES
 * inside the library, one per GPU, held until the process ends.  The call allocates
 * nothing (no hipMalloc / hipFree, no allocating library routine) and never
 * synchronises; a unit whose scratch need (glowq_workspace_bytes, less the partial
 * results of K slices, which this call does not use) exceeds the array is refused with
 * GLOWQ_ERR_WORKSPACE.  Every call on a GPU shares that GPU's array:
 * calls that may overlap in time on one GPU race (use glowq_group_forward with
 * separate workspaces for those), and the unit's status word is not observable.
 * Results are those of glowq_group_forward. */
#define GLOWQ_STATIC_SCRATCH_BYTES (16u << 20)
glowq_status glowq_group_forward_static(const glowq_unit* u, int32_t restore, void* stream);

/* glowq_block_forward: the same for `n_units` independent units (for example
 * the four units of one decoder block, or a whole stack), unit i restored iff
 * restore_mask[i] != 0 (HOST, one byte per unit; NULL = restore every unit).
 * No unit's Y may alias another unit's X within one call.  The glue between
 * the units of a real decoder block (attention, activation, norms, residual)
 * is not part of GlowQ and not part of this library. */
glowq_status glowq_block_forward(const glowq_unit* units, int32_t n_units,
                                 const uint8_t* restore_mask, void* workspace,
                                 size_t workspace_bytes, void* stream);

/* glowq_layerwise_forward: the comparison point of the latency study (Sec. 4.3,
 * the table's "Layerwise" rows): nothing is shared.  Every module of every unit has
 * a right factor of its own, the projection is computed once PER MODULE,
 * R_i = X B_i^T, and Y_i = X dequant(W_q,i)^T + R_i A_i^T.  B_modules is a HOST array
 * with one DEVICE pointer per module, unit after unit in module order (the sum of the
 * units' n_modules entries; each [r][d_in], activation type, 16-byte aligned); the
 * units' own B is ignored.  The same kernels run: the call treats every module as a
 * unit of its own and forwards all of them as one block, so launches are shared as
 * in glowq_block_forward, and only the projections and the reads of B multiply.
 * Every unit needs r > 0; all units are corrected (no restore mask).  The workspace
 * holds one slice per module, in the same order, each as long as
 * glowq_workspace_bytes of that one-module unit: size it with
 * glowq_layerwise_workspace_bytes, zero it with glowq_workspace_init.  Status words:
 * word 3 of each slice, as described above. */
glowq_status glowq_layerwise_workspace_bytes(const glowq_unit* units, int32_t n_units,
                                             size_t* bytes);
glowq_status glowq_layerwise_forward(const glowq_unit* units, int32_t n_units,
                                     const void* const* B_modules, void* workspace,
                                     size_t workspace_bytes, void* stream);

/* ---- importance of a unit and the GlowQ-S selection (Sec. 3.3, Eqs. 10-11) ----
 * glowq_unit_importance: the two scores by which units are ranked for selective
 * restore, from the unit's full-precision weights, its prepared weights and its stored
 * factors (offline work, no part of the forward):
 *   scores[0] = g_ner = ||E_u||_F^2 / ||W_u||_F^2   (Eq. 11), E_u = W_u - dequant(W_q,u),
 *               the dequantised weight being the stored 16-bit value, all modules stacked;
 *   scores[1] = g_ec  = sum_{j<=r} sigma_j^2 / ||E_u||_F^2 (Eq. 10 with Sigma_x = I), the
 *               numerator read off the balanced factors as sum_j ||A[:,j]||^2 ||B[j,:]||^2
 *               (exact for factors that come from the stack's SVD, Eqs. A.1.9a-b, up to
 *               their 16-bit storage); 0 for r == 0.
 * W_modules: HOST array of u->n_modules DEVICE pointers, fp32 [d_out][d_in] each, 16-byte
 * aligned.  Of `u` the call reads modules[i].w_prepared / A / d_out, B, r, d_in,
 * group_size and act_dtype (X, Y, T are ignored).  scratch: DEVICE, 8-byte aligned,
 * GLOWQ_IMPORTANCE_SCRATCH_BYTES, any contents (cleared by the call).  scores: DEVICE
 * double[2].  All sums are float64; their order varies from run to run (atomic adds), so
 * results agree to rounding, not to the bit.
 * glowq_select_units: the restore mask of the k highest scores (HOST in, HOST out; among
 * equal scores the lower index first); mask[i] = 1 for selected units. */
#define GLOWQ_IMPORTANCE_SCRATCH_BYTES 4096
glowq_status glowq_unit_importance(const glowq_unit* u, const float* const* W_modules,
                                   void* scratch, double* scores, void* stream);
glowq_status glowq_select_units(const double* scores, int32_t n_units, int32_t k,
                                uint8_t* restore_mask);

/* ---- the quantiser (offline) ------------------------------------------------
 * glowq_quantize_rtn: round-to-nearest asymmetric INT4 of one module's full-precision
 * weights, per (row, group of group_size input channels) (Sec. 4.1: INT4 weights with
 * grouped scales; the paper fixes no more than that).  For each group: the range [lo, hi]
 * widened to contain 0; s = binary16(max((hi - lo) / 15, 2^-14)); z = clamp(rint(-lo / s),
 * 0, 15); q = clamp(rint(w / s) + z, 0, 15), rint to even, divisions in float64 on the
 * rounded s.  W: DEVICE fp32 [d_out][d_in].  Outputs are the canonical arrays that
 * glowq_prepare_weights takes: wq DEVICE uint32 [d_out][d_in/8], scales and zeros DEVICE
 * binary16 [d_out][d_in/G].  Same shape limits as glowq_prepare_weights. */
glowq_status glowq_quantize_rtn(const float* W, int32_t d_out, int32_t d_in, int32_t group_size,
                                uint32_t* wq, uint16_t* scales, uint16_t* zeros, void* stream);

/* ---- the shared factors of a unit, computed on the GPU (offline) ------------
 * glowq_factorize_unit: balanced rank-r factors of the unit's stacked quantisation error
 * by the randomised, covariance-aligned procedure of Alg. 1 (App. A.3-A.4), from the
 * unit's full-precision weights and its prepared weights:
 *   E_cat = [W_i - dequant(W_q,i)]_i stacked by rows (m = sum of d_out rows),
 *   M     = E_cat diag(sigma_x)^(1/2)                      (sigma_x_diag NULL: identity),
 *   Y     = M Omega, then q times Y <- M (M^T Y);  Q = orth(Y);  Q^T M = U~ S V^T,
 *   A     = Q U~_r S_r^(1/2)  (rows split by module),  B = S_r^(1/2) V_r^T diag(sigma_x)^(-1/2)
 * (a zero variance gets a zero in the inverse root).  The products run on the stack itself
 * instead of on the triangular factor of its thin QR: with M_core = Q_e^T M every quantity
 * is the same or Q_e times the core's, so A and B are those of Alg. 1 up to rounding and up
 * to the sign of each rank (the pair (A[:,j], B[j,:]) may come out negated).
 * u: n_modules, modules[i].w_prepared / d_out, d_in, group_size and act_dtype are read
 * (X, Y, T, r, A, B are ignored).  r: the rank, a multiple of 8 up to GLOWQ_MAX_RANK and
 * at most m; p >= 0 the oversampling, r + p <= GLOWQ_MAX_SKETCH and <= d_in; q the power
 * steps, at most GLOWQ_MAX_POWER_STEPS.  W_modules: HOST array of n_modules DEVICE pointers, fp32
 * [d_out][d_in], 16-byte aligned.  sigma_x_diag: DEVICE double [d_in] or NULL.  Omega:
 * DEVICE double [d_in][r + p] row-major, the Gaussian test matrix, drawn by the caller.
 * workspace: DEVICE, 256-byte aligned, glowq_factorize_workspace_bytes(u, r, p) bytes, any
 * contents.  A_out: HOST array of n_modules DEVICE pointers, act dtype [d_out][r]; B_out:
 * DEVICE act dtype [r][d_in]; both rounded to the activation type, ties to even, from
 * float64.  sigma_out: DEVICE double [r + p] or NULL, the singular values of Q^T M in
 * descending order (the first r are those of the factors: |A[:,j]|^2 = |B[j,:]|^2 =
 * sigma_j for sigma_x = 1).  All arithmetic is float64 with sums in a fixed order: the
 * same inputs give the same bits.  The call enqueues a few thousand small launches on
 * `stream` and returns; it allocates nothing. */
#define GLOWQ_MAX_SKETCH 256
#define GLOWQ_MAX_POWER_STEPS 8
glowq_status glowq_factorize_workspace_bytes(const glowq_unit* u, int32_t r, int32_t p,
                                             size_t* bytes);
glowq_status glowq_factorize_unit(const glowq_unit* u, const float* const* W_modules,
                                  const double* sigma_x_diag, int32_t r, int32_t p, int32_t q,
                                  const double* Omega, void* workspace, size_t workspace_bytes,
                                  void* const* A_out, void* B_out, double* sigma_out,
                                  void* stream);

/* ---- microscaling variant: MXFP4 weights, MXFP8 activations (W4A8) ------------
 * The same forward (Sec. 3.3, Eqs. 8-9) on the floating-point-like datatypes of the paper's
 * datatype appendix and the W4A8 rows of its main results:
 *   Y_i = Xq dequant(W_mx,i)^T + R A_i^T,   R = X B^T,
 * Xq the activations quantised to MXFP8 (E4M3) inside the call, W_mx,i MXFP4 (E2M1) weights,
 * the correction from the 16-bit X, B and A_i exactly as in the W4A16 calls.  Formats of the
 * OCP Microscaling (MX) v1.0 specification: blocks of 32 consecutive input channels share an
 * E8M0 scale 2^(code - 127); conversion: shared exponent floor(log2(max |v|)) - emax (2 for
 * E2M1, 8 for E4M3) clamped to [-127, 127], elements rounded to nearest even and clamped to
 * the largest finite value; a block of zeros gets code 127.  The main product runs on the
 * block-scaled matrix instruction, fp32 accumulation.
 * glowq_mx_prepare_weights: codes DEVICE uint32 [d_out][d_in/8], element 8j+e of a row in
 *   bits 4e..4e+3 of word j (E2M1 code, sign in bit 3); scales DEVICE uint8 [d_out][d_in/32];
 *   w_prepared DEVICE, glowq_mx_prepared_bytes(d_out, d_in) bytes.  d_in a multiple of 128,
 *   d_out a multiple of 8 (else GLOWQ_ERR_UNSUPPORTED).
 * glowq_mx_quantize_activations: the activation quantiser by itself; X DEVICE act dtype
 *   [T][d_in]; codes DEVICE uint8 [T][d_in] (E4M3), scales DEVICE uint8 [T][d_in/32].
 * glowq_mx_group_forward: `u` as for glowq_group_forward with modules[i].w_prepared from
 *   glowq_mx_prepare_weights (group_size is ignored); workspace DEVICE, 256-byte aligned,
 *   glowq_mx_workspace_bytes(u) bytes (it depends on T), any contents.  Up to 4 tokens (and
 *   T d_in <= 16384, d_in <= 12288): ONE launch on `stream`; the projection's workgroups lead
 *   the grid and hand R over inside the launch, every hand-off validated by a tag of the
 *   launch (nothing to reset, graph replays included), every wait bounded; should a wait ever
 *   expire, the rows concerned are stored as NaN rather than without their correction.  Up to
 *   16 tokens otherwise: two launches (activation quantiser and projection; the weight
 *   stream).  More tokens: the activation quantiser, the stand-alone projection when restored,
 *   and a tiled product (128 tokens x 128 rows per workgroup).  Calls that share a workspace
 *   must not overlap. */
glowq_status glowq_mx_prepared_bytes(int32_t d_out, int32_t d_in, size_t* bytes);
glowq_status glowq_mx_prepare_weights(const uint32_t* codes, const uint8_t* scales, int32_t d_out,
                                      int32_t d_in, void* w_prepared, void* stream);
glowq_status glowq_mx_quantize_activations(const void* X, int32_t T, int32_t d_in, int32_t act_dtype,
                                           uint8_t* codes, uint8_t* scales, void* stream);
glowq_status glowq_mx_workspace_bytes(const glowq_unit* u, size_t* bytes);
glowq_status glowq_mx_group_forward(const glowq_unit* u, int32_t restore, void* workspace,
                                    size_t workspace_bytes, void* stream);

/* ---- inspection hooks (bit-exactness checks of the storage format) ---------
 * Both read the prepared layout of one module (the buffer the forward kernels
 * stream) with small kernels of their own.
 * glowq_debug_unpack:  q_out DEVICE uint8 [d_out][d_in], values 0..15.
 * glowq_debug_dequant: w_out DEVICE act dtype [d_out][d_in],
 *                      round_to_act((q - z) * s), one rounding, formed by the
 *                      reference dequantiser of the library.  The forward kernels
 *                      use instruction sequences of their own; what THEY multiply
 *                      with can be read through a forward call whose X is rows of
 *                      the identity and r = 0. */
glowq_status glowq_debug_unpack(const void* w_prepared, int32_t d_out, int32_t d_in,
                                int32_t group_size, uint8_t* q_out, void* stream);
glowq_status glowq_debug_dequant(const void* w_prepared, int32_t d_out, int32_t d_in,
                                 int32_t group_size, int32_t act_dtype, void* w_out,
                                 void* stream);

#ifdef __cplusplus
}
#endif
#endif /* GLOWQ_H */
