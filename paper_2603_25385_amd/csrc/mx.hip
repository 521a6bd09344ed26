// Microscaling variant of the group forward: MXFP4 weights and MXFP8
// activations in the main product, on the block-scaled matrix instruction of gfx950
// (v_mfma_scale_f32_16x16x128_f8f6f4), the 16-bit low-rank correction unchanged (paper
// Sec. 3.3, Eqs. 8-9, on the datatypes of the datatype appendix and the W4A8 rows of the
// main results; formats of the OCP MX v1.0 specification: blocks of 32 channels, E8M0
// scale, E2M1 / E4M3 elements).
//
// Operand layouts of the instruction (activations as A in fp8, weights as B in fp4),
// verified on the hardware:
//   A, fp8: lane l = token (l & 15), group g = l >> 4; register w, byte b holds channel
//           (w < 4 ? 0 : 64) + 16 g + 4 (w & 3) + b of the 128-channel tile
//   B, fp4: lane l = row (l & 15), group g; register w < 4, nibble n holds channel 32 g + 8 w + n
//   scales: the scale of (token or row i, 32-channel block kb) comes from lane i + 16 kb,
//           the byte of its scale register that the instruction's byte selector names
//   D:      lane l, register v holds (token 4 (l >> 4) + v, row l & 15)
// So a weight lane's four registers are 32 consecutive channels, exactly one MX block with
// its scale in the same lane, and a weight tile record is the canonical packed words of 16
// rows x 128 channels, lane after lane: no bit is touched between HBM and the matrix core.
//
// Weight storage (glowq_mx_prepare_weights): codes region [row block][tile][lane][4 words],
// then scales region [row block][tile][lane] bytes.  Rows past d_out: code 0, scale 127.
#include <algorithm>
#include "common.hpp"
#include "launch.hpp"
#include "proj_device.hpp"

namespace glowq {

typedef int v8i_t __attribute__((ext_vector_type(8)));

// ---------------------------------------------------------------------------------------
// preparation of the weights: one thread per word of the codes region / byte of the scales
// ---------------------------------------------------------------------------------------
__global__ void k_mx_prepare(const uint32_t* __restrict__ codes, const uint8_t* __restrict__ scales,
                             int d_out, int d_in, uint32_t* __restrict__ out_codes,
                             uint8_t* __restrict__ out_scales, long long n_words, long long n_scales) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const int ktiles = d_in / 128;
  if (idx < n_words) {
    const int w = (int)(idx & 3), lane = (int)((idx >> 2) & 63);
    const long long tile = idx >> 8;
    const int kt = (int)(tile % ktiles), rb = (int)(tile / ktiles);
    const int row = rb * 16 + (lane & 15);
    out_codes[idx] = row < d_out ? codes[(long long)row * (d_in / 8) + 16 * kt + 4 * (lane >> 4) + w] : 0u;
  }
  if (idx < n_scales) {
    const int lane = (int)(idx & 63);
    const long long tile = idx >> 6;
    const int kt = (int)(tile % ktiles), rb = (int)(tile / ktiles);
    const int row = rb * 16 + (lane & 15);
    out_scales[idx] = row < d_out ? scales[(long long)row * (d_in / 32) + 4 * kt + (lane >> 4)] : (uint8_t)127;
  }
}

// ---------------------------------------------------------------------------------------
// MXFP8 (E4M3) quantisation of the activations
// ---------------------------------------------------------------------------------------
// 16-bit pattern of the activation type as fp32 (exact)
template <int ACT>
__device__ inline float act16_f32(uint32_t h) {
  if constexpr (ACT == ACT_F16) return (float)__builtin_bit_cast(_Float16, (uint16_t)h);
  else return __builtin_bit_cast(float, h << 16);
}

// Sixteen consecutive channels of one token (lo, hi: their 16-bit patterns), half of an MX
// block; the other half is with the neighbouring lane (lane ^ 1), so both lanes of a pair
// must call this together.  Returns the sixteen E4M3 codes and the block's E8M0 scale code.
// Everything is exact but the one rounding to E4M3: the block maximum through the integer
// patterns of the magnitudes (they order as the values do), the values as fp32, the division
// by the power of two as a product, the clamp to +-448 (a scaled magnitude lies below 512),
// and the rounding itself by the conversion instruction (nearest even, subnormal codes kept,
// a zero keeps its sign bit, which the product ignores: the stored code of a zero is +0).
template <int ACT>
__device__ inline void mx_quantize16(const u32x4_t lo, const u32x4_t hi, u32x4_t& codes, int& scale_code) {
  typedef unsigned short u16x2_t __attribute__((ext_vector_type(2)));
  u16x2_t mm = {0, 0};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const u16x2_t a = __builtin_bit_cast(u16x2_t, lo[e] & 0x7fff7fffu), c = __builtin_bit_cast(u16x2_t, hi[e] & 0x7fff7fffu);
    mm = __builtin_elementwise_max(mm, __builtin_elementwise_max(a, c));
  }
  uint32_t m16 = max((uint32_t)mm[0], (uint32_t)mm[1]);
  m16 = max(m16, (uint32_t)__shfl_xor((int)m16, 1, 64));
  int shared = 0;
  if (m16 != 0u) {
    const uint32_t mmax = __builtin_bit_cast(uint32_t, act16_f32<ACT>(m16));
    const int ef = (int)(mmax >> 23);
    // floor(log2 max) - emax; a maximum below 2^-126 (bfloat16 only) has no exponent field
    const int fl = ef != 0 ? ef - 127 : (31 - __builtin_clz(mmax)) - 149;
    shared = max(-127, min(127, fl - 8));
  }
  const float inv = __builtin_bit_cast(float, (uint32_t)(127 - shared) << 23);        // 2^-shared
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const uint32_t w0 = q < 2 ? lo[2 * q] : hi[2 * q - 4], w1 = q < 2 ? lo[2 * q + 1] : hi[2 * q - 3];
    const float x0 = __builtin_amdgcn_fmed3f(act16_f32<ACT>(w0 & 0xffffu) * inv, -448.f, 448.f);
    const float x1 = __builtin_amdgcn_fmed3f(act16_f32<ACT>(w0 >> 16) * inv, -448.f, 448.f);
    const float x2 = __builtin_amdgcn_fmed3f(act16_f32<ACT>(w1 & 0xffffu) * inv, -448.f, 448.f);
    const float x3 = __builtin_amdgcn_fmed3f(act16_f32<ACT>(w1 >> 16) * inv, -448.f, 448.f);
    int word = __builtin_amdgcn_cvt_pk_fp8_f32(x0, x1, 0, false);
    word = __builtin_amdgcn_cvt_pk_fp8_f32(x2, x3, word, true);
    // -0 -> +0: a byte of 0x80 loses its sign
    const uint32_t u = (uint32_t)word;
    const uint32_t nz = (u & 0x7f7f7f7fu) + 0x7f7f7f7fu;          // bit 7 of a byte set iff its low seven bits are not zero
    codes[q] = u & (nz | 0x7f7f7f7fu);
  }
  scale_code = shared + 127;
}

// Two neighbouring lanes per (token, block of 32).  idx counts (token, 16-channel piece);
// every lane of a wave must call this (lanes past the end take part in the shuffle and
// store nothing).
// FRAG false: the canonical layouts, codes [T][d_in] and scales [T][d_in / 32].  FRAG true:
// fragment order, as the forward kernels read it -- per (16-token block, 128-channel tile)
// two 1 KiB chunks of codes [half][lane][16 bytes], lane = token + 16 g holding the channels
// 64 half + 16 g .. + 16 of its token (the fp8 operand of the matrix instruction as it
// stands, so that a wave's fetch is one contiguous KiB), and 64 scale bytes [lane], lane =
// token + 16 block.  Slots of tokens past T are not written.
template <int ACT, bool FRAG>
__device__ inline void mx_quantize_block(const uint16_t* __restrict__ X, int T, int d_in,
                                         uint8_t* __restrict__ codes, uint8_t* __restrict__ scales, long long idx) {
  const int pieces = d_in / 16;
  const bool live = idx < (long long)T * pieces;
  const long long it = live ? idx : 0;
  const int t = (int)(it / pieces), h = (int)(it - (long long)t * pieces);
  const u32x4_t* src = (const u32x4_t*)(X + (long long)t * d_in + 16 * h);
  u32x4_t c;
  int sc;
  mx_quantize16<ACT>(src[0], src[1], c, sc);
  if (!live) return;
  const int b = h >> 1;
  if (FRAG) {
    const int ktiles = d_in / 128, kt = b >> 2, kb = b & 3;
    const long long tile = (long long)(t >> 4) * ktiles + kt;
    const int g = 2 * (kb & 1) + (h & 1);                        // 16-channel piece within the half
    *(u32x4_t*)(codes + (tile * 2 + (kb >> 1)) * 1024 + ((t & 15) + 16 * g) * 16) = c;
    if (!(h & 1)) scales[tile * 64 + (t & 15) + 16 * kb] = (uint8_t)sc;
  } else {
    *(u32x4_t*)(codes + (long long)t * d_in + 16 * h) = c;
    if (!(h & 1)) scales[(long long)t * (d_in / 32) + b] = (uint8_t)sc;
  }
}

template <int ACT, bool FRAG>
__global__ void __launch_bounds__(256) k_mx_quantize_x(const uint16_t* __restrict__ X, int T, int d_in,
                                                       uint8_t* __restrict__ codes, uint8_t* __restrict__ scales) {
  mx_quantize_block<ACT, FRAG>(X, T, d_in, codes, scales, (long long)blockIdx.x * blockDim.x + threadIdx.x);
}

// First launch of the forward (workgroups of 16 waves).  The leading workgroups compute the
// shared projection R = X B^T: workgroup (slice kz, rank block nb) takes `kslice` channels
// (a multiple of 512; at most 4 slices) of 16 ranks, its sixteen waves a sixteenth of the
// slice each (every load of a wave in flight at once), the parts meet in LDS and leave fp32
// partial sums Rpart[slice][16][r].  The other workgroups quantise the activations.  Nothing
// waits inside.
struct MxFrontArgs {
  const uint16_t* X;
  const uint16_t* B;         // act dtype [r][d_in], or NULL when not restored
  float* Rpart;
  uint8_t* xcodes;
  uint8_t* xscales;
  int T, d_in, r, ks, kslice;
};
constexpr int MX_FRONT_THREADS = 1024;

template <int ACT>
__global__ void __launch_bounds__(MX_FRONT_THREADS) k_mx_front(MxFrontArgs a) {
  __shared__ float part[16][64][4];
  const int nbs = (a.r + 15) >> 4;
  const int n_proj = a.B ? a.ks * nbs : 0;
  if ((int)blockIdx.x >= n_proj) {
    mx_quantize_block<ACT, true>(a.X, a.T, a.d_in, a.xcodes, a.xscales,
                                 (long long)(blockIdx.x - n_proj) * MX_FRONT_THREADS + threadIdx.x);
    return;
  }
  const int kz = (int)blockIdx.x % a.ks, nb = (int)blockIdx.x / a.ks;
  const int w = threadIdx.x >> 6, l = threadIdx.x & 63, i = l & 15, g = l >> 4;
  const int per = a.kslice / 16;                                       // (a multiple of 32)
  const int kbeg = min(a.d_in, kz * a.kslice + w * per), kend = min(a.d_in, kbeg + per);
  const int rank = 16 * nb + i;
  const bool tok = i < a.T, live = rank < a.r;
  float4_t acc = {0.f, 0.f, 0.f, 0.f};
  const uint16_t* xp = a.X + (long long)(tok ? i : 0) * a.d_in + 8 * g;
  const uint16_t* bp = a.B + (long long)(live ? rank : 0) * a.d_in + 8 * g;
#pragma unroll 8
  for (int k0 = kbeg; k0 < kend; k0 += 32) {
    u32x4_t xa = {0, 0, 0, 0}, bb = {0, 0, 0, 0};
    if (tok) xa = *(const u32x4_t*)(xp + k0);
    if (live) bb = *(const u32x4_t*)(bp + k0);
    acc = mfma16<ACT>(xa, bb, acc);
  }
#pragma unroll
  for (int v = 0; v < 4; ++v) part[w][l][v] = acc[v];
  __syncthreads();
  if (w != 0) return;
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    float sum = 0.f;
#pragma unroll
    for (int q = 0; q < 16; ++q) sum += part[q][l][v];
    const int t = 4 * g + v;
    if (t < a.T && live) a.Rpart[((long long)kz * 16 + t) * a.r + rank] = sum;
  }
}

// ---------------------------------------------------------------------------------------
// the forward in two launches (5 to 16 tokens, and fewer tokens of shapes the one-launch
// kernel below does not hold).  One workgroup (4 waves) per RB consecutive 16-row blocks of
// one module; wave w takes the 128-channel tiles w, w + 4, ... and the correction step of
// ranks 32 w ..; the four partial tiles of a row block meet in LDS and wave q stores block q.
// Launched with RB = 1: with the activations in fragment order (a wave's fetch of a tile is
// two contiguous KiB) three times the waves in flight are worth more than an activation tile
// in registers that serves three weight tiles (RB = 3: 16.3 instead of 15.7 us at sixteen
// tokens on a 3 x 4096 x 4096 unit).
// Measured no faster: sixteen waves per workgroup; a walk over the tiles that starts at
// another place in every workgroup.  Measured slower: sixteen slices of the projection instead
// of four.  Measured much slower (24 instead of 13 us at one token):
// letting the projection workgroup that finishes last add the slices into R behind a
// device-scope fence, so that the correction step reads R instead of sixteen partial sums.
// ---------------------------------------------------------------------------------------
struct MxModule {
  const uint32_t* codes;     // prepared codes region
  const uint8_t* scales;     // prepared scales region
  const uint16_t* A;         // act dtype [d_out][r]
  void* Y;
  int d_out, ldy;
  int first_block;           // index of the module's first row block in the grid
};

struct MxArgs {
  MxModule mod[GLOWQ_MAX_MODULES];
  int n_modules;
  const uint16_t* X;         // act dtype [T][d_in] (the one-launch kernel quantises it itself)
  const uint8_t* xcodes;     // E4M3, fragment order (see mx_quantize_block)
  const uint8_t* xscales;    // E8M0, fragment order
  const float* Rpart;        // fp32 [ks][16][r] partial sums of R, or NULL when not restored
  int ks;
  int T, d_in, r;
  int out_f32;
};

template <int ACT, int RB>
__global__ void __launch_bounds__(256) k_mx_decode(MxArgs a) {
  __shared__ float part[4][RB][64][4];
  int mi = 0;
#pragma unroll
  for (int i = 1; i < GLOWQ_MAX_MODULES; ++i)
    if (i < a.n_modules && (int)blockIdx.x >= a.mod[i].first_block) mi = i;
  const MxModule& m = a.mod[mi];
  const int rb0 = ((int)blockIdx.x - m.first_block) * RB;          // first of this workgroup's row blocks
  const int n_rb = (m.d_out + 15) / 16;
  const int w = threadIdx.x >> 6, l = threadIdx.x & 63, i = l & 15, g = l >> 4;
  const int ktiles = a.d_in / 128;
  const bool tok = i < a.T;
  float4_t acc[RB];
  const u32x4_t* wc[RB];
  const uint8_t* ws[RB];
#pragma unroll
  for (int q = 0; q < RB; ++q) {
    acc[q] = float4_t{0.f, 0.f, 0.f, 0.f};
    const int rb = min(rb0 + q, n_rb - 1);                         // (a row block past the end repeats the last; not stored)
    wc[q] = (const u32x4_t*)m.codes + ((long long)rb * ktiles) * 64 + l;
    ws[q] = m.scales + ((long long)rb * ktiles) * 64 + l;
  }
  const uint8_t* xc = a.xcodes + l * 16;            // fragment order: a tile is two chunks of 1 KiB
  const uint8_t* xs = a.xscales + l;
#pragma unroll 8
  for (int kt = w; kt < ktiles; kt += 4) {
    u32x4_t bw[RB];
    int sb[RB];
#pragma unroll
    for (int q = 0; q < RB; ++q) {
      bw[q] = wc[q][(long long)kt * 64];
      sb[q] = ws[q][(long long)kt * 64];
    }
    u32x4_t a0 = {0, 0, 0, 0}, a1 = {0, 0, 0, 0};
    int sa = 127;
    if (tok) {
      a0 = *(const u32x4_t*)(xc + 2048 * kt);
      a1 = *(const u32x4_t*)(xc + 2048 * kt + 1024);
      sa = xs[64 * kt];
    }
    const v8i_t A = {(int)a0[0], (int)a0[1], (int)a0[2], (int)a0[3], (int)a1[0], (int)a1[1], (int)a1[2], (int)a1[3]};
#pragma unroll
    for (int q = 0; q < RB; ++q) {
      const v8i_t B = {(int)bw[q][0], (int)bw[q][1], (int)bw[q][2], (int)bw[q][3], 0, 0, 0, 0};
      acc[q] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(A, B, acc[q], 0, 4, 0, sa, 0, sb[q]);
    }
  }
  // the wave's correction step (ranks 32 w + 8 g .. + 8; r <= 128, so a wave has at most one):
  // R is the sum of the projection's slices, in slice order, rounded to the activation type
  // (token rows as A, weight rows as B)
  if (a.Rpart != nullptr && 32 * w < a.r) {
    u32x4_t ra = {0, 0, 0, 0};
    const int j0 = 32 * w + 8 * g;
    if (j0 < a.r && tok) {
      float rs[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
      for (int kz = 0; kz < a.ks; ++kz) {
        const float4_t* p = (const float4_t*)(a.Rpart + ((long long)kz * 16 + i) * a.r + j0);
        const float4_t p0 = p[0], p1 = p[1];
#pragma unroll
        for (int e = 0; e < 4; ++e) { rs[e] += p0[e]; rs[4 + e] += p1[e]; }
      }
#pragma unroll
      for (int e = 0; e < 4; ++e)
        ra[e] = (uint32_t)to_act16<ACT>(rs[2 * e]) | ((uint32_t)to_act16<ACT>(rs[2 * e + 1]) << 16);
    }
#pragma unroll
    for (int q = 0; q < RB; ++q) {
      u32x4_t rbv = {0, 0, 0, 0};
      const int row = (rb0 + q) * 16 + i;
      if (j0 < a.r && row < m.d_out) rbv = *(const u32x4_t*)(m.A + (long long)row * a.r + j0);
      acc[q] = mfma16<ACT>(ra, rbv, acc[q]);
    }
  }
#pragma unroll
  for (int q = 0; q < RB; ++q)
#pragma unroll
    for (int v = 0; v < 4; ++v) part[w][q][l][v] = acc[q][v];
  __syncthreads();
  // wave q stores row block q
  if (w >= RB) return;
  const int row = (rb0 + w) * 16 + i;
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int t = 4 * g + v;
    const float y = ((part[0][w][l][v] + part[1][w][l][v]) + part[2][w][l][v]) + part[3][w][l][v];
    if (t < a.T && row < m.d_out) {
      if (a.out_f32) ((float*)m.Y)[(long long)t * m.ldy + row] = y;
      else ((uint16_t*)m.Y)[(long long)t * m.ldy + row] = to_act16<ACT>(y);
    }
  }
}

// ---------------------------------------------------------------------------------------
// up to four tokens, one launch.  The leading workgroups are the projection (one wave per
// rank and K part, proj_wave_direct: every partial sum is published as one 8-byte slot
// {fp32 bits, low word of the launch tag} that validates itself); the others take one 16-row
// block each and do everything else themselves: every workgroup quantises the whole X into
// LDS (T d_in values, one to four 16-value pieces of some eighty instructions per thread,
// under the latency of its own weight loads, which go out right behind the loads of X: loads
// return in order, so X is there first),
// its four waves take the 128-channel tiles round robin, eight tiles per register buffer and
// two buffers in flight, and each wave asks for the slots of its own correction step in the
// middle of its first round (global -> LDS, device scope) and checks them after its stream.
// A slot that does not carry this launch's tag is asked for again; the
// projection workgroups lead the grid and wait for nothing, the wait is bounded all the same,
// and a wave that gives up stores NaN in its rows rather than leave the correction out
// unnoticed.
// LDS: part [4][64][4] floats, then the E4M3 codes [tile][half][g][4 tokens][16 bytes], then
// the scale codes [tile][block][4 tokens], then per wave and K part 1 KiB of slots.
// ---------------------------------------------------------------------------------------
constexpr int MXS_MAX_TOKENS = 4;
constexpr int MXS_ITEMS = 4;          // 16-channel pieces of X per thread, at most
constexpr int MXS_ROUND = 8;          // tiles per wave and register buffer
constexpr int MXS_MAX_PARTS = 2;      // K parts of the in-launch projection

// lds_dma16 at device scope (not served from a cache that may hold an older copy)
__device__ inline void lds_dma16_coherent(const void* gptr, uint32_t lds_base) {
  const uint32_t m = __builtin_amdgcn_readfirstlane(lds_base);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off sc1"
               : : "v"(gptr), "s"(m) : "memory", "m0");
}

template <int ACT>
__global__ void __launch_bounds__(256, 4) k_mx_decode_small(MxArgs a, ProjArgs p, int n_prod) {
  extern __shared__ __attribute__((aligned(16))) uint8_t mxs_lds[];
  const int w = threadIdx.x >> 6, l = threadIdx.x & 63, i = l & 15, g = l >> 4;
  if ((int)blockIdx.x < n_prod) {
    proj_wave_direct<ACT>(p, (int)blockIdx.x * 4 + w, l);
    return;
  }
  const int ktiles = a.d_in / 128;
  float* part = (float*)mxs_lds;
  u32x4_t* xq = (u32x4_t*)(mxs_lds + 4096);
  uint8_t* xsc = mxs_lds + 4096 + (size_t)ktiles * 512;
  const int blk = (int)blockIdx.x - n_prod;
  int mi = 0;
#pragma unroll
  for (int q = 1; q < GLOWQ_MAX_MODULES; ++q)
    if (q < a.n_modules && blk >= a.mod[q].first_block) mi = q;
  const MxModule& m = a.mod[mi];
  const int rb = blk - m.first_block;
  const bool tok = i < a.T;

  // X first: this thread's 16-channel pieces (token t, tile kt, half, g), piece index
  // tid + 256 n; the two halves of a block sit in neighbouring lanes
  const int n_items = a.T * ktiles * 8;
  u32x4_t xl[MXS_ITEMS], xh[MXS_ITEMS];
#pragma unroll
  for (int n = 0; n < MXS_ITEMS; ++n) {
    const int idx = min((int)threadIdx.x + 256 * n, n_items - 1);          // past the end: loaded again, not stored
    const int t = idx / (8 * ktiles), rem = idx - t * 8 * ktiles;
    const u32x4_t* src = (const u32x4_t*)(a.X + (size_t)t * a.d_in + 16 * rem);   // 128 kt + 64 half + 16 g = 16 rem
    if (256 * n < n_items) { xl[n] = src[0]; xh[n] = src[1]; }
  }
  // then the weights: the wave's tiles w, w + 4, ...
  const u32x4_t* wc = (const u32x4_t*)m.codes + ((size_t)rb * ktiles) * 64 + l;
  const uint8_t* ws = m.scales + ((size_t)rb * ktiles) * 64 + l;
  const int nj = (ktiles - w + 3) >> 2;
  u32x4_t bwA[MXS_ROUND], bwB[MXS_ROUND];
  int sbA[MXS_ROUND], sbB[MXS_ROUND];
  auto load = [&](u32x4_t (&bw)[MXS_ROUND], int (&sb)[MXS_ROUND], int j0) {
#pragma unroll
    for (int q = 0; q < MXS_ROUND; ++q) {
      const int kt = min(w + 4 * (j0 + q), ktiles - 1);                     // past the end: loaded again, not used
      bw[q] = wc[(size_t)kt * 64];
      sb[q] = ws[(size_t)kt * 64];
    }
  };
  load(bwA, sbA, 0);
  // the wave's correction step: ranks 32 w + 8 g .. + 8 of A_i
  const int j0r = 32 * w + 8 * g;
  const bool corr = p.B != nullptr && 32 * w < a.r;
  u32x4_t rbv = {0, 0, 0, 0};
  if (corr) {
    const int row = rb * 16 + i;
    if (j0r < a.r && row < m.d_out) rbv = *(const u32x4_t*)(m.A + (size_t)row * a.r + j0r);
  }
  // quantise (every lane of a wave goes through the same rounds)
#pragma unroll
  for (int n = 0; n < MXS_ITEMS; ++n) {
    if (256 * n < n_items) {
      const int idx = (int)threadIdx.x + 256 * n;
      u32x4_t c;
      int sc;
      mx_quantize16<ACT>(xl[n], xh[n], c, sc);
      if (idx < n_items) {
        const int t = idx / (8 * ktiles), rem = idx - t * 8 * ktiles;
        const int kt = rem >> 3, half = (rem >> 2) & 1, gg = rem & 3;
        xq[((kt * 2 + half) * 4 + gg) * 4 + t] = c;
        if (!(gg & 1)) xsc[kt * 16 + (2 * half + (gg >> 1)) * 4 + t] = (uint8_t)sc;
      }
    }
  }
  __syncthreads();

  // The slots of the wave's correction step travel global -> LDS, one load per K part: lane
  // (unit e = l & 3, token (l >> 2) & 3, rank group l >> 4) fetches 16 bytes = two slots, so
  // that the 64 bytes of a (rank group, token) lie together, [group][token][unit].  Asked
  // for in the middle of the wave's first round of tiles: behind the weights in the queue
  // (loads return in order), and late enough for the projection to have published.
  uint8_t* rfw = mxs_lds + 4096 + (size_t)ktiles * 528 + (size_t)w * (MXS_MAX_PARTS * 1024);
  const uint32_t rfw_lds = lds_address(rfw);
  const u32x4_t* rsrc;
  {
    const int e = l & 3, tk = min((l >> 2) & 3, a.T - 1), j0 = min(32 * w + 8 * (l >> 4), max(a.r - 8, 0));
    rsrc = (const u32x4_t*)((const unsigned long long*)p.Rpart + (size_t)tk * p.ksplit * a.r + j0) + e;
  }
  auto r_issue = [&]() {
#pragma unroll
    for (int part = 0; part < MXS_MAX_PARTS; ++part)
      if (part < p.ksplit) lds_dma16_coherent(rsrc + (size_t)part * (a.r >> 1), rfw_lds + part * 1024);
  };

  float4_t acc = {0.f, 0.f, 0.f, 0.f};
  auto run = [&](const u32x4_t (&bw)[MXS_ROUND], const int (&sb)[MXS_ROUND], int j0) {
#pragma unroll
    for (int q = 0; q < MXS_ROUND; ++q) {
      if (q == MXS_ROUND / 2 && j0 == 0 && corr) r_issue();
      const int kt = w + 4 * (j0 + q);
      if (kt < ktiles) {
        u32x4_t a0 = {0, 0, 0, 0}, a1 = {0, 0, 0, 0};
        int sa = 127;
        if (tok) {
          a0 = xq[((kt * 2 + 0) * 4 + g) * 4 + i];
          a1 = xq[((kt * 2 + 1) * 4 + g) * 4 + i];
          sa = xsc[kt * 16 + g * 4 + i];
        }
        const v8i_t A = {(int)a0[0], (int)a0[1], (int)a0[2], (int)a0[3], (int)a1[0], (int)a1[1], (int)a1[2], (int)a1[3]};
        const v8i_t B = {(int)bw[q][0], (int)bw[q][1], (int)bw[q][2], (int)bw[q][3], 0, 0, 0, 0};
        acc = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(A, B, acc, 0, 4, 0, sa, 0, sb[q]);
      }
    }
  };
  for (int j0 = 0; j0 < nj; j0 += 2 * MXS_ROUND) {
    const bool second = j0 + MXS_ROUND < nj;
    if (second) load(bwB, sbB, j0 + MXS_ROUND);
    run(bwA, sbA, j0);
    if (second) {
      if (j0 + 2 * MXS_ROUND < nj) load(bwA, sbA, j0 + 2 * MXS_ROUND);
      run(bwB, sbB, j0 + MXS_ROUND);
    }
  }

  if (corr) {
    if (nj <= 0) r_issue();                           // (a wave without a tile has not asked yet)
    const bool on = tok && j0r < a.r;
    const uint32_t tag = (uint32_t)(launch_tag() & 0xffffffffull);
    const u32x4_t* mine = (const u32x4_t*)(rfw + (size_t)(g * 4 + (tok ? i : 0)) * 64);
    float s[8];
    bool done = false;
    for (int spin = 0; spin < (1 << 16); ++spin) {
      vm_wait<0>();                                   // the slots asked for last have landed in LDS
      bool ok = true;
#pragma unroll
      for (int e = 0; e < 8; ++e) s[e] = 0.f;
#pragma unroll
      for (int part = 0; part < MXS_MAX_PARTS; ++part) {
        if (part < p.ksplit) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const u32x4_t u = mine[part * 64 + e];
            const uint32_t v0 = u[0], t0 = u[1], v1 = u[2], t1 = u[3];
            ok = ok && t0 == tag && t1 == tag;
            s[2 * e] += __builtin_bit_cast(float, v0);
            s[2 * e + 1] += __builtin_bit_cast(float, v1);
          }
        }
      }
      if (!on) ok = true;
      if (__builtin_amdgcn_ballot_w64(!ok) == 0ull) {
        done = true;
        break;
      }
      __builtin_amdgcn_s_sleep(2);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     // (the reads above are done with the rows)
      r_issue();
    }
    u32x4_t ra = {0, 0, 0, 0};
    if (on) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        ra[e] = (uint32_t)to_act16<ACT>(s[2 * e]) | ((uint32_t)to_act16<ACT>(s[2 * e + 1]) << 16);
    }
    acc = mfma16<ACT>(ra, rbv, acc);
    if (!done) {
      const float nan = __builtin_bit_cast(float, 0x7fc00000u);
      acc = float4_t{nan, nan, nan, nan};
    }
  }
#pragma unroll
  for (int v = 0; v < 4; ++v) part[(w * 64 + l) * 4 + v] = acc[v];
  __syncthreads();
  if (w != 0) return;
  const int row = rb * 16 + i;
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int t = 4 * g + v;
    const float y = ((part[l * 4 + v] + part[(64 + l) * 4 + v]) + part[(128 + l) * 4 + v]) + part[(192 + l) * 4 + v];
    if (t < a.T && row < m.d_out) {
      if (a.out_f32) ((float*)m.Y)[(size_t)t * m.ldy + row] = y;
      else ((uint16_t*)m.Y)[(size_t)t * m.ldy + row] = to_act16<ACT>(y);
    }
  }
}

// ---------------------------------------------------------------------------------------
// more than 16 tokens: a tiled product on the same instruction.  Workgroup tile 128 tokens x
// 128 rows, four waves as 2 x 2 with 64 x 64 each (16 accumulator tiles), K in steps of one
// 128-channel tile through two LDS buffers that are filled by direct global -> LDS loads:
// at the top of step k every wave issues its share of step k + 1 into the other buffer,
// multiplies step k, waits for its own loads and meets the others at one barrier.  No
// register holds staged data, three workgroups share a CU.  (Three buffers with the loads
// two steps ahead, two workgroups per CU: no faster.  The register-resident loop of this
// instruction measures 2.42 PFLOP/s on this machine, for fp8 x fp4 and fp4 x fp4 operands and
// for the 32x32x64 shape alike - the rate of the 16-bit instructions, not twice it.)  Both tiles sit in LDS in fragment order, so that a wave's
// fragment read is 1 KiB lane after lane (no bank conflict by construction): the weight tile
// is the prepared layout as it is in memory; the activation tile is [token block][half]
// [lane][16 bytes], which is how the quantiser leaves it in the workspace, so every load is
// one contiguous KiB.  Slots of tokens past T hold whatever the workspace held (a row of the
// first operand touches its own output row only, and those are not stored).  The correction (R from the stand-alone projection, in the activation type) is
// r / 32 more 16-bit instructions per accumulator tile in the epilogue.
// ---------------------------------------------------------------------------------------
constexpr int MXG_TOK = 128, MXG_ROWS = 128;
constexpr int MXG_A = 0, MXG_B = 16384, MXG_ASC = 24576, MXG_BSC = 25088, MXG_BUF = 25600;   // byte offsets in a buffer
constexpr int MXG_DEPTH = 2;      // LDS buffers

struct MxGemmArgs {
  MxModule mod[GLOWQ_MAX_MODULES];      // first_block: index of the module's first workgroup
  int n_modules;
  const uint8_t* xcodes;
  const uint8_t* xscales;
  const uint16_t* R16;                  // act dtype [T][r], or NULL when not restored
  int T, d_in, r, out_f32;
  int tok_tiles;                        // ceil(T / 128); token tiles of a row tile are neighbours in the grid
};

template <int ACT>
__global__ void __launch_bounds__(256) k_mx_gemm(MxGemmArgs a) {
  __shared__ __attribute__((aligned(16))) uint8_t lds[MXG_DEPTH * MXG_BUF];
  int mi = 0;
#pragma unroll
  for (int i = 1; i < GLOWQ_MAX_MODULES; ++i)
    if (i < a.n_modules && (int)blockIdx.x >= a.mod[i].first_block) mi = i;
  const MxModule& m = a.mod[mi];
  const int local = (int)blockIdx.x - m.first_block;
  const int tt = local % a.tok_tiles, nt = local / a.tok_tiles;
  const int tok0 = tt * MXG_TOK, rb0 = nt * 8;
  const int n_rb = (m.d_out + 15) / 16, ktiles = a.d_in / 128;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, i = l & 15, g = l >> 4;
  const int wm = w >> 1, wn = w & 1;
  // this wave's share of a step's loads: activation chunks 4w .. 4w + 3 (chunk = token block,
  // half), weight row blocks 2w, 2w + 1, and one of the four 256-byte pieces of the scales
  const int n_tb = (a.T + 15) / 16;                 // token blocks that exist (a tile's blocks past them repeat the last)
  const uint8_t* asrc[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int chunk = 4 * w + q, tb = min(tok0 / 16 + (chunk >> 1), n_tb - 1), h = chunk & 1;
    asrc[q] = a.xcodes + (((long long)tb * ktiles) * 2 + h) * 1024 + l * 16;
  }
  const u32x4_t* bsrc[2];
#pragma unroll
  for (int q = 0; q < 2; ++q)
    bsrc[q] = (const u32x4_t*)m.codes + ((long long)min(rb0 + 2 * w + q, n_rb - 1) * ktiles) * 64 + l;
  const uint32_t* scsrc;
  long long sc_step;                    // dwords per K tile
  if (w < 2) {
    const int tb = min(tok0 / 16 + 4 * w + (l >> 4), n_tb - 1);
    scsrc = (const uint32_t*)(a.xscales + ((long long)tb * ktiles) * 64) + (l & 15);
    sc_step = 16;
  } else {
    const int rbi = 4 * (w - 2) + (l >> 4);
    scsrc = (const uint32_t*)(m.scales + ((long long)min(rb0 + rbi, n_rb - 1) * ktiles) * 64) + (l & 15);
    sc_step = 16;
  }
  const uint32_t lds0 = lds_address(lds);
  auto issue = [&](int kt, int buf) {
    const uint32_t base = lds0 + buf * MXG_BUF;
#pragma unroll
    for (int q = 0; q < 4; ++q) lds_dma16(asrc[q] + 2048 * kt, base + MXG_A + (4 * w + q) * 1024);
#pragma unroll
    for (int q = 0; q < 2; ++q) lds_dma16(bsrc[q] + (long long)kt * 64, base + MXG_B + (2 * w + q) * 1024);
    lds_dma4(scsrc + kt * sc_step, base + (w < 2 ? MXG_ASC + 256 * w : MXG_BSC + 256 * (w - 2)));
  };
  float4_t acc[4][4];
#pragma unroll
  for (int tb = 0; tb < 4; ++tb)
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) acc[tb][nb] = float4_t{0.f, 0.f, 0.f, 0.f};
  issue(0, 0);
  vm_wait<0>();
  __syncthreads();
  for (int kt = 0; kt < ktiles; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < ktiles) issue(kt + 1, buf ^ 1);
    const uint8_t* L = lds + buf * MXG_BUF;
    v8i_t B[4];
    int sb[4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
      const int rbi = 4 * wn + nb;
      const u32x4_t bw = *(const u32x4_t*)(L + MXG_B + rbi * 1024 + l * 16);
      B[nb] = v8i_t{(int)bw[0], (int)bw[1], (int)bw[2], (int)bw[3], 0, 0, 0, 0};
      sb[nb] = L[MXG_BSC + rbi * 64 + l];
    }
#pragma unroll
    for (int tb = 0; tb < 4; ++tb) {
      const int tbg = 4 * wm + tb;
      const u32x4_t lo = *(const u32x4_t*)(L + MXG_A + (2 * tbg) * 1024 + l * 16);
      const u32x4_t hi = *(const u32x4_t*)(L + MXG_A + (2 * tbg + 1) * 1024 + l * 16);
      const int sa = L[MXG_ASC + tbg * 64 + l];
      const v8i_t A = {(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
#pragma unroll
      for (int nb = 0; nb < 4; ++nb)
        acc[tb][nb] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(A, B[nb], acc[tb][nb], 0, 4, 0, sa, 0, sb[nb]);
    }
    vm_wait<0>();          // this wave's loads of the next step have landed ...
    __syncthreads();       // ... and everybody's; everybody is done reading this step's buffer
  }
  // correction: + R A_i^T (token rows as A, weight rows as B; lane (i, g): ranks 32 s + 8 g .. + 8)
  if (a.R16) {
    for (int s = 0; 32 * s < a.r; ++s) {
      const int j0 = 32 * s + 8 * g;
      u32x4_t rb[4];
#pragma unroll
      for (int nb = 0; nb < 4; ++nb) {
        const int row = (rb0 + 4 * wn + nb) * 16 + i;
        rb[nb] = (j0 < a.r && row < m.d_out) ? *(const u32x4_t*)(m.A + (long long)row * a.r + j0) : u32x4_t{0, 0, 0, 0};
      }
#pragma unroll
      for (int tb = 0; tb < 4; ++tb) {
        const int tok = tok0 + 64 * wm + 16 * tb + i;
        const u32x4_t ra = (j0 < a.r && tok < a.T) ? *(const u32x4_t*)(a.R16 + (long long)tok * a.r + j0) : u32x4_t{0, 0, 0, 0};
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) acc[tb][nb] = mfma16<ACT>(ra, rb[nb], acc[tb][nb]);
      }
    }
  }
#pragma unroll
  for (int tb = 0; tb < 4; ++tb)
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
      const int row = (rb0 + 4 * wn + nb) * 16 + i;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int tok = tok0 + 64 * wm + 16 * tb + 4 * g + v;
        if (tok < a.T && row < m.d_out) {
          if (a.out_f32) ((float*)m.Y)[(long long)tok * m.ldy + row] = acc[tb][nb][v];
          else ((uint16_t*)m.Y)[(long long)tok * m.ldy + row] = to_act16<ACT>(acc[tb][nb][v]);
        }
      }
    }
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
size_t mx_prepared_bytes(int d_out, int d_in) {
  return (size_t)((d_out + 15) / 16) * (size_t)(d_in / 128) * (1024 + 64);
}

hipError_t launch_mx_prepare(const uint32_t* codes, const uint8_t* scales, int d_out, int d_in, void* prepared,
                             hipStream_t st) {
  const long long tiles = (long long)((d_out + 15) / 16) * (d_in / 128);
  const long long n_words = tiles * 256, n_scales = tiles * 64;
  k_mx_prepare<<<dim3((unsigned)((n_words + 255) / 256)), dim3(256), 0, st>>>(
      codes, scales, d_out, d_in, (uint32_t*)prepared, (uint8_t*)prepared + n_words * 4, n_words, n_scales);
  return hipGetLastError();
}

hipError_t launch_mx_quantize_x(const void* X, int T, int d_in, int act, uint8_t* codes, uint8_t* scales,
                                bool fragment_order, hipStream_t st) {
  const long long n = (long long)T * (d_in / 16);
  dim3 grid((unsigned)((n + 255) / 256)), block(256);
  const uint16_t* x = (const uint16_t*)X;
  if (act == GLOWQ_F16) {
    if (fragment_order) k_mx_quantize_x<ACT_F16, true><<<grid, block, 0, st>>>(x, T, d_in, codes, scales);
    else k_mx_quantize_x<ACT_F16, false><<<grid, block, 0, st>>>(x, T, d_in, codes, scales);
  } else {
    if (fragment_order) k_mx_quantize_x<ACT_BF16, true><<<grid, block, 0, st>>>(x, T, d_in, codes, scales);
    else k_mx_quantize_x<ACT_BF16, false><<<grid, block, 0, st>>>(x, T, d_in, codes, scales);
  }
  return hipGetLastError();
}

static size_t up256(size_t b) { return (b + 255) & ~(size_t)255; }

MxWorkspace plan_mx_workspace(const glowq_unit& u) {
  MxWorkspace w;
  if (u.T > MX_MAX_TOKENS) {
    // the tiled path: the unit's ordinary slice (partial sums and R of the stand-alone
    // projection), then the quantised activations
    w.ks = w.kslice = 0;
    w.off_rpart = 0;
    w.off_xcodes = up256(plan_unit_workspace(u, nullptr).bytes);
    const size_t t16 = (size_t)(u.T + 15) / 16 * 16;           // whole 16-token blocks
    w.off_xscales = w.off_xcodes + up256(t16 * u.d_in);
    w.bytes = w.off_xscales + up256(t16 * (u.d_in / 32));
    return w;
  }
  // K slices of the projection: at most 4, a multiple of 512 channels each
  w.kslice = ((u.d_in + 3) / 4 + 511) / 512 * 512;
  w.ks = (u.d_in + w.kslice - 1) / w.kslice;
  w.off_rpart = 0;
  // (partial sums [ks][16][r] of the two-launch path, or the one-launch path's slots
  // [T <= 4][parts <= 4][r] of 8 bytes)
  const size_t rr = u.r > 0 ? u.r : 0;
  w.off_xcodes = up256(std::max((size_t)w.ks * 16 * rr * 4, (size_t)MXS_MAX_TOKENS * MXS_MAX_PARTS * rr * 8));
  w.off_xscales = w.off_xcodes + up256((size_t)MX_MAX_TOKENS * u.d_in);
  w.bytes = w.off_xscales + up256((size_t)MX_MAX_TOKENS * (u.d_in / 32));
  return w;
}

static hipError_t launch_mx_gemm(const glowq_unit& u, bool restore, char* workspace, hipStream_t st) {
  const MxWorkspace w = plan_mx_workspace(u);
  uint8_t* xcodes = (uint8_t*)(workspace + w.off_xcodes);
  uint8_t* xscales = (uint8_t*)(workspace + w.off_xscales);
  hipError_t err = launch_mx_quantize_x(u.X, u.T, u.d_in, u.act_dtype, xcodes, xscales, true, st);
  if (err != hipSuccess) return err;
  const bool corrected = restore && u.r > 0;
  const UnitWorkspace uw = plan_unit_workspace(u, workspace);
  if (corrected) {
    err = launch_proj(u, uw, nullptr, true, st);          // R = X B^T in the activation type
    if (err != hipSuccess) return err;
  }
  MxGemmArgs a;
  a.n_modules = u.n_modules;
  a.tok_tiles = (u.T + MXG_TOK - 1) / MXG_TOK;
  int blocks = 0;
  for (int i = 0; i < u.n_modules; ++i) {
    const glowq_module& m = u.modules[i];
    const long long tiles = (long long)((m.d_out + 15) / 16) * (u.d_in / 128);
    a.mod[i].codes = (const uint32_t*)m.w_prepared;
    a.mod[i].scales = (const uint8_t*)m.w_prepared + tiles * 1024;
    a.mod[i].A = (const uint16_t*)m.A;
    a.mod[i].Y = m.Y;
    a.mod[i].d_out = m.d_out;
    a.mod[i].ldy = m.ldy;
    a.mod[i].first_block = blocks;
    blocks += ((m.d_out + MXG_ROWS - 1) / MXG_ROWS) * a.tok_tiles;
  }
  a.xcodes = xcodes;
  a.xscales = xscales;
  a.R16 = corrected ? (const uint16_t*)(uw.base + uw.off_r16) : nullptr;
  a.T = u.T; a.d_in = u.d_in; a.r = u.r;
  a.out_f32 = u.out_dtype == GLOWQ_F32;
  if (u.act_dtype == GLOWQ_F16) k_mx_gemm<ACT_F16><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(a);
  else k_mx_gemm<ACT_BF16><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(a);
  return hipGetLastError();
}

static int fill_mx_modules(const glowq_unit& u, int rb_per_wg, MxArgs& a) {
  a.n_modules = u.n_modules;
  int blocks = 0;
  for (int i = 0; i < u.n_modules; ++i) {
    const glowq_module& m = u.modules[i];
    const long long tiles = (long long)((m.d_out + 15) / 16) * (u.d_in / 128);
    a.mod[i].codes = (const uint32_t*)m.w_prepared;
    a.mod[i].scales = (const uint8_t*)m.w_prepared + tiles * 1024;
    a.mod[i].A = (const uint16_t*)m.A;
    a.mod[i].Y = m.Y;
    a.mod[i].d_out = m.d_out;
    a.mod[i].ldy = m.ldy;
    a.mod[i].first_block = blocks;
    blocks += ((m.d_out + 15) / 16 + rb_per_wg - 1) / rb_per_wg;
  }
  a.X = (const uint16_t*)u.X;
  a.T = u.T;
  a.d_in = u.d_in;
  a.r = u.r;
  a.out_f32 = u.out_dtype == GLOWQ_F32;
  return blocks;
}

// what the one-launch kernel holds: X of a workgroup in MXS_ITEMS pieces per thread, its
// codes in LDS
static bool mx_one_launch(const glowq_unit& u) {
  return u.T <= MXS_MAX_TOKENS && (long long)u.T * (u.d_in / 16) <= 256 * MXS_ITEMS && u.d_in <= 12288;
}

static hipError_t launch_mx_small(const glowq_unit& u, bool restore, char* workspace, hipStream_t st) {
  const MxWorkspace w = plan_mx_workspace(u);
  const bool corrected = restore && u.r > 0;
  MxArgs a;
  const int blocks = fill_mx_modules(u, 1, a);
  a.xcodes = a.xscales = nullptr;
  a.Rpart = nullptr;
  a.ks = 0;
  ProjArgs p;
  p.X = (const uint16_t*)u.X;
  p.B = corrected ? (const uint16_t*)u.B : nullptr;
  p.T = u.T; p.K = u.d_in; p.r = u.r;
  // K parts of at least 2048 channels, at most MXS_MAX_PARTS, whole 32-channel steps
  const int want = std::min(MXS_MAX_PARTS, (u.d_in + 2047) / 2048);
  p.kslice = ((u.d_in / 32 + want - 1) / want) * 32;
  p.ksplit = (u.d_in + p.kslice - 1) / p.kslice;
  p.Rpart = (float*)(workspace + w.off_rpart);
  p.R32 = nullptr; p.R16 = nullptr; p.ctl = nullptr; p.groups = 1;
  const int n_prod = corrected ? (u.r * p.ksplit + 3) / 4 : 0;        // one wave per (rank, part)
  const size_t lds = 4096 + (size_t)(u.d_in / 128) * (512 + 16) + 4 * MXS_MAX_PARTS * 1024;
  dim3 grid((unsigned)(n_prod + blocks)), block(256);
  if (u.act_dtype == GLOWQ_F16) k_mx_decode_small<ACT_F16><<<grid, block, lds, st>>>(a, p, n_prod);
  else k_mx_decode_small<ACT_BF16><<<grid, block, lds, st>>>(a, p, n_prod);
  return hipGetLastError();
}

hipError_t launch_mx_forward(const glowq_unit& u, bool restore, char* workspace, hipStream_t st) {
  if (u.T > MX_MAX_TOKENS) return launch_mx_gemm(u, restore, workspace, st);
  if (mx_one_launch(u)) return launch_mx_small(u, restore, workspace, st);
  const MxWorkspace w = plan_mx_workspace(u);
  uint8_t* xcodes = (uint8_t*)(workspace + w.off_xcodes);
  uint8_t* xscales = (uint8_t*)(workspace + w.off_xscales);
  float* rpart = (float*)(workspace + w.off_rpart);
  const bool corrected = restore && u.r > 0;
  const bool f16 = u.act_dtype == GLOWQ_F16;
  MxFrontArgs fa;
  fa.X = (const uint16_t*)u.X;
  fa.B = corrected ? (const uint16_t*)u.B : nullptr;
  fa.Rpart = rpart;
  fa.xcodes = xcodes;
  fa.xscales = xscales;
  fa.T = u.T; fa.d_in = u.d_in; fa.r = u.r; fa.ks = w.ks; fa.kslice = w.kslice;
  const int qblocks = (u.T * (u.d_in / 16) + MX_FRONT_THREADS - 1) / MX_FRONT_THREADS;
  dim3 fgrid((unsigned)(qblocks + (corrected ? w.ks * ((u.r + 15) / 16) : 0)));
  if (f16) k_mx_front<ACT_F16><<<fgrid, dim3(MX_FRONT_THREADS), 0, st>>>(fa);
  else k_mx_front<ACT_BF16><<<fgrid, dim3(MX_FRONT_THREADS), 0, st>>>(fa);
  MxArgs a;
  const int blocks = fill_mx_modules(u, 1, a);
  a.xcodes = xcodes;
  a.xscales = xscales;
  a.Rpart = corrected ? rpart : nullptr;
  a.ks = w.ks;
  dim3 grid((unsigned)blocks), block(256);
  if (f16) k_mx_decode<ACT_F16, 1><<<grid, block, 0, st>>>(a);
  else k_mx_decode<ACT_BF16, 1><<<grid, block, 0, st>>>(a);
  return hipGetLastError();
}

}  // namespace glowq
