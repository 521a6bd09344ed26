// Device-side building blocks shared by every GlowQ kernel: the prepared weight
// layout, the single-rounding dequantiser (W4A16 storage, paper Sec. 4.1), and
// thin wrappers over the gfx950 matrix-core instructions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "trace.hpp"

namespace glowq {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

enum Act { ACT_F16 = 0, ACT_BF16 = 1 };

// ---------------------------------------------------------------------------
// Prepared layout of one module's weights (built by prepare.hip): an array of tile
// records [rows16][d_in/128], one record = 16 rows x 128 channels:
//   words 0..255   : the packed weights, [64 lanes][4 words] -- one contiguous 1 KiB
//                    wave load.  Lane l holds row 16*rb + (l & 15); word j of lane l
//                    holds channels 128*kb + 32*j + 8*(l >> 4) + e, e = 0..7 -- exactly
//                    the B operand of one 16x16x32 matrix-core instruction per word;
//                    inside a word, nibble i holds e = 2i and nibble i + 4 holds
//                    e = 2i + 1, so that ((w >> 4i) & 0x000F000F) is the pair
//                    (e = 2i, e = 2i + 1)
//   words 256..271 : (s, z) of the 16 rows for the tile's first quantisation group,
//                    low half = scale bits, high half = zero-point bits
//   words 272..287 : the same for the second group (G = 64 only)
// so a tile's scales sit in the same DRAM page as its weights.  rows16 =
// ceil(d_out / 16); rows past d_out hold q = 0, s = 1, z = 0 (dequantise to 0).
// ---------------------------------------------------------------------------
struct PreparedView {
  const uint32_t* base;
  int rows16;      // 16-row blocks
  int ktiles;      // d_in / 128
  int rec_words;   // 272 (G = 128) or 288 (G = 64)
};

__host__ __device__ inline int prepared_rec_words(int G) { return 256 + 16 * (128 / G); }
__host__ __device__ inline size_t prepared_total_bytes(int d_out, int d_in, int G) {
  return (size_t)((d_out + 15) / 16) * (size_t)(d_in / 128) * prepared_rec_words(G) * 4;
}
__host__ __device__ inline PreparedView prepared_view(const void* p, int d_out, int d_in, int G) {
  PreparedView v;
  v.base = (const uint32_t*)p;
  v.rows16 = (d_out + 15) / 16;
  v.ktiles = d_in / 128;
  v.rec_words = prepared_rec_words(G);
  return v;
}

// the 16-row x 128-channel tile record (rb, kb) of a prepared weight
__device__ inline const uint32_t* tile_record(const PreparedView& v, int rb, int kb) {
  return v.base + ((size_t)rb * v.ktiles + kb) * v.rec_words;
}

// value of a 16-bit pattern of the activation type, exactly
template <int ACT> __device__ inline double act16_value(uint32_t bits16) {
  if (ACT == ACT_F16) return (double)(float)__builtin_bit_cast(_Float16, (uint16_t)bits16);
  return (double)__builtin_bit_cast(float, bits16 << 16);
}

// round a float64 to the activation type, ties to even, one rounding; returns the bits
template <int ACT> __device__ inline uint32_t act16_round(double x) {
  constexpr int FB = ACT == ACT_F16 ? 10 : 7;          // fraction bits
  constexpr int EMIN = ACT == ACT_F16 ? -14 : -126;    // exponent of the smallest normal
  constexpr int BIAS = ACT == ACT_F16 ? 15 : 127;
  constexpr uint32_t INF = ACT == ACT_F16 ? 0x7c00u : 0x7f80u;
  const uint64_t u = __builtin_bit_cast(uint64_t, x);
  const uint32_t sign = (uint32_t)(u >> 48) & 0x8000u;
  const uint64_t mag = u & 0x7fffffffffffffffull;
  if (mag > 0x7ff0000000000000ull) return sign | INF | (1u << (FB - 1));
  const double ax = __builtin_bit_cast(double, mag);
  uint32_t out;
  if (ax < __builtin_ldexp(1.0, EMIN)) {
    // below the normal range the grid is uniform: scale (exact), round once
    out = (uint32_t)__builtin_rint(ax * __builtin_ldexp(1.0, FB - EMIN));
  } else {
    constexpr int SH = 52 - FB;
    const uint64_t r = mag + ((1ull << (SH - 1)) - 1) + ((mag >> SH) & 1);   // carry may reach the exponent
    const long long e = (long long)(r >> 52) - 1023 + BIAS;
    out = e >= 2 * BIAS + 1 ? INF : ((uint32_t)e << FB) | ((uint32_t)(r >> SH) & ((1u << FB) - 1));
  }
  return sign | out;
}

// Per (row, group) constants of the dequantiser, derived once from an sz word.
template <int ACT> struct GroupConst;
template <> struct GroupConst<ACT_F16> {
  half2_t s2;    // (s, s)
  half2_t nb2;   // (-(1024 + z), -(1024 + z)), exact in binary16 for integer z <= 1023
  half2_t nb2b;  // (-(64 + z), -(64 + z)), for nibbles read under the exponent of 64
  __device__ inline void set(uint32_t szw) {
    _Float16 s = __builtin_bit_cast(_Float16, (uint16_t)(szw & 0xffffu));
    _Float16 z = __builtin_bit_cast(_Float16, (uint16_t)(szw >> 16));
    _Float16 nb = -((_Float16)1024.0f + z);
    _Float16 nbb = -((_Float16)64.0f + z);
    s2 = half2_t{s, s};
    nb2 = half2_t{nb, nb};
    nb2b = half2_t{nbb, nbb};
  }
};
template <> struct GroupConst<ACT_BF16> {
  float s;     // scale widened
  float nzs;   // -z * s, exact in fp32 (<= 4 + 11 significant bits)
  __device__ inline void set(uint32_t szw) {
    s = (float)__builtin_bit_cast(_Float16, (uint16_t)(szw & 0xffffu));
    float z = (float)__builtin_bit_cast(_Float16, (uint16_t)(szw >> 16));
    nzs = -z * s;
  }
  // -(1024 + z) s and -(64 + z) s: exact in fp32 (11 + 11 significant bits)
  __device__ inline float c1024() const { return __builtin_fmaf(-1024.0f, s, nzs); }
  __device__ inline float c64() const { return __builtin_fmaf(-64.0f, s, nzs); }
};

// Eight dequantised weights of one prepared word, in channel order e = 0..7,
// as four 32-bit registers of packed 16-bit values (a matrix-core operand).
//
// binary16: (q - z) is formed exactly (see q_minus_z_f16) and the packed multiply
// by s rounds once, to nearest even -- the definition of the stored weight.
// bfloat16: q widens to fp32 exactly, fma(q, s, -z s) is exact in fp32, and the
// packed fp32 -> bf16 conversion rounds once, to nearest even.
template <int ACT>
__device__ inline u32x4_t dequant_word(uint32_t w, const GroupConst<ACT>& g);

// (x & mask) | magic in one instruction; the mask travels in a scalar register and the
// magic constant in a vector register (gfx9 three-operand encodings take no literals)
__device__ inline uint32_t and_or(uint32_t x, uint32_t mask, uint32_t magic) {
  uint32_t r;
  asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "s"(mask), "v"(magic));
  return r;
}

// The eight values (q - z) of one prepared word as binary16 pairs, exact.  Nibbles at bits
// 0-3 / 16-19 are OR-ed into the fraction of 0x6400 (1024 + q), nibbles at bits 4-7 / 20-23
// into the fraction of 0x5400 (64 + q: one unit in the last place is 1/16 there, so bit 4
// weighs 1), the other four take the same two forms after one shift by 8; adding
// -(1024 + z) or -(64 + z) cancels the offset and the zero-point in one packed add.
__device__ inline u32x4_t q_minus_z_f16(uint32_t w, half2_t nb2, half2_t nb2b) {
  const uint32_t ws = w >> 8;
  u32x4_t out;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t src = i < 2 ? w : ws;
    const uint32_t t = (i & 1) ? and_or(src, 0x00F000F0u, 0x54005400u) : and_or(src, 0x000F000Fu, 0x64006400u);
    const half2_t v = __builtin_bit_cast(half2_t, t) + ((i & 1) ? nb2b : nb2);
    out[i] = __builtin_bit_cast(uint32_t, v);
  }
  return out;
}

// The eight nibbles of a prepared word as binary16 pairs WITHOUT the subtraction: pairs 0
// and 2 hold 1024 + q, pairs 1 and 3 hold 64 + q (five instructions).  For callers that
// take the offsets and the zero-point out of the contraction's result instead:
// sum_k x_k (off_k + q_k) - sum_k x_k off_k - z sum_k x_k = sum_k x_k (q_k - z).
__device__ inline u32x4_t nibble_forms_f16(uint32_t w) {
  const uint32_t ws = w >> 8;
  u32x4_t out;
  out[0] = and_or(w, 0x000F000Fu, 0x64006400u);
  out[1] = and_or(w, 0x00F000F0u, 0x54005400u);
  out[2] = and_or(ws, 0x000F000Fu, 0x64006400u);
  out[3] = and_or(ws, 0x00F000F0u, 0x54005400u);
  return out;
}

template <>
__device__ inline u32x4_t dequant_word<ACT_F16>(uint32_t w, const GroupConst<ACT_F16>& g) {
  u32x4_t d = q_minus_z_f16(w, g.nb2, g.nb2b);
  u32x4_t out;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t di = d[i];   // (bit_cast of a vector element lvalue reads element 0)
    half2_t v = __builtin_bit_cast(half2_t, di) * g.s2;   // the one rounding
    out[i] = __builtin_bit_cast(uint32_t, v);
  }
  return out;
}

template <>
__device__ inline u32x4_t dequant_word<ACT_BF16>(uint32_t w, const GroupConst<ACT_BF16>& g) {
  // nibble positions 0,2,4,6 (channels e = 0,4,1,5) and 1,3,5,7 (e = 2,6,3,7), one per byte,
  // so that each widening is a single byte-to-float conversion
  const uint32_t m0 = w & 0x0F0F0F0Fu;
  const uint32_t m1 = (w >> 4) & 0x0F0F0F0Fu;
  const float q0 = (float)(m0 & 0xFFu), q4 = (float)((m0 >> 8) & 0xFFu);
  const float q1 = (float)((m0 >> 16) & 0xFFu), q5 = (float)(m0 >> 24);
  const float q2 = (float)(m1 & 0xFFu), q6 = (float)((m1 >> 8) & 0xFFu);
  const float q3 = (float)((m1 >> 16) & 0xFFu), q7 = (float)(m1 >> 24);
  const float qs[8] = {q0, q1, q2, q3, q4, q5, q6, q7};
  u32x4_t out;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    bf16x2_t v;
    v[0] = (__bf16)__builtin_fmaf(qs[2 * i], g.s, g.nzs);
    v[1] = (__bf16)__builtin_fmaf(qs[2 * i + 1], g.s, g.nzs);
    out[i] = __builtin_bit_cast(uint32_t, v);
  }
  return out;
}

// dequant_word for NW words at once, cut into single vector-ALU instructions for a
// caller that schedules by hand.  Measured on gfx950 with one wave per SIMD: a matrix
// instruction (16x16x32) takes 8 of its 16 cycles of issue, two more instructions ride
// free behind it, every further one costs 4 cycles, and a vector-ALU instruction that
// reads the result of one of the two instructions before it stalls 4 cycles.  Hence the
// order: the words are taken two at a time, and within a pair instruction `idx`
// alternates between the two words, so that dependent instructions are two apart
// (with two waves per SIMD the other wave's instructions fall in between as well).  Running idx =
// 0 .. N_OPS-1 in order leaves in out[w] exactly what dequant_word returns for w[w].
template <int ACT, int NW> struct DequantLockstep;
template <int NW> struct DequantLockstep<ACT_F16, NW> {
  static constexpr int PH = 15, GS = NW < 2 ? NW : 2;
  static_assert(NW % GS == 0, "words are taken two at a time");
  static constexpr int N_OPS = NW * PH;
  uint32_t ws[GS];   // the word, shifted for the pair in flight
  half2_t d[GS];     // (q - z) pair in flight
  __device__ inline void set_group(int, const GroupConst<ACT_F16>&) {}
  __device__ inline void op(int idx, const u32x4_t (&wq)[NW], int j, const GroupConst<ACT_F16> (&g)[NW],
                            u32x4_t (&out)[NW]) {
    const int r_ = idx % (GS * PH), c = r_ % GS, w = (idx / (GS * PH)) * GS + c, ph = r_ / GS;
    // phases: ao0 add0 mul0 | shr1 ao1 add1 mul1 | shr2 ao2 add2 mul2 | shr3 ao3 add3 mul3
    const int i = (ph + 1) >> 2, kind = (ph + 1) & 3;   // kind 0 shr, 1 and_or, 2 add, 3 mul
    if (kind == 0) ws[c] = wq[w][j] >> (4 * i);
    else if (kind == 1) {
      const uint32_t t = and_or(i == 0 ? wq[w][j] : ws[c], 0x000F000Fu, 0x64006400u);
      d[c] = __builtin_bit_cast(half2_t, t);
    } else if (kind == 2) d[c] = d[c] + g[w].nb2;
    else {
      const half2_t v = d[c] * g[w].s2;   // the one rounding
      out[w][i] = __builtin_bit_cast(uint32_t, v);
    }
  }
};
// bfloat16 in 17 instructions per word.  The nibbles take the same binary16 forms as in
// the shift-free binary16 recipe (1024 + q under the exponent of 1024, 64 + q under the
// exponent of 64); a mixed-precision fused multiply-add then reads one half of such a
// pair as binary16 and computes (1024 + q) s - (1024 + z) s in fp32.  Both products have at
// most 22 significant bits and the result (q - z) s at most 15, so the fp32 value is
// exact, and the packed fp32 -> bfloat16 conversion is the one rounding of the stored
// weight.  c[w][0] = -(1024 + z) s and c[w][1] = -(64 + z) s of word w's group travel
// beside the group constants (set by the caller when a new group starts).
template <int NW> struct DequantLockstep<ACT_BF16, NW> {
  static constexpr int PH = 17, GS = NW < 2 ? NW : 2;
  static constexpr int N_OPS = NW * PH;
  uint32_t ws[GS];   // the word shifted by 8
  uint32_t t[GS];    // binary16 pair in flight
  float f[GS][2];
  float c[NW][2];
  __device__ inline void set_group(int w, const GroupConst<ACT_BF16>& g) {
    c[w][0] = g.c1024();
    c[w][1] = g.c64();
  }
  // fp32 = (binary16 half `hi` of pair) * s + c
  template <int HI> __device__ static inline float mix(uint32_t pair, float s, float c_) {
    float r;
    if (HI) asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(pair), "v"(s), "v"(c_));
    else asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(pair), "v"(s), "v"(c_));
    return r;
  }
  __device__ inline void op(int idx, const u32x4_t (&wq)[NW], int j, const GroupConst<ACT_BF16> (&g)[NW],
                            u32x4_t (&out)[NW]) {
    // words in pairs, instruction by instruction alternating between the two; an odd last
    // word runs alone
    constexpr int PAIRED = (NW / GS) * GS * PH;
    const int r_ = idx < PAIRED ? idx % (GS * PH) : idx - PAIRED;
    const int cc = idx < PAIRED ? r_ % GS : 0;
    const int w = idx < PAIRED ? (idx / (GS * PH)) * GS + cc : NW - 1;
    const int ph = idx < PAIRED ? r_ / GS : r_;
    // phases: shr | ao0 mixlo0 mixhi0 pack0 | ao1 ... | ao2 ... | ao3 ...
    if (ph == 0) { ws[cc] = wq[w][j] >> 8; return; }
    const int i = (ph - 1) >> 2, kind = (ph - 1) & 3;
    if (kind == 0) {
      const uint32_t src = i < 2 ? wq[w][j] : ws[cc];
      t[cc] = (i & 1) ? and_or(src, 0x00F000F0u, 0x54005400u) : and_or(src, 0x000F000Fu, 0x64006400u);
    } else if (kind == 1) f[cc][0] = mix<0>(t[cc], g[w].s, c[w][i & 1]);
    else if (kind == 2) f[cc][1] = mix<1>(t[cc], g[w].s, c[w][i & 1]);
    else {
      bf16x2_t v;
      v[0] = (__bf16)f[cc][0];
      v[1] = (__bf16)f[cc][1];
      out[w][i] = __builtin_bit_cast(uint32_t, v);
    }
  }
};

// binary16 with two fewer instructions per word (needs one more constant per block and
// one more register for the second magic constant).
template <int NW> struct DequantLockstepF16Shiftless {
  // Nibbles at bits 0-3 / 16-19 of a word become 1024 + q under the exponent of 1024
  // (0x6400), nibbles at bits 4-7 / 20-23 become 64 + q under the exponent of 64 (0x5400:
  // one unit in the last place is 1/16, so bit 4 weighs 1) -- no shift; the other four
  // nibbles take the same two forms after one shift by 8.  13 instructions per word.
  static constexpr int PH = 13, GS = NW < 2 ? NW : 2;
  static_assert(NW % GS == 0, "words are taken two at a time");
  static constexpr int N_OPS = NW * PH;
  uint32_t ws[GS];   // the word shifted by 8
  half2_t d[GS];     // (q - z) pair in flight
  __device__ inline void set_group(int, const GroupConst<ACT_F16>&) {}
  __device__ inline void op(int idx, const u32x4_t (&wq)[NW], int j, const GroupConst<ACT_F16> (&g)[NW],
                            u32x4_t (&out)[NW]) {
    const int r_ = idx % (GS * PH), c = r_ % GS, w = (idx / (GS * PH)) * GS + c, ph = r_ / GS;
    // phases: ao0 add0 mul0 | ao1 add1 mul1 | shr | ao2 add2 mul2 | ao3 add3 mul3
    const int p = ph < 6 ? ph : ph - 1;            // phase with the shift taken out
    const int i = p / 3, kind = p % 3;             // pair, 0 and_or / 1 add / 2 mul
    if (ph == 6) ws[c] = wq[w][j] >> 8;
    else if (kind == 0) {
      const uint32_t src = i < 2 ? wq[w][j] : ws[c];
      const uint32_t t = (i & 1) ? and_or(src, 0x00F000F0u, 0x54005400u) : and_or(src, 0x000F000Fu, 0x64006400u);
      d[c] = __builtin_bit_cast(half2_t, t);
    } else if (kind == 1) d[c] = d[c] + ((i & 1) ? g[w].nb2b : g[w].nb2);
    else {
      const half2_t v = d[c] * g[w].s2;   // the one rounding
      out[w][i] = __builtin_bit_cast(uint32_t, v);
    }
  }
};

// Nibble e (channel order) of a prepared word.
__device__ inline uint32_t prepared_nibble(uint32_t w, int e) {
  return (w >> (4 * (e >> 1) + 16 * (e & 1))) & 0xFu;
}

// D(16x16, fp32) += A(16x32) * B(32x16).  Lane l supplies row (l & 15) of A and
// column (l & 15) of B, eight k values each, k group (l >> 4); the eight values of
// lane l in A pair with the eight values of lane l in B, so any k order is fine as
// long as both operands use the same one.  D: lane l holds column (l & 15), rows
// 4*(l >> 4) + v in element v.
template <int ACT>
__device__ inline float4_t mfma16(u32x4_t a, u32x4_t b, float4_t c) {
  if constexpr (ACT == ACT_F16) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, a),
                                                  __builtin_bit_cast(half8_t, b), c, 0, 0, 0);
  } else {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  }
}

template <int ACT> __device__ inline uint16_t to_act16(float v) {
  if constexpr (ACT == ACT_F16) return __builtin_bit_cast(uint16_t, (_Float16)v);
  else return __builtin_bit_cast(uint16_t, (__bf16)v);
}

// Direct global -> LDS loads issued as assembly: lane l's BYTES land at lds_base + BYTES l
// (lds_base: byte address in LDS, the same in every lane).  As assembly because the
// compiler treats the builtin form as an access of unknown kind: while one is in flight
// EVERY wait it places for any load becomes "wait for all loads", which undoes any
// double buffering around it.  Issued like this the compiler does not know the load exists:
// its own waits only ever turn out stricter than needed (an unknown load in flight makes a
// wait for "all but the last N" cover one load more), and whoever reads the landed bytes
// places the wait (s_waitcnt vmcnt) by hand; loads of a wave complete in issue order.
__device__ inline void lds_dma16(const void* gptr, uint32_t lds_base) {
  const uint32_t m = __builtin_amdgcn_readfirstlane(lds_base);   // (a scalar register, whatever the compiler believes)
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               : : "v"(gptr), "s"(m) : "memory", "m0");
}
__device__ inline void lds_dma4(const void* gptr, uint32_t lds_base) {
  const uint32_t m = __builtin_amdgcn_readfirstlane(lds_base);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off"
               : : "v"(gptr), "s"(m) : "memory", "m0");
}
// lds_dma4 at device scope: not served from an L2 line that may hold what another compute
// unit's workgroup wrote before its latest store (the XCDs' L2s are not coherent with each other)
__device__ inline void lds_dma4_coherent(const void* gptr, uint32_t lds_base) {
  const uint32_t m = __builtin_amdgcn_readfirstlane(lds_base);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off sc1"
               : : "v"(gptr), "s"(m) : "memory", "m0");
}
__device__ inline uint32_t lds_address(const void* p) {
  return __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p);
}

// LDS reads issued as assembly (the result is pending until an lds_wait that names it)
__device__ inline void lds_read(u32x4_t& v, uint32_t addr, int imm) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(imm) : "memory");
}
__device__ inline void lds_read32(uint32_t& v, uint32_t addr, int imm) {
  asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(imm) : "memory");
}
template <int N> __device__ inline void lds_wait(u32x4_t& v) {
  asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(v) : "n"(N) : "memory");
}

// A 16-byte global load whose completion is waited for by hand (vm_wait): the compiler
// does not see it as a memory operation, so it adds no wait of its own, and the waits
// it does add for loads it knows never cover these.
__device__ inline void vm_load(u32x4_t& v, const void* p) {
  asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(v) : "v"(p) : "memory");
}
template <int N> __device__ inline void vm_wait() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// ties a value to a point behind a wait, so that nothing that uses it moves above
__device__ inline void after_wait(u32x4_t& v) { asm volatile("" : "+v"(v)); }
__device__ inline void after_wait32(uint32_t& v) { asm volatile("" : "+v"(v)); }

// Control words at the head of a unit's workspace slice.
struct Control {
  uint32_t unused[3];
  uint32_t status;           // word 3; nonzero: a bounded wait expired and the unit's correction was left out
  uint32_t pad[12];
};

// A value that is the same for every workgroup of one kernel launch and differs from
// launch to launch, graph replays included: the queue's packet index of this dispatch
// mixed with the address of the queue it sits in.  Odd, hence never zero.
extern "C" __device__ unsigned long long glowq_llvm_dispatch_id(void) __asm("llvm.amdgcn.dispatch.id");
__device__ inline unsigned long long launch_tag() {
  const unsigned long long q = (unsigned long long)__builtin_amdgcn_queue_ptr();
  const unsigned long long t = q * 0x9E3779B97F4A7C15ull + glowq_llvm_dispatch_id();
  return (t << 1) | 1ull;
}

}  // namespace glowq
