// Workgroup body of the decode path: one 16-row block of one module against up
// to 32 tokens, streamed once over the packed weights (paper Eq. 9).
#pragma once
#include "common.hpp"
#include "proj_device.hpp"
#include "../../include/glowq.h"

namespace glowq {

constexpr int DEC_WAVES = 4;
constexpr int DEC_CHUNK = 4;   // tiles per register buffer; two buffers are in flight
// `mid` (the fetch of R) is issued behind this tile of the wave's first chunk: measured,
// one token, 7B-sized group: 9.5 / 9.2 / 9.5 us behind tile 0 / 1 / 3 (earlier, more
// waves read R before it is published and pay a second fetch; later, the fetch itself
// ends after the wave's stream)
constexpr int DEC_MID_TILE = 1;

struct ModuleArgs {
  const uint32_t* rec;   // tile records (see common.hpp)
  const uint16_t* A;
  void* Y;
  int d_out, ldy, rows16, blk_start;
};

struct DecodeArgs {
  ModuleArgs mod[GLOWQ_MAX_MODULES];
  int n_modules;
  const uint16_t* X;
  int T, K, r, G;
  int restore, out_f32;
  Control* ctl;        // control words of the unit's workspace slice (null if not restored)
};

// One tile (16 rows x 128 channels) against TBK blocks of 16 tokens.
// sz0 / sz1: the (s, z) words of the tile's first and second 64 channels (equal
// when the quantisation group is 128 wide).  xfrag(tb, j) returns the A operand of
// word j: lane (i, kq) holds X[token 16 tb + i][32 j + 8 kq .. + 8] of this tile.
// NV: elements of a lane's accumulator that can hold real tokens (1 when T == 1: token 0
// is element 0 of lanes 0..15), so that the per-group scaling touches nothing else.
template <int ACT, int TBK, bool G128, int NV = 4, class XF>
__device__ inline void decode_tile(const u32x4_t w, uint32_t sz0, uint32_t sz1, XF xfrag,
                                   float4_t (&acc)[TBK]) {
  if constexpr (ACT == ACT_F16) {
    constexpr int HALVES = G128 ? 1 : 2;
    constexpr int WPH = 4 / HALVES;          // words per scale group
#pragma unroll
    for (int hf = 0; hf < HALVES; ++hf) {
      GroupConst<ACT_F16> g;
      g.set(hf == 0 ? sz0 : sz1);
      const float s = (float)g.s2[0];
      float4_t tmp[TBK];
#pragma unroll
      for (int jj = 0; jj < WPH; ++jj) {
        const int j = hf * WPH + jj;
        const u32x4_t wf = q_minus_z_f16(w[j], g.nb2, g.nb2b);
#pragma unroll
        for (int tb = 0; tb < TBK; ++tb) {
          const u32x4_t xf = xfrag(tb, j);
          if (jj == 0) tmp[tb] = mfma16<ACT>(xf, wf, float4_t{0.f, 0.f, 0.f, 0.f});
          else tmp[tb] = mfma16<ACT>(xf, wf, tmp[tb]);   // D[token][row]
        }
      }
#pragma unroll
      for (int tb = 0; tb < TBK; ++tb)
#pragma unroll
        for (int v = 0; v < NV; ++v) acc[tb][v] = __builtin_fmaf(s, tmp[tb][v], acc[tb][v]);
    }
  } else {
    GroupConst<ACT> g0, g1;
    g0.set(sz0);
    g1.set(sz1);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const u32x4_t wf = dequant_word<ACT>(w[j], (G128 || j < 2) ? g0 : g1);
#pragma unroll
      for (int tb = 0; tb < TBK; ++tb) acc[tb] = mfma16<ACT>(xfrag(tb, j), wf, acc[tb]);
    }
  }
}

// One token, binary16, group size 128, with the offsets and the zero-point taken out of
// the contraction's result: the word's nibbles go to the matrix cores as 1024 + q and
// 64 + q (five instructions per word instead of nine), and
//   sum_k x_k (q_k - z) = tmp - c1 - z S,   c1 = sum_k x_k off_k,   S = sum_k x_k.
// c1 and S come from the matrix cores as well, which have time to spare here: a second
// product of the same X fragment with a constant operand whose column 0 holds the offsets
// and whose column 1 holds ones (offsets_operand), accumulated exactly like tmp, so that
// what the two sums lose to rounding (2^-24 at the magnitude of 1024 sum |x|) is largely
// the same on both sides of the subtraction; nothing is lost when X is a row of the
// identity.  Token 0 sits in element 0 of lanes 0..15, so c1 is lane 0's and S lane 1's.
__device__ inline u32x4_t offsets_operand(int lane) {
  const int n = lane & 15;
  const uint32_t p1024 = 0x64006400u, p64 = 0x54005400u, ones = 0x3C003C00u;
  if (n == 0) return u32x4_t{p1024, p64, p1024, p64};
  if (n == 1) return u32x4_t{ones, ones, ones, ones};
  return u32x4_t{0u, 0u, 0u, 0u};
}
template <class XF>
__device__ inline void decode_tile_offsets(const u32x4_t w, uint32_t sz, XF xfrag, const u32x4_t offc,
                                           float4_t (&acc)[1]) {
  float4_t tmp, off;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const u32x4_t wf = nibble_forms_f16(w[j]);
    const u32x4_t xf = xfrag(0, j);
    tmp = mfma16<ACT_F16>(xf, wf, j == 0 ? float4_t{0.f, 0.f, 0.f, 0.f} : tmp);     // D[token][row]
    off = mfma16<ACT_F16>(xf, offc, j == 0 ? float4_t{0.f, 0.f, 0.f, 0.f} : off);   // D[token][0 | 1]
  }
  const float c1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, off[0]), 0));
  const float S = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, off[0]), 1));
  const float s = (float)__builtin_bit_cast(_Float16, (uint16_t)(sz & 0xffffu));
  const float z = (float)__builtin_bit_cast(_Float16, (uint16_t)(sz >> 16));
  const float u = __builtin_fmaf(z, S, c1);
  acc[0][0] = __builtin_fmaf(s, tmp[0] - u, acc[0][0]);
}

// T <= 4: the same stream with X staged through LDS.  Each wave owns the K tiles it
// multiplies, so it also owns their slice of X: per chunk of four tiles one direct
// global->LDS load per token (64 lanes x 16 bytes = the 4 x 256 bytes of X the chunk
// needs) travels with the chunk's weight loads, and the A operands come back with
// 128-bit LDS reads (a broadcast for one token).  No workgroup barrier is involved.
constexpr int DEC_SMALL_T = 4;
constexpr int DEC_XROW = 1040;                       // bytes per token and chunk (1 KiB + pad)
// one chunk buffer holds TM rows (TM: the most tokens the kernel instance takes; the
// single-token instance leaves room for four workgroups per compute unit); a wave has two
__host__ __device__ constexpr int dec_xbuf_bytes(int T) { return (T * DEC_XROW + 63) / 64 * 64; }


// 4 < T <= 32: a workgroup takes DEC_RG consecutive 16-row blocks of the unit (they may
// belong to different modules) and runs them against the same X fragments, held in
// registers: X is read once per workgroup instead of once per row block.  Two tiles per
// register buffer, two buffers in flight.
constexpr int DEC_RG = 3;
#ifndef GLOWQ_DEC_RCH
#define GLOWQ_DEC_RCH 2
#endif
constexpr int DEC_RCH = GLOWQ_DEC_RCH;

// `mark(n)` runs after the n-th buffer has been consumed.
template <int ACT, int TBK, bool G128, int NW, typename MARK>
__device__ inline void decode_stream_rows(const DecodeArgs& a, const uint32_t* const (&recb)[DEC_RG],
                                          int wave, int lane, float4_t (&acc)[DEC_RG][TBK], MARK mark) {
  const int n = lane & 15, kq = lane >> 4;
  const int ktiles = a.K >> 7;
  const int rw = G128 ? 272 : 288;             // words per tile record
  // this wave's tiles: kb = wave + NW * t, t = 0 .. ntw - 1
  const int ntw = (ktiles - wave + NW - 1) / NW;
  if (ntw <= 0) return;
  // tokens past T read the last valid token: their rows of D are never stored
  const uint16_t* xrow[TBK];
#pragma unroll
  for (int tb = 0; tb < TBK; ++tb)
    xrow[tb] = a.X + (size_t)min(16 * tb + n, a.T - 1) * a.K + 8 * kq + 128 * wave;

  struct Buf {
    u32x4_t x[DEC_RCH][TBK][4];
    u32x4_t w[DEC_RCH][DEC_RG];
    uint32_t s[DEC_RCH][DEC_RG][2];
  };
  Buf A, B;
  auto load = [&](int t0, Buf& b) {
#pragma unroll
    for (int c = 0; c < DEC_RCH; ++c) {
      const int t = min(t0 + c, ntw - 1);          // clamped: a duplicate tile is never used
#pragma unroll
      for (int tb = 0; tb < TBK; ++tb)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          b.x[c][tb][j] = *(const u32x4_t*)(xrow[tb] + (size_t)t * (128 * NW) + 32 * j);
#pragma unroll
      for (int g = 0; g < DEC_RG; ++g) {
        const uint32_t* rec = recb[g] + (size_t)t * (NW * rw);
        b.w[c][g] = __builtin_nontemporal_load((const u32x4_t*)rec + lane);
        b.s[c][g][0] = __builtin_nontemporal_load(rec + 256 + n);
        if constexpr (G128) b.s[c][g][1] = b.s[c][g][0];
        else b.s[c][g][1] = __builtin_nontemporal_load(rec + 272 + n);
      }
    }
  };
  auto run = [&](int t0, const Buf& b) {
#pragma unroll
    for (int c = 0; c < DEC_RCH; ++c) {
      if (t0 + c < ntw) {
#pragma unroll
        for (int g = 0; g < DEC_RG; ++g)
          decode_tile<ACT, TBK, G128>(b.w[c][g], b.s[c][g][0], b.s[c][g][1],
                                      [&](int tb, int j) { return b.x[c][tb][j]; }, acc[g]);
      }
    }
  };
  // Between the issue of a buffer's loads and its use every load is issued unconditionally:
  // the compiler can then count, at the wait, how many younger loads may stay in flight
  // (a load behind a branch in between makes it wait for ALL loads, the next buffer's
  // included, and the double buffering is gone).  Hence the peeled tail.
  // (and the scheduler may not move a buffer's first use up into the previous buffer's
  // run, behind which that buffer's loads have only just been issued)
  auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
  int done = 0;                                    // buffers consumed; `mark` hears of each
  load(0, A);
  int t0 = 0;
  while (t0 + 2 * DEC_RCH < ntw) {                 // both next buffers hold at least one tile
    load(t0 + DEC_RCH, B);
    fence();
    run(t0, A);
    mark(++done);
    fence();
    load(t0 + 2 * DEC_RCH, A);
    fence();
    run(t0 + DEC_RCH, B);
    mark(++done);
    fence();
    t0 += 2 * DEC_RCH;
  }
  if (t0 + DEC_RCH < ntw) {
    load(t0 + DEC_RCH, B);
    fence();
    run(t0, A);
    mark(++done);
    fence();
    run(t0 + DEC_RCH, B);
    mark(++done);
  } else {
    fence();
    run(t0, A);
    mark(++done);
  }
}

// X staging and its ordering.  Loads of a wave complete in the order they were issued,
// so a chunk's X has landed as soon as any load issued after it has: with room for three
// chunk buffers (TM <= 2) the X of chunk k+1 goes out ahead of the weights of chunk k
// and needs no wait at all by the time it is read; with two buffers (TM = 4) the X of
// chunk k goes out ahead of its own weights and is read once their first words are
// here.  The operand reads are issued as assembly, one tile ahead of their use, behind a
// register dependency on such a "later" load, so that neither the compiler's scheduler
// nor its own bookkeeping of LDS-bound loads has a say in the order.
// `mid` runs once, behind tile DEC_MID_TILE of the wave's first chunk (or right away if the
// wave has no tiles).
template <int TM> struct DecX {
  static constexpr bool EARLY = TM <= 2;
  static constexpr int NBUF = EARLY ? 3 : 2;
  static constexpr int WAVE_BYTES = NBUF * dec_xbuf_bytes(TM);
};

template <int ACT, bool G128, int NV, int TM, bool OFFS, class MID>
__device__ inline void decode_stream_small(const DecodeArgs& a, const ModuleArgs& M, int rb,
                                           int wave, int lane, float4_t (&acc)[1],
                                           char* lds_wave, MID mid) {
  constexpr bool EARLY = DecX<TM>::EARLY;
  constexpr int NBUF = DecX<TM>::NBUF;
  const int n = lane & 15, kq = lane >> 4;
  const int ktiles = a.K >> 7;
  const int rw = G128 ? 272 : 288;             // words per tile record
  const int ntw = (ktiles - wave + DEC_WAVES - 1) / DEC_WAVES;
  if (ntw <= 0) { mid(); return; }
  const uint32_t* rec0 = M.rec + ((size_t)rb * ktiles + wave) * rw;
  // staging: lane -> (tile of the chunk, 16-byte piece of its 128 channels)
  const int lc = lane >> 4, lp = lane & 15;
  const uint16_t* xsrc = a.X + 128 * wave + 8 * lp;
  // reading: lane (i, kq) -> token min(i, T - 1), piece 4 j + kq
  constexpr int xbuf = dec_xbuf_bytes(TM);
  const uint32_t lds_wave_addr = lds_address(lds_wave);
  const uint32_t xrd = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds_wave +
                       (uint32_t)(min(n, a.T - 1) * DEC_XROW + kq * 16);

  u32x4_t wA[DEC_CHUNK], wB[DEC_CHUNK];
  uint32_t sA[DEC_CHUNK][2], sB[DEC_CHUNK][2];

  auto load_x = [&](int idx) {   // X of chunk idx -> ring buffer idx % NBUF
    const int tx = min(idx * DEC_CHUNK + lc, ntw - 1);
    const uint16_t* src = xsrc + (size_t)tx * (128 * DEC_WAVES);
    const uint32_t dst = lds_wave_addr + (uint32_t)((idx % NBUF) * xbuf);
    for (int tok = 0; tok < a.T; ++tok) lds_dma16(src + (size_t)tok * a.K, dst + tok * DEC_XROW);
  };
  auto load_chunk = [&](int idx, u32x4_t (&w)[DEC_CHUNK], uint32_t (&s)[DEC_CHUNK][2]) {
    // X first: a tile needs its X before anything else
    load_x(EARLY ? idx + 1 : idx);
    const int t0 = idx * DEC_CHUNK;
#pragma unroll
    for (int c = 0; c < DEC_CHUNK; ++c) {
      const int t = min(t0 + c, ntw - 1);          // clamped: a duplicate tile is never used
      const uint32_t* rec = rec0 + (size_t)t * (DEC_WAVES * rw);
      w[c] = __builtin_nontemporal_load((const u32x4_t*)rec + lane);
      s[c][0] = __builtin_nontemporal_load(rec + 256 + n);
      if constexpr (G128) s[c][1] = s[c][0];
      else s[c][1] = __builtin_nontemporal_load(rec + 272 + n);
    }
  };
  uint32_t landed = 0;   // a word of a load issued after the X that is read next
  const u32x4_t offc = offsets_operand(lane);   // (OFFS only)
  auto run_chunk = [&](int idx, const u32x4_t (&w)[DEC_CHUNK], const uint32_t (&s)[DEC_CHUNK][2]) {
    const int t0 = idx * DEC_CHUNK;
    const uint32_t w00 = w[0][0];
    if (!EARLY || idx == 0) landed = w00;
    uint32_t xc = xrd + (uint32_t)((idx % NBUF) * xbuf);
    asm volatile("" : "+v"(xc) : "v"(landed));
    u32x4_t xf[2][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) lds_read(xf[0][j], xc, 64 * j);
#pragma unroll
    for (int c = 0; c < DEC_CHUNK; ++c) {
      if (c + 1 < DEC_CHUNK) {
#pragma unroll
        for (int j = 0; j < 4; ++j) lds_read(xf[(c + 1) & 1][j], xc, (c + 1) * 256 + 64 * j);
        asm volatile("s_waitcnt lgkmcnt(4)" : "+v"(xf[c & 1][0]), "+v"(xf[c & 1][1]), "+v"(xf[c & 1][2]),
                     "+v"(xf[c & 1][3]) : : "memory");
      } else {
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(xf[c & 1][0]), "+v"(xf[c & 1][1]), "+v"(xf[c & 1][2]),
                     "+v"(xf[c & 1][3]) : : "memory");
      }
      if (t0 + c < ntw) {
        if constexpr (OFFS) {
          decode_tile_offsets(w[c], s[c][0], [&](int, int j) { return xf[c & 1][j]; }, offc, acc);
        } else {
          decode_tile<ACT, 1, G128, NV>(w[c], s[c][0], s[c][1], [&](int, int j) { return xf[c & 1][j]; }, acc);
        }
      }
      if (c == DEC_MID_TILE && idx == 0) mid();
    }
    landed = w00;   // the next chunk's X went out before this chunk's weights (EARLY)
  };

  // Between the issue of a chunk's loads and their use every load the compiler knows of is
  // issued unconditionally (peeled tail), and the scheduler is kept from moving a chunk's
  // first use up into the previous chunk's run: then each run waits for its own chunk only,
  // with the next one in flight.
  auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
  const int nchunks = (ntw + DEC_CHUNK - 1) / DEC_CHUNK;
  if (EARLY) load_x(0);
  load_chunk(0, wA, sA);
  int idx = 0;
  while (idx + 2 < nchunks) {
    load_chunk(idx + 1, wB, sB);
    fence();
    run_chunk(idx, wA, sA);
    fence();
    load_chunk(idx + 2, wA, sA);
    fence();
    run_chunk(idx + 1, wB, sB);
    fence();
    idx += 2;
  }
  if (idx + 1 < nchunks) {
    load_chunk(idx + 1, wB, sB);
    fence();
    run_chunk(idx, wA, sA);
    fence();
    run_chunk(idx + 1, wB, sB);
  } else {
    fence();
    run_chunk(idx, wA, sA);
  }
}

// Direct mode (T <= 4): every (rank, K part) wave of the projection leaves, per token,
// one 8-byte slot {partial sum, low word of its launch tag}; slot of (t, part, j) is
// slots[(t ksplit + part) r + j], so the eight ranks a lane needs for its matrix operand
// are one 64-byte line per part.  Each wave fetches, for its own correction step only,
// the slots of its lanes (lane (token n, kq): ranks 32 wave + 8 kq .. + 8), checks that
// every one carries THIS launch's tag, adds the parts in part order and rounds to the
// activation type: no LDS, no workgroup barrier.
//
// The first attempt is issued during the weight stream, so its latency is hidden: the
// projection waves publish within the first couple of microseconds.  It is a device-scope
// load like the retries: an ordinary load can be served from a line that this XCD's L2
// still holds from an earlier launch through the same workspace (always, when the same
// operands are used launch after launch), which then costs a second fetch at the end of the
// stream (one token on a 3 x 4096 x 4096 unit: 9.4 -> 8.9 us).  A slot read too early shows
// an older tag and is read again.  The wait is bounded (the projection waves wait for
// nothing, so it cannot expire); if it did, ctl->status is set and the correction is left
// out rather than hang.
constexpr int DEC_MAX_PARTS = 4;   // K parts of the direct projection (see plan_unit_workspace)
struct RFetch {
  u32x4_t v[DEC_MAX_PARTS][4];     // per part: 8 slots = 64 bytes
  const unsigned long long* q;     // this lane's first slot of part 0
  int part_stride;                 // slots between parts
  bool on;                         // this lane contributes ranks of a real token
};

__device__ inline void r_fetch_plan(const DecodeArgs& a, const ProjArgs& p, int j0c, bool lane_on,
                                    int lane, RFetch& f) {
  const int n = lane & 15;
  f.on = lane_on && n < a.T;
  f.part_stride = a.r;
  f.q = (const unsigned long long*)p.Rpart + (size_t)(f.on ? n : 0) * p.ksplit * a.r + j0c;
}
// First attempt: the wave's 32 ranks of every (token, part), 256 bytes each, go straight
// into its rows of LDS (a load the compiler accounts for exactly, issued in the middle of
// the weight stream, no registers held).  Lanes past rank r load nothing.
__device__ inline void r_fetch_issue(const DecodeArgs& a, const ProjArgs& p, int wave, int lane,
                                     uint32_t* lds_rf_wave) {
  const bool in = 32 * wave + (lane >> 1) < a.r;
  const uint32_t* src = (const uint32_t*)p.Rpart + (size_t)64 * wave + lane;
  const uint32_t dst = lds_address(lds_rf_wave);
  for (int t = 0; t < a.T; ++t)
    for (int part = 0; part < p.ksplit; ++part)
      if (in) lds_dma4_coherent(src + (size_t)(t * p.ksplit + part) * a.r * 2, dst + (t * DEC_MAX_PARTS + part) * 256);
}
__device__ inline void r_fetch_take(const DecodeArgs& a, const ProjArgs& p, int lane,
                                    const uint32_t* lds_rf_wave, RFetch& f) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the loads above have landed
  const int n = lane & 15, kq = lane >> 4;
#pragma unroll
  for (int part = 0; part < DEC_MAX_PARTS; ++part)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f.v[part][i] = u32x4_t{0u, 0u, 0u, 0u};
      if (f.on && part < p.ksplit)
        f.v[part][i] = *(const u32x4_t*)(lds_rf_wave + (n * DEC_MAX_PARTS + part) * 64 + 16 * kq + 4 * i);
    }
}
// returns false if the bounded wait expired (status recorded); rf: the lane's operand
template <int ACT>
__device__ inline bool r_fetch_finish(const ProjArgs& p, RFetch& f, u32x4_t& rf) {
  const uint32_t tag = (uint32_t)(launch_tag() & 0xffffffffull);
  float s[8];
  bool done = false;
  for (int spin = 0; spin < (1 << 14); ++spin) {
    bool ok = true;
#pragma unroll
    for (int e = 0; e < 8; ++e) s[e] = 0.f;
#pragma unroll
    for (int part = 0; part < DEC_MAX_PARTS; ++part) {
      if (part < p.ksplit) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const u32x4_t q = f.v[part][i];
          const uint32_t v0 = q[0], t0 = q[1], v1 = q[2], t1 = q[3];   // (bit_cast of a vector
          ok = ok && (t0 == tag) && (t1 == tag);                       //  element reads element 0)
          s[2 * i] += __builtin_bit_cast(float, v0);
          s[2 * i + 1] += __builtin_bit_cast(float, v1);
        }
      }
    }
    if (!f.on) ok = true;
    if (__builtin_amdgcn_ballot_w64(!ok) == 0ull) {
      done = true;
      break;
    }
    __builtin_amdgcn_s_sleep(2);
    // again, past every cache that may hold a stale copy
#pragma unroll
    for (int part = 0; part < DEC_MAX_PARTS; ++part) {
      if (f.on && part < p.ksplit) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const unsigned long long* q = f.q + (size_t)part * f.part_stride + 2 * i;
          const unsigned long long lo = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          const unsigned long long hi = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          f.v[part][i] = u32x4_t{(uint32_t)lo, (uint32_t)(lo >> 32), (uint32_t)hi, (uint32_t)(hi >> 32)};
        }
      }
    }
  }
  if (!done) {
    if ((threadIdx.x & 63) == 0) atomicOr(&p.ctl->status, 1u);
    return false;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
    rf[i] = f.on ? ((uint32_t)to_act16<ACT>(s[2 * i]) | ((uint32_t)to_act16<ACT>(s[2 * i + 1]) << 16)) : 0u;
  return true;
}

// A_i fragments of this wave's correction steps (32 ranks each; wave w takes steps
// w, w + 4, ...: at most one step per wave up to rank 128).  They are asked for before the
// weight stream and travel global -> LDS directly, 16 bytes per lane into a 1 KiB row of
// the wave's own: a load into registers inside the `if (restored)` would make the wave
// wait for it at the end of that block, one memory round trip before it has asked for a
// single weight.  The row is read back after the stream (correction_take).
struct CorrFrag {
  u32x4_t af;
  int j0c;
  bool active, ok;
};
__device__ inline CorrFrag correction_prefetch(const DecodeArgs& a, const ModuleArgs& M, int rb,
                                               int wave, int lane, uint32_t* lds_row) {
  CorrFrag c;
  const int n = lane & 15, kq = lane >> 4;
  c.active = a.restore && wave * 32 < a.r;
  const int j0 = wave * 32 + 8 * kq;
  c.ok = j0 < a.r;                          // ranks past r contribute zeros on both sides
  c.j0c = c.ok ? j0 : 0;
  c.af = u32x4_t{0u, 0u, 0u, 0u};
  if (c.active) {
    const int row = min(rb * 16 + n, M.d_out - 1);
    lds_dma16(M.A + (size_t)row * a.r + c.j0c, lds_address(lds_row));
  }
  return c;
}
// after every load of the wave has completed (s_waitcnt vmcnt(0)); lanes whose ranks lie
// past r get zeros
__device__ inline void correction_take(CorrFrag& c, const uint32_t* lds_row, int lane) {
  if (c.active && c.ok) c.af = *(const u32x4_t*)(lds_row + 4 * lane);
}

// Correction R A_i^T as r more channels of the contraction (4 < T <= 32).  R comes from
// the projection workgroups of the same launch as self-validating 8-byte slots
// {fp32 partial sum, launch tag}, slot (t, part, j) at slots[(t ksplit + part) r + j]: one
// contiguous region per unit.  The workgroup gathers it together: a thread owns pairs of
// adjacent ranks of a token and reads their slots of every part with 16-byte
// device-coherent loads (consecutive lanes read consecutive addresses), checks the tags,
// adds the parts in part order, rounds to the activation type and leaves R in LDS, from
// where every lane takes the operand words of its token and rank chunk.  (Eight-byte
// loads per lane, token and rank straight from memory cost several times the whole
// weight stream's tail: one request per lane and slot.)  The projection workgroups lead
// the grid and wait for nothing; the wait is bounded all the same, and a workgroup that
// gives up records it in ctl->status and leaves the correction out.
// r_lds: act dtype [16 TBK][r]; flag: one LDS word.  Returns false if the bounded wait
// expired (the same answer in every thread of the workgroup).
__device__ inline void vm_load_dev(u32x4_t& v, const void* p) {
  asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v) : "v"(p) : "memory");
}
template <int ACT, int TBK, int NW, int MAXP>
__device__ inline bool fetch_r_coop_parts(const DecodeArgs& a, const ProjArgs& p, uint16_t* r_lds, uint32_t* flag) {
  const int tid = threadIdx.x;
  const int hp = a.r >> 1;                     // rank pairs (16-byte units) per token and part
  const int n_el = a.T * hp;                   // (token, rank pair) elements, <= 32 * 64
  const uint32_t tag = (uint32_t)(launch_tag() & 0xffffffffull);
  const u32x4_t* units = (const u32x4_t*)p.Rpart;
  constexpr int EPR = 2;                       // elements per thread and round
  if (tid == 0) *flag = 0u;
  __syncthreads();
  for (int spin = 0; spin < (1 << 12); ++spin) {
    bool ok = true;
    for (int e0 = 0; e0 < n_el; e0 += EPR * NW * 64) {
      u32x4_t v[EPR][MAXP];
      int el[EPR];
#pragma unroll
      for (int k = 0; k < EPR; ++k) {
        el[k] = e0 + k * NW * 64 + tid;
        const int ec = min(el[k], n_el - 1);   // clamped: loaded again, not used
        const int tok = ec / hp, rp = ec - tok * hp;
        const size_t u0 = (size_t)tok * p.ksplit * hp + rp;
#pragma unroll
        for (int part = 0; part < MAXP; ++part) {
          vm_load_dev(v[k][part], units + u0 + (size_t)min(part, p.ksplit - 1) * hp);
        }
      }
      vm_wait<0>();
#pragma unroll
      for (int k = 0; k < EPR; ++k) {
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int part = 0; part < MAXP; ++part) {
          after_wait(v[k][part]);
          if (part < p.ksplit) {
            // (elements copied to scalars first: a bit cast applied directly to a vector
            // element reads element 0)
            const uint32_t w0 = v[k][part][0], t0 = v[k][part][1], w1 = v[k][part][2], t1 = v[k][part][3];
            ok = ok && t0 == tag && t1 == tag;
            s0 += __builtin_bit_cast(float, w0);
            s1 += __builtin_bit_cast(float, w1);
          }
        }
        if (el[k] < n_el)
          ((uint32_t*)r_lds)[el[k]] = (uint32_t)to_act16<ACT>(s0) | ((uint32_t)to_act16<ACT>(s1) << 16);
      }
    }
    if (!ok) *flag = 1u;
    __syncthreads();
    const bool failed = *flag != 0u;
    if (!failed) return true;                  // R is complete in LDS
    __syncthreads();
    if (tid == 0) *flag = 0u;
    __builtin_amdgcn_s_sleep(32);
    __syncthreads();
  }
  if (tid == 0) atomicOr(&a.ctl->status, 1u);
  return false;
}

template <int ACT, int TBK, int NW>
__device__ inline bool fetch_r_coop(const DecodeArgs& a, const ProjArgs& p, uint16_t* r_lds, uint32_t* flag) {
  // (MAXP: the parts a thread loads per element; at most four for these token counts)
  if (p.ksplit <= 4) return fetch_r_coop_parts<ACT, TBK, NW, 4>(a, p, r_lds, flag);
  return fetch_r_coop_parts<ACT, TBK, NW, 8>(a, p, r_lds, flag);
}

// Folds the NW waves' fp32 tiles of one row block through LDS and stores the result.
// lds: NW * TBK * 256 floats
template <int ACT, int TBK, int NW = DEC_WAVES>
__device__ inline void decode_reduce_store(const DecodeArgs& a, const ModuleArgs& M, int rb,
                                           int wave, int lane, const float4_t (&acc)[TBK],
                                           float* lds) {
#pragma unroll
  for (int tb = 0; tb < TBK; ++tb)
#pragma unroll
    for (int v = 0; v < 4; ++v) lds[((wave * TBK + tb) * 4 + v) * 64 + lane] = acc[tb][v];
  __syncthreads();
  if (wave >= 4) return;                         // (uniform per wave; no barrier follows in here)
  const int v = wave, ln = lane;                 // 256 threads <-> (v, lane) of one token block
  const int row = rb * 16 + (ln & 15);
#pragma unroll
  for (int tb = 0; tb < TBK; ++tb) {
    const int t = 16 * tb + 4 * (ln >> 4) + v;
    if (t < a.T && row < M.d_out) {
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) s += lds[((w * TBK + tb) * 4 + v) * 64 + ln];
      const size_t off = (size_t)t * M.ldy + row;
      if (a.out_f32) ((float*)M.Y)[off] = s;
      else ((uint16_t*)M.Y)[off] = to_act16<ACT>(s);
    }
  }
}

__device__ inline const ModuleArgs& find_module(const DecodeArgs& a, int blk) {
  int mi = 0;
#pragma unroll
  for (int i = 1; i < GLOWQ_MAX_MODULES; ++i)
    if (i < a.n_modules && blk >= a.mod[i].blk_start) mi = i;
  return a.mod[mi];
}
// The scalars of a unit's descriptor, copied out of the kernel argument in one place: the
// scalar loads then go out together at the head of the kernel instead of one by one, each
// with a wait of its own, wherever a field happens to be needed first.  (mod[] is left
// out: a workgroup copies the one module it works on.)
__device__ inline DecodeArgs decode_scalars(const DecodeArgs& a) {
  DecodeArgs l;
  l.n_modules = a.n_modules;
  l.X = a.X;
  l.T = a.T;
  l.K = a.K;
  l.r = a.r;
  l.G = a.G;
  l.restore = a.restore;
  l.out_f32 = a.out_f32;
  l.ctl = a.ctl;
  return l;
}

// grp: index of the workgroup's group of DEC_RG row blocks; n_blocks: row blocks of the unit
// NW: waves of the workgroup (they take the K tiles round robin).
// lds: DEC_RG * NW * TBK * 256 floats (fold); r_lds: act dtype [16 TBK][GLOWQ_MAX_RANK];
// flag: one word; lds_af: NW * DEC_RG rows of 256 words (the A_i fragments' landing place)
template <int ACT, int TBK, int NW>
__device__ inline void decode_workgroup(const DecodeArgs& a_arg, const ProjArgs& p_arg, int grp, int n_blocks,
                                        float* lds, uint16_t* r_lds, uint32_t* flag, uint32_t* lds_af) {
  const DecodeArgs a = decode_scalars(a_arg);
  const ProjArgs p = p_arg;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int ktiles = a.K >> 7;
  const int rw = a.G == 128 ? 272 : 288;

  float4_t acc[DEC_RG][TBK];
  const uint32_t* recb[DEC_RG];
  CorrFrag cf[DEC_RG];
#pragma unroll
  for (int g = 0; g < DEC_RG; ++g) {
#pragma unroll
    for (int tb = 0; tb < TBK; ++tb) acc[g][tb] = float4_t{0.f, 0.f, 0.f, 0.f};
    // a group past the unit's last block repeats it (computed, not stored)
    const int blk = min(grp * DEC_RG + g, n_blocks - 1);
    const ModuleArgs M = find_module(a_arg, blk);
    const int rb = blk - M.blk_start;
    recb[g] = M.rec + ((size_t)rb * ktiles + wave) * rw;
    cf[g] = correction_prefetch(a, M, rb, wave, lane, lds_af + (wave * DEC_RG + g) * 256);
  }
  const bool corr = a.restore && a.r > 0;                       // uniform
  GLOWQ_WTRACE_DECL;
  GLOWQ_WSTAMP(0);
  GLOWQ_WTRACE_HWID(7);
  auto mark = [&](int done) {
    if (done == 1) GLOWQ_WSTAMP(1);
  };
  if (a.G == 128) decode_stream_rows<ACT, TBK, true, NW>(a, recb, wave, lane, acc, mark);
  else decode_stream_rows<ACT, TBK, false, NW>(a, recb, wave, lane, acc, mark);
  GLOWQ_WSTAMP(2);
  // R, once per workgroup (all row blocks of the group use the same fragments)
  u32x4_t rf[TBK];
#pragma unroll
  for (int tb = 0; tb < TBK; ++tb) rf[tb] = u32x4_t{0u, 0u, 0u, 0u};
  bool have_r = false;
  if (corr) {                                      // uniform
    // (waits for all the wave's loads)
    have_r = fetch_r_coop<ACT, TBK, NW>(a, p, r_lds, flag);
#pragma unroll
    for (int g = 0; g < DEC_RG; ++g) correction_take(cf[g], lds_af + (wave * DEC_RG + g) * 256, lane);
    if (have_r && cf[0].active && cf[0].ok) {
#pragma unroll
      for (int tb = 0; tb < TBK; ++tb) {
        const int tok = 16 * tb + (lane & 15);
        if (tok < a.T) rf[tb] = *(const u32x4_t*)(r_lds + (size_t)tok * a.r + cf[0].j0c);
      }
    }
  }
  GLOWQ_WSTAMP(3);
  // all row blocks' tiles go through LDS together: one barrier for the group
#pragma unroll
  for (int g = 0; g < DEC_RG; ++g) {
    if (cf[g].active && have_r) {
#pragma unroll
      for (int tb = 0; tb < TBK; ++tb) acc[g][tb] = mfma16<ACT>(rf[tb], cf[g].af, acc[g][tb]);
    }
#pragma unroll
    for (int tb = 0; tb < TBK; ++tb)
#pragma unroll
      for (int v = 0; v < 4; ++v) lds[(((g * NW + wave) * TBK + tb) * 4 + v) * 64 + lane] = acc[g][tb][v];
  }
  __syncthreads();
  GLOWQ_WSTAMP(4);
  if (wave < 4) {                                  // 256 threads <-> (v, lane) of one token block
#pragma unroll
    for (int g = 0; g < DEC_RG; ++g) {
      const int blk = grp * DEC_RG + g;
      if (blk >= n_blocks) break;                  // uniform
      const ModuleArgs M = find_module(a_arg, blk);
      const int v = wave;
      const int row = (blk - M.blk_start) * 16 + (lane & 15);
#pragma unroll
      for (int tb = 0; tb < TBK; ++tb) {
        const int t = 16 * tb + 4 * (lane >> 4) + v;
        if (t < a.T && row < M.d_out) {
          float s = 0.f;
#pragma unroll
          for (int w = 0; w < NW; ++w) s += lds[(((g * NW + w) * TBK + tb) * 4 + v) * 64 + lane];
          const size_t off = (size_t)t * M.ldy + row;
          if (a.out_f32) ((float*)M.Y)[off] = s;
          else ((uint16_t*)M.Y)[off] = to_act16<ACT>(s);
        }
      }
    }
  }
  GLOWQ_WSTAMP(6);
  GLOWQ_WTRACE_FLUSH();
}

// T <= 4.  lds: DEC_WAVES * 256 floats for the fold; lds_x: DEC_WAVES * DecX<TM>::WAVE_BYTES;
// lds_rf: DEC_WAVES * TM * DEC_MAX_PARTS rows of 64 words; lds_af: DEC_WAVES rows of 256 words.
template <int ACT, int TM>
__device__ inline void decode_workgroup_small(const DecodeArgs& a_arg, const ProjArgs& p_arg, int blk,
                                              float* lds, char* lds_x, uint32_t* lds_rf, uint32_t* lds_af) {
  const ModuleArgs M = find_module(a_arg, blk);      // by value, like the scalars
  const DecodeArgs a = decode_scalars(a_arg);
  const ProjArgs p = p_arg;
  const int rb = blk - M.blk_start;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

  float4_t acc[1] = {float4_t{0.f, 0.f, 0.f, 0.f}};
  GLOWQ_WTRACE_DECL;
  GLOWQ_WSTAMP(0);
  CorrFrag cf = correction_prefetch(a, M, rb, wave, lane, lds_af + wave * 256);
  RFetch rfetch;
  r_fetch_plan(a, p, cf.j0c, a.restore && cf.active && cf.ok, lane, rfetch);
  uint32_t* lds_rf_wave = lds_rf + wave * (TM * DEC_MAX_PARTS * 64);
  auto mid = [&]() {
    GLOWQ_WSTAMP(1);
    if (a.restore && cf.active) r_fetch_issue(a, p, wave, lane, lds_rf_wave);
  };
  char* lds_wave = lds_x + wave * DecX<TM>::WAVE_BYTES;
  if (a.G == 128) {
    if constexpr (TM == 1 && ACT == ACT_F16) {
      decode_stream_small<ACT, true, 1, TM, true>(a, M, rb, wave, lane, acc, lds_wave, mid);
    } else if constexpr (TM == 1) {
      decode_stream_small<ACT, true, 1, TM, false>(a, M, rb, wave, lane, acc, lds_wave, mid);
    } else {
      decode_stream_small<ACT, true, 4, TM, false>(a, M, rb, wave, lane, acc, lds_wave, mid);
    }
  } else {
    decode_stream_small<ACT, false, 4, TM, false>(a, M, rb, wave, lane, acc, lds_wave, mid);
  }
  GLOWQ_WSTAMP(2);
  if (a.restore && cf.active) {
    u32x4_t rf;
    r_fetch_take(a, p, lane, lds_rf_wave, rfetch);   // (waits for all the wave's loads)
    GLOWQ_WSTAMP(3);
    correction_take(cf, lds_af + wave * 256, lane);
    if (r_fetch_finish<ACT>(p, rfetch, rf)) acc[0] = mfma16<ACT>(rf, cf.af, acc[0]);
    GLOWQ_WSTAMP(4);
  }
  decode_reduce_store<ACT, 1>(a, M, rb, wave, lane, acc, lds);
  GLOWQ_WSTAMP(6);
  GLOWQ_WTRACE_FLUSH();
}

}  // namespace glowq
