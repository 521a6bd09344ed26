// Workgroup body of the decode path: one 16-row block of one module against up
// to 32 tokens, streamed once over the packed weights (paper Eq. 9).
#pragma once
#include "common.hpp"
#include "../../include/glowq.h"

namespace glowq {

constexpr int DEC_WAVES = 4;
constexpr int DEC_CHUNK = 4;   // tiles per register buffer; two buffers are in flight

struct ModuleArgs {
  const u32x4_t* tiles;
  const uint32_t* sz;
  const uint16_t* A;
  void* Y;
  int d_out, ldy, rows16, blk_start;
};

struct DecodeArgs {
  ModuleArgs mod[GLOWQ_MAX_MODULES];
  int n_modules;
  const uint16_t* X;
  const uint16_t* R16;
  int T, K, r, G;
  int restore, out_f32;
};

// One tile (16 rows x 128 channels) against TBK blocks of 16 tokens.
// sz0 / sz1: the (s, z) words of the tile's first and second 64 channels (equal
// when the quantisation group is 128 wide).
template <int ACT, int TBK, bool G128>
__device__ inline void decode_tile(const u32x4_t w, uint32_t sz0, uint32_t sz1,
                                   const uint16_t* const (&xk)[TBK], float4_t (&acc)[TBK]) {
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
        const u32x4_t wf = q_minus_z_f16(w[j], g.nb2);
#pragma unroll
        for (int tb = 0; tb < TBK; ++tb) {
          const u32x4_t xf = *(const u32x4_t*)(xk[tb] + 32 * j);
          if (jj == 0) tmp[tb] = mfma16<ACT>(xf, wf, float4_t{0.f, 0.f, 0.f, 0.f});
          else tmp[tb] = mfma16<ACT>(xf, wf, tmp[tb]);   // D[token][row]
        }
      }
#pragma unroll
      for (int tb = 0; tb < TBK; ++tb)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[tb][v] = __builtin_fmaf(s, tmp[tb][v], acc[tb][v]);
    }
  } else {
    GroupConst<ACT> g0, g1;
    g0.set(sz0);
    g1.set(sz1);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const u32x4_t wf = dequant_word<ACT>(w[j], (G128 || j < 2) ? g0 : g1);
#pragma unroll
      for (int tb = 0; tb < TBK; ++tb) {
        const u32x4_t xf = *(const u32x4_t*)(xk[tb] + 32 * j);
        acc[tb] = mfma16<ACT>(xf, wf, acc[tb]);
      }
    }
  }
}

template <int ACT, int TBK, bool G128>
__device__ inline void decode_stream(const DecodeArgs& a, const ModuleArgs& M, int rb, int wave,
                                     int lane, float4_t (&acc)[TBK]) {
  const int n = lane & 15, kq = lane >> 4;
  const int ktiles = a.K >> 7;
  const int rows_pad = M.rows16 * 16;
  // this wave's tiles: kb = wave + DEC_WAVES * t, t = 0 .. ntw - 1
  const int ntw = (ktiles - wave + DEC_WAVES - 1) / DEC_WAVES;
  const u32x4_t* tile0 = M.tiles + ((size_t)rb * ktiles + wave) * 64 + lane;
  const uint32_t* szp = M.sz + rb * 16 + n;
  // tokens past T read the last valid token: their rows of D are never stored
  const uint16_t* xrow[TBK];
#pragma unroll
  for (int tb = 0; tb < TBK; ++tb)
    xrow[tb] = a.X + (size_t)min(16 * tb + n, a.T - 1) * a.K + 8 * kq + 128 * wave;

  u32x4_t wA[DEC_CHUNK], wB[DEC_CHUNK];
  uint32_t sA[DEC_CHUNK][2], sB[DEC_CHUNK][2];

  auto load_chunk = [&](int t0, u32x4_t (&w)[DEC_CHUNK], uint32_t (&s)[DEC_CHUNK][2]) {
#pragma unroll
    for (int c = 0; c < DEC_CHUNK; ++c) {
      const int t = min(t0 + c, ntw - 1);          // clamped: a duplicate tile is never used
      const int kb = wave + DEC_WAVES * t;
      w[c] = __builtin_nontemporal_load(tile0 + (size_t)t * (DEC_WAVES * 64));
      if constexpr (G128) {
        s[c][0] = szp[(size_t)kb * rows_pad];
        s[c][1] = s[c][0];
      } else {
        s[c][0] = szp[(size_t)(2 * kb) * rows_pad];
        s[c][1] = szp[(size_t)(2 * kb + 1) * rows_pad];
      }
    }
  };
  auto run_chunk = [&](int t0, const u32x4_t (&w)[DEC_CHUNK], const uint32_t (&s)[DEC_CHUNK][2]) {
    if (t0 + DEC_CHUNK <= ntw) {
#pragma unroll
      for (int c = 0; c < DEC_CHUNK; ++c) {
        const uint16_t* xk[TBK];
#pragma unroll
        for (int tb = 0; tb < TBK; ++tb) xk[tb] = xrow[tb] + (size_t)(t0 + c) * (128 * DEC_WAVES);
        decode_tile<ACT, TBK, G128>(w[c], s[c][0], s[c][1], xk, acc);
      }
    } else {
#pragma unroll
      for (int c = 0; c < DEC_CHUNK; ++c) {
        if (t0 + c < ntw) {
          const uint16_t* xk[TBK];
#pragma unroll
          for (int tb = 0; tb < TBK; ++tb)
            xk[tb] = xrow[tb] + (size_t)(t0 + c) * (128 * DEC_WAVES);
          decode_tile<ACT, TBK, G128>(w[c], s[c][0], s[c][1], xk, acc);
        }
      }
    }
  };

  if (ntw <= 0) return;
  load_chunk(0, wA, sA);
  for (int t0 = 0; t0 < ntw; t0 += 2 * DEC_CHUNK) {
    if (t0 + DEC_CHUNK < ntw) load_chunk(t0 + DEC_CHUNK, wB, sB);
    run_chunk(t0, wA, sA);
    if (t0 + DEC_CHUNK < ntw) {
      if (t0 + 2 * DEC_CHUNK < ntw) load_chunk(t0 + 2 * DEC_CHUNK, wA, sA);
      run_chunk(t0 + DEC_CHUNK, wB, sB);
    }
  }
}

// Correction R A_i^T as r more channels; wave w takes the 32-rank steps w, w + 4, ...
template <int ACT, int TBK>
__device__ inline void decode_correction(const DecodeArgs& a, const ModuleArgs& M, int rb,
                                         int wave, int lane, float4_t (&acc)[TBK]) {
  const int n = lane & 15, kq = lane >> 4;
  const int row = min(rb * 16 + n, M.d_out - 1);
  for (int jj = wave; jj * 32 < a.r; jj += DEC_WAVES) {
    const int j0 = jj * 32 + 8 * kq;
    const bool ok = j0 < a.r;                 // ranks past r contribute zeros on both sides
    const int j0c = ok ? j0 : 0;
    u32x4_t af = *(const u32x4_t*)(M.A + (size_t)row * a.r + j0c);
    if (!ok) af = u32x4_t{0u, 0u, 0u, 0u};
#pragma unroll
    for (int tb = 0; tb < TBK; ++tb) {
      const int tok = min(16 * tb + n, a.T - 1);
      u32x4_t rf = *(const u32x4_t*)(a.R16 + (size_t)tok * a.r + j0c);
      if (!ok) rf = u32x4_t{0u, 0u, 0u, 0u};
      acc[tb] = mfma16<ACT>(rf, af, acc[tb]);
    }
  }
}

// lds: DEC_WAVES * TBK * 256 floats
template <int ACT, int TBK>
__device__ inline void decode_reduce_store(const DecodeArgs& a, const ModuleArgs& M, int rb,
                                           int wave, int lane, const float4_t (&acc)[TBK],
                                           float* lds) {
#pragma unroll
  for (int tb = 0; tb < TBK; ++tb)
#pragma unroll
    for (int v = 0; v < 4; ++v) lds[((wave * TBK + tb) * 4 + v) * 64 + lane] = acc[tb][v];
  __syncthreads();
  const int v = wave, ln = lane;                 // 256 threads <-> (v, lane) of one token block
  const int row = rb * 16 + (ln & 15);
#pragma unroll
  for (int tb = 0; tb < TBK; ++tb) {
    const int t = 16 * tb + 4 * (ln >> 4) + v;
    if (t < a.T && row < M.d_out) {
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < DEC_WAVES; ++w) s += lds[((w * TBK + tb) * 4 + v) * 64 + ln];
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

template <int ACT, int TBK>
__device__ inline void decode_workgroup(const DecodeArgs& a, int blk, float* lds) {
  const ModuleArgs& M = find_module(a, blk);
  const int rb = blk - M.blk_start;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

  float4_t acc[TBK];
#pragma unroll
  for (int tb = 0; tb < TBK; ++tb) acc[tb] = float4_t{0.f, 0.f, 0.f, 0.f};

  if (a.G == 128) decode_stream<ACT, TBK, true>(a, M, rb, wave, lane, acc);
  else decode_stream<ACT, TBK, false>(a, M, rb, wave, lane, acc);
  if (a.restore) decode_correction<ACT, TBK>(a, M, rb, wave, lane, acc);
  decode_reduce_store<ACT, TBK>(a, M, rb, wave, lane, acc, lds);
}

}  // namespace glowq
