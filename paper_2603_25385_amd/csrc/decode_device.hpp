// Workgroup body of the decode path: one 16-row block of one module against up
// to 32 tokens, streamed once over the packed weights (paper Eq. 9).
#pragma once
#include "common.hpp"
#include "proj_device.hpp"
#include "../../include/glowq.h"

namespace glowq {

constexpr int DEC_WAVES = 4;
constexpr int DEC_CHUNK = 4;   // tiles per register buffer; two buffers are in flight

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
  const uint16_t* R16;
  int T, K, r, G;
  int restore, out_f32;
  // single-launch mode: the projection runs in the first workgroups of the same grid
  Control* ctl;        // control words of the unit's workspace slice
  int in_launch_proj;  // 1: wait for this launch's tag before reading R; 0: R is already
                       // in memory when the kernel starts
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
        const u32x4_t wf = q_minus_z_f16(w[j], g.nb2);
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

template <int ACT, int TBK, bool G128>
__device__ inline void decode_stream(const DecodeArgs& a, const ModuleArgs& M, int rb, int wave,
                                     int lane, float4_t (&acc)[TBK]) {
  const int n = lane & 15, kq = lane >> 4;
  const int ktiles = a.K >> 7;
  const int rw = G128 ? 272 : 288;             // words per tile record
  // this wave's tiles: kb = wave + DEC_WAVES * t, t = 0 .. ntw - 1
  const int ntw = (ktiles - wave + DEC_WAVES - 1) / DEC_WAVES;
  const uint32_t* rec0 = M.rec + ((size_t)rb * ktiles + wave) * rw;
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
      const uint32_t* rec = rec0 + (size_t)t * (DEC_WAVES * rw);
      w[c] = __builtin_nontemporal_load((const u32x4_t*)rec + lane);
      s[c][0] = __builtin_nontemporal_load(rec + 256 + n);
      if constexpr (G128) s[c][1] = s[c][0];
      else s[c][1] = __builtin_nontemporal_load(rec + 272 + n);
    }
  };
  auto run_chunk = [&](int t0, const u32x4_t (&w)[DEC_CHUNK], const uint32_t (&s)[DEC_CHUNK][2]) {
    if (t0 + DEC_CHUNK <= ntw) {
#pragma unroll
      for (int c = 0; c < DEC_CHUNK; ++c) {
        const size_t xo = (size_t)(t0 + c) * (128 * DEC_WAVES);
        decode_tile<ACT, TBK, G128>(w[c], s[c][0], s[c][1], [&](int tb, int j) {
          return *(const u32x4_t*)(xrow[tb] + xo + 32 * j); }, acc);
      }
    } else {
#pragma unroll
      for (int c = 0; c < DEC_CHUNK; ++c) {
        if (t0 + c < ntw) {
          const size_t xo = (size_t)(t0 + c) * (128 * DEC_WAVES);
          decode_tile<ACT, TBK, G128>(w[c], s[c][0], s[c][1], [&](int tb, int j) {
            return *(const u32x4_t*)(xrow[tb] + xo + 32 * j); }, acc);
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

// T <= 4: the same stream with X staged through LDS.  Each wave owns the K tiles it
// multiplies, so it also owns their slice of X: per chunk of four tiles one direct
// global->LDS load per token (64 lanes x 16 bytes = the 4 x 256 bytes of X the chunk
// needs) travels with the chunk's weight loads, and the A operands come back with
// 128-bit LDS reads (a broadcast for one token).  No workgroup barrier is involved.
constexpr int DEC_SMALL_T = 4;
constexpr int DEC_XROW = 1040;                       // bytes per token and chunk (1 KiB + pad)
constexpr int DEC_XBUF = DEC_SMALL_T * DEC_XROW;     // one chunk buffer
constexpr int DEC_XWAVE = 2 * DEC_XBUF;              // two chunk buffers per wave

// `mid` runs once, after the wave's first chunk has been consumed (or right away if the
// wave has no tiles).
template <int ACT, bool G128, int NV, class MID>
__device__ inline void decode_stream_small(const DecodeArgs& a, const ModuleArgs& M, int rb,
                                           int wave, int lane, float4_t (&acc)[1],
                                           char* lds_wave, MID mid) {
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
  const char* xrd = lds_wave + min(n, a.T - 1) * DEC_XROW + kq * 16;

  u32x4_t wA[DEC_CHUNK], wB[DEC_CHUNK];
  uint32_t sA[DEC_CHUNK][2], sB[DEC_CHUNK][2];

  auto load_chunk = [&](int t0, int buf, u32x4_t (&w)[DEC_CHUNK], uint32_t (&s)[DEC_CHUNK][2]) {
    // X first: loads return in order, and a tile needs its X before anything else
    const int tx = min(t0 + lc, ntw - 1);
    const uint16_t* src = xsrc + (size_t)tx * (128 * DEC_WAVES);
    for (int tok = 0; tok < a.T; ++tok)
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(src + (size_t)tok * a.K),
          (__attribute__((address_space(3))) void*)(lds_wave + buf * DEC_XBUF + tok * DEC_XROW),
          16, 0, 0);
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
  auto run_chunk = [&](int t0, int buf, const u32x4_t (&w)[DEC_CHUNK],
                       const uint32_t (&s)[DEC_CHUNK][2]) {
#pragma unroll
    for (int c = 0; c < DEC_CHUNK; ++c) {
      if (t0 + c < ntw) {
        const char* xc = xrd + buf * DEC_XBUF + c * 256;
        decode_tile<ACT, 1, G128, NV>(w[c], s[c][0], s[c][1], [&](int, int j) {
          return *(const u32x4_t*)(xc + 64 * j); }, acc);
      }
    }
  };

  load_chunk(0, 0, wA, sA);
  for (int t0 = 0; t0 < ntw; t0 += 2 * DEC_CHUNK) {
    if (t0 + DEC_CHUNK < ntw) load_chunk(t0 + DEC_CHUNK, 1, wB, sB);
    run_chunk(t0, 0, wA, sA);
    if (t0 == 0) mid();
    if (t0 + DEC_CHUNK < ntw) {
      if (t0 + 2 * DEC_CHUNK < ntw) load_chunk(t0 + 2 * DEC_CHUNK, 0, wA, sA);
      run_chunk(t0 + DEC_CHUNK, 1, wB, sB);
    }
  }
}

// Single-launch mode: a wave that is about to read R polls the tag that the last
// projection workgroup stores, with release semantics, once R is complete.  The tag is
// unique to the launch, so nothing has to be reset afterwards and a value left by an
// earlier launch can never be mistaken for this one's.  The projection workgroups have
// the lowest indices of the grid and never wait for anything, so the poll ends as soon
// as they have run; the loop is bounded all the same, and a wave that gives up records
// it in ctl->status and leaves the correction out rather than hang.
__device__ inline bool wait_r_ready(const DecodeArgs& a) {
  if (!a.in_launch_proj) return true;
  const unsigned long long tag = launch_tag();
  bool ok = false;
  for (int spin = 0; spin < (1 << 20); ++spin) {
    const unsigned long long v = __hip_atomic_load(&a.ctl->r_tag, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
    if (v == tag) { ok = true; break; }
    __builtin_amdgcn_s_sleep(8);
  }
  // No cache invalidation here (it would hit every wave of the grid): R is read with
  // device-coherent loads instead, see load_r16().  The compiler must not hoist them.
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
  if (!ok && (threadIdx.x & 63) == 0) atomicOr(&a.ctl->status, 1u);
  return ok;
}

// Eight 16-bit values of R read with device-scope loads: they bypass whatever this
// compute unit or this XCD's L2 may still hold for the address from an earlier call.
__device__ inline u32x4_t load_r16(const uint16_t* p) {
  const uint32_t* q = (const uint32_t*)p;
  u32x4_t v;
  v[0] = __hip_atomic_load(q + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  v[1] = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  v[2] = __hip_atomic_load(q + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  v[3] = __hip_atomic_load(q + 3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return v;
}

// Direct mode (T <= 4): every (rank, K part) wave of the projection leaves, per token,
// one 8-byte slot {partial sum, low word of its launch tag}.  The workgroup loads all
// slots of its unit (all of a thread's loads are in flight together), checks that every
// slot carries THIS launch's tag, adds the parts in part order and leaves R, rounded to
// the activation type, in LDS.  All threads of the workgroup take part.
//
// The first attempt uses ordinary (L2-cached) loads and is issued in the middle of the
// weight stream, so its latency is hidden: the projection waves publish within the first
// couple of microseconds, long before any weight chunk has been consumed, and one
// workgroup per XCD pays the miss.  A slot read too early shows an older tag; then, and
// only then, the retries use device-scope loads, which cannot be served from a stale
// cached line.  The wait is bounded (the projection waves wait for nothing, so it cannot
// expire); if it did, ctl->status is set and the correction is left out rather than hang.
struct GatherR {
  unsigned long long v[8];
  const unsigned long long* q;
  int outputs, groups, g, e, z0, z1;
  bool active, issued;
};

__device__ inline void gather_r_plan(const DecodeArgs& a, const ProjArgs& p, GatherR& st) {
  st.outputs = a.T * a.r;                               // <= 512
  st.groups = 1;
  while (st.groups * 2 * st.outputs <= DEC_WAVES * 64 && st.groups * 2 <= p.ksplit)
    st.groups *= 2;
  st.issued = false;
}

__device__ inline void gather_r_slice(const ProjArgs& p, GatherR& st, int idx) {
  const int spg = (p.ksplit + st.groups - 1) / st.groups;   // parts per group
  st.g = idx / st.outputs;
  st.e = idx - st.g * st.outputs;
  st.active = st.g < st.groups;
  st.q = (const unsigned long long*)p.Rpart + (size_t)(st.active ? st.e : 0) * p.kstride;
  st.z0 = st.active ? st.g * spg : 0;
  st.z1 = st.active ? min(p.ksplit, st.z0 + spg) : 0;
}

// issue the first (cached) attempt for this thread's first eight parts
__device__ inline void gather_r_issue(const DecodeArgs& a, const ProjArgs& p, GatherR& st) {
  if (!a.restore) return;
  gather_r_slice(p, st, threadIdx.x);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    st.v[i] = 0ull;
    if (st.z0 < st.z1)
      st.v[i] = __hip_atomic_load(st.q + min(st.z0 + i, st.z1 - 1), __ATOMIC_RELAXED,
                                  __HIP_MEMORY_SCOPE_WORKGROUP);
  }
  st.issued = true;
}

// lds_f: 512 floats of scratch; lds_r: T * r 16-bit values
template <int ACT>
__device__ inline bool gather_r_finish(const DecodeArgs& a, const ProjArgs& p, GatherR& st,
                                       float* lds_f, uint16_t* lds_r) {
  const int tid = threadIdx.x;
  const uint32_t tag = (uint32_t)(launch_tag() & 0xffffffffull);
  const int passes = (st.outputs + DEC_WAVES * 64 - 1) / (DEC_WAVES * 64);   // 2 only if groups == 1
  for (int pass = 0; pass < passes; ++pass) {
    gather_r_slice(p, st, tid + pass * DEC_WAVES * 64);
    const bool use_prefetch = st.issued && pass == 0;
    float s = 0.f;
    bool done = false;
    for (int spin = 0; spin < (1 << 14); ++spin) {
      bool ok = true;
      s = 0.f;
      for (int zb = st.z0; zb < st.z1; zb += 8) {
        unsigned long long v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const unsigned long long* qi = st.q + min(zb + i, st.z1 - 1);
          if (spin == 0 && use_prefetch && zb == st.z0) v[i] = st.v[i];
          else if (spin == 0)
            v[i] = __hip_atomic_load(qi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
          else v[i] = __hip_atomic_load(qi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          if (zb + i < st.z1) {
            ok = ok && ((uint32_t)(v[i] >> 32) == tag);
            s += __builtin_bit_cast(float, (uint32_t)v[i]);
          }
        }
      }
      if (__syncthreads_and(ok ? 1 : 0)) { done = true; break; }
      __builtin_amdgcn_s_sleep(32);
    }
    if (!done) {
      if (tid == 0) atomicOr(&p.ctl->status, 1u);
      return false;
    }
    if (st.active) {
      if (st.groups == 1) lds_r[st.e] = to_act16<ACT>(s);
      else lds_f[st.g * st.outputs + st.e] = s;
    }
  }
  __syncthreads();
  if (st.groups > 1) {
    if (tid < st.outputs) {
      float s = 0.f;
      for (int g = 0; g < st.groups; ++g) s += lds_f[g * st.outputs + tid];
      lds_r[tid] = to_act16<ACT>(s);
    }
    __syncthreads();
  }
  return true;
}

// A_i fragments of this wave's correction steps (32 ranks each; wave w takes steps
// w, w + 4, ...: at most one step per wave up to rank 128).  Loaded before the weight
// stream so that their latency is hidden behind it.
struct CorrFrag {
  u32x4_t af;
  int j0c;
  bool active, ok;
};
__device__ inline CorrFrag correction_prefetch(const DecodeArgs& a, const ModuleArgs& M, int rb,
                                               int wave, int lane) {
  CorrFrag c;
  const int n = lane & 15, kq = lane >> 4;
  c.active = a.restore && wave * 32 < a.r;
  const int j0 = wave * 32 + 8 * kq;
  c.ok = j0 < a.r;                          // ranks past r contribute zeros on both sides
  c.j0c = c.ok ? j0 : 0;
  c.af = u32x4_t{0u, 0u, 0u, 0u};
  if (c.active) {
    const int row = min(rb * 16 + n, M.d_out - 1);
    c.af = *(const u32x4_t*)(M.A + (size_t)row * a.r + c.j0c);
    if (!c.ok) c.af = u32x4_t{0u, 0u, 0u, 0u};
  }
  return c;
}

// Correction R A_i^T as r more channels of the contraction.
template <int ACT, int TBK>
__device__ inline void decode_correction(const DecodeArgs& a, const CorrFrag& c, int lane,
                                         float4_t (&acc)[TBK]) {
  if (!c.active) return;
  if (!wait_r_ready(a)) return;
  const int n = lane & 15;
#pragma unroll
  for (int tb = 0; tb < TBK; ++tb) {
    const int tok = min(16 * tb + n, a.T - 1);
    u32x4_t rf = load_r16(a.R16 + (size_t)tok * a.r + c.j0c);
    if (!c.ok) rf = u32x4_t{0u, 0u, 0u, 0u};
    acc[tb] = mfma16<ACT>(rf, c.af, acc[tb]);
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

  const CorrFrag cf = correction_prefetch(a, M, rb, wave, lane);
  if (a.G == 128) decode_stream<ACT, TBK, true>(a, M, rb, wave, lane, acc);
  else decode_stream<ACT, TBK, false>(a, M, rb, wave, lane, acc);
  decode_correction<ACT, TBK>(a, cf, lane, acc);
  decode_reduce_store<ACT, TBK>(a, M, rb, wave, lane, acc, lds);
}

// T <= 4.  lds: DEC_WAVES * 256 floats for the fold; lds_x: DEC_WAVES * DEC_XWAVE bytes;
// lds_r: DEC_SMALL_T * GLOWQ_MAX_RANK 16-bit values.
template <int ACT>
__device__ inline void decode_workgroup_small(const DecodeArgs& a, const ProjArgs& p, int blk,
                                              float* lds, char* lds_x, uint16_t* lds_r) {
  const ModuleArgs& M = find_module(a, blk);
  const int rb = blk - M.blk_start;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

  float4_t acc[1] = {float4_t{0.f, 0.f, 0.f, 0.f}};
  GLOWQ_STAMP(0);
#ifdef GLOWQ_TRACE
  if (threadIdx.x == 0 && blockIdx.x < 8192) {
    unsigned hw = __builtin_amdgcn_s_getreg((4 << 0) | (0 << 6) | (31 << 11));    // HW_ID
    unsigned xcc = __builtin_amdgcn_s_getreg((20 << 0) | (0 << 6) | (31 << 11));  // XCC_ID
    g_trace[blockIdx.x][7] = ((unsigned long long)xcc << 32) | hw;
  }
#endif
  const CorrFrag cf = correction_prefetch(a, M, rb, wave, lane);
  GatherR gr;
  gather_r_plan(a, p, gr);
  auto mid = [&]() { gather_r_issue(a, p, gr); };
  char* lds_wave = lds_x + wave * DEC_XWAVE;
  if (a.G == 128) {
    if (a.T == 1) decode_stream_small<ACT, true, 1>(a, M, rb, wave, lane, acc, lds_wave, mid);
    else decode_stream_small<ACT, true, 4>(a, M, rb, wave, lane, acc, lds_wave, mid);
  } else {
    decode_stream_small<ACT, false, 4>(a, M, rb, wave, lane, acc, lds_wave, mid);
  }
  GLOWQ_STAMP(1);
  if (a.restore) {
    const bool got = gather_r_finish<ACT>(a, p, gr, lds, lds_r);
    GLOWQ_STAMP(3);
    if (got && cf.active) {
      const int tok = min(lane & 15, a.T - 1);
      u32x4_t rf = *(const u32x4_t*)(lds_r + tok * a.r + cf.j0c);
      if (!cf.ok) rf = u32x4_t{0u, 0u, 0u, 0u};
      acc[0] = mfma16<ACT>(rf, cf.af, acc[0]);
    }
  }
  decode_reduce_store<ACT, 1>(a, M, rb, wave, lane, acc, lds);
  GLOWQ_STAMP(4);
}

}  // namespace glowq
