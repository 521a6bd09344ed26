// Workgroup body of the shared projection R = X B^T (paper Sec. 3.3, Eq. 8).
// Used by the stand-alone projection kernel and, as the producer role, by the
// single-launch decode kernel.
#pragma once
#include "common.hpp"

namespace glowq {

struct ProjArgs {
  const uint16_t* X;   // act dtype [T][K]
  const uint16_t* B;   // act dtype [r][K]
  int T, K, r;
  int ksplit;          // K slices
  int kslice;          // channels per slice, multiple of 32
  float* Rpart;        // stand-alone projection: fp32 [slice][T][r]; in-launch projection
                       // of the decode kernels: 8-byte slots {fp32 bits, launch tag}
  float* R32;          // optional fp32 [T][r]
  uint16_t* R16;       // optional act dtype [T][r]
  Control* ctl;        // control words of the unit's workspace slice
  int groups;          // in-launch projection of 5 to 32 tokens: workgroups that share a K
                       // slice, each with its own run of 16-rank blocks (1 or 2)
};

// One workgroup = (16-token block tb, K slice kz, group ng of the slice's 16-rank blocks);
// any whole number of waves.
// lds: blockDim.x / 64 * 256 floats.
// No reduction here: every partial sum is published as one 8-byte device-scope store
// {fp32 bits, low word of the launch tag}, slot (t, kz, j) = slots[(t ksplit + kz) r + j],
// and the consumers add the slices (no fence, no counter, nothing to wait for).
template <int ACT>
__device__ inline void proj_workgroup(const ProjArgs& a, int tb, int kz, int ng, float* lds) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;
  const int nbs = (a.r + 15) >> 4;
  const int nb_per = (nbs + a.groups - 1) / a.groups;
  const int nb0 = ng * nb_per, nb1 = min(nbs, nb0 + nb_per);      // this workgroup's rank blocks
  const int i = lane & 15, kq = lane >> 4;
  // tokens past T and ranks past r are computed from clamped (valid, finite) rows and
  // never stored: row i of D depends on row i of the first operand only, column n on
  // column n of the second only
  const int tok = min(tb * 16 + i, a.T - 1);

  float4_t acc[8];
#pragma unroll
  for (int nb = 0; nb < 8; ++nb) acc[nb] = float4_t{0.f, 0.f, 0.f, 0.f};
  GLOWQ_STAMP(0);

  const int k_begin = kz * a.kslice;
  const int k_end = min(a.K, k_begin + a.kslice);
  const uint16_t* xrow = a.X + (size_t)tok * a.K + 8 * kq;
  // steps of 32 channels, interleaved over the waves; the loads of PB steps are in
  // flight together (a step past the end re-reads the first one and multiplies by zero)
  constexpr int PB = 4;
  for (int k0 = k_begin + wave * 32; k0 < k_end; k0 += PB * nw * 32) {
    u32x4_t xf[PB], bf[PB][8];
#pragma unroll
    for (int s = 0; s < PB; ++s) {
      const int k = k0 + s * nw * 32;
      const bool in = k < k_end;
      const int kc = in ? k : k0;
      xf[s] = *(const u32x4_t*)(xrow + kc);
      if (!in) xf[s] = u32x4_t{0u, 0u, 0u, 0u};
#pragma unroll
      for (int nb = 0; nb < 8; ++nb) {
        if (nb >= nb0 && nb < nb1) {
          const int rank = min(nb * 16 + i, a.r - 1);
          bf[s][nb] = *(const u32x4_t*)(a.B + (size_t)rank * a.K + kc + 8 * kq);
        }
      }
    }
#pragma unroll
    for (int s = 0; s < PB; ++s)
#pragma unroll
      for (int nb = 0; nb < 8; ++nb)
        if (nb >= nb0 && nb < nb1) acc[nb] = mfma16<ACT>(xf[s], bf[s][nb], acc[nb]);   // D[token][rank]
  }

  GLOWQ_STAMP(1);
  // fold the waves' tiles and store this slice's partial sum
#pragma unroll
  for (int nb = 0; nb < 8; ++nb) {
    if (nb >= nb0 && nb < nb1) {
#pragma unroll
      for (int v = 0; v < 4; ++v) lds[(wave * 4 + v) * 64 + lane] = acc[nb][v];
      __syncthreads();
      for (int o = tid; o < 256; o += blockDim.x) {
        const int v = o >> 6, ln = o & 63;
        float s = 0.f;
        for (int w = 0; w < nw; ++w) s += lds[(w * 4 + v) * 64 + ln];
        const int t = tb * 16 + 4 * (ln >> 4) + v;
        const int rank = nb * 16 + (ln & 15);
        if (t < a.T && rank < a.r) {
          const unsigned long long tag_hi = (launch_tag() & 0xffffffffull) << 32;
          __hip_atomic_store((unsigned long long*)a.Rpart + ((size_t)t * a.ksplit + kz) * a.r + rank,
                             tag_hi | (unsigned long long)__builtin_bit_cast(uint32_t, s),
                             __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
      __syncthreads();
    }
  }
  GLOWQ_STAMP(2);
}

// Projection for a handful of tokens (T <= 4), built for the shortest dependency chain:
// one WAVE computes, for one rank j and one of `ksplit` K parts, the T partial sums
// sum_k X[t][k] B[j][k] -- contiguous reads of B and X, all of a batch in flight
// together, fp32 accumulation, a butterfly reduction -- and publishes each as ONE 8-byte
// device-scope store {fp32 bits, low word of the launch tag}.  A slot therefore
// validates itself: no fence, no flag, no ordering between stores, and the wave never
// waits for anything.  The consumers add the parts (r_fetch_finish).  Slot of
// (t, part, j): slots[(t ksplit + part) r + j].
template <int ACT>
__device__ inline void proj_wave_direct(const ProjArgs& a, int wave_global, int lane) {
  const int rank = wave_global % a.r, part = wave_global / a.r;   // a workgroup shares a part
  if (part >= a.ksplit) return;
  const int k_begin = part * a.kslice;
  const int k_end = min(a.K, k_begin + a.kslice);
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  const uint16_t* brow = a.B + (size_t)rank * a.K;
  constexpr int BATCH = 4;   // 512-channel steps whose loads are in flight together
  for (int k0 = k_begin + 8 * lane; k0 < k_end; k0 += 512 * BATCH) {
    u32x4_t bv[BATCH], xv[4][BATCH];
#pragma unroll
    for (int it = 0; it < BATCH; ++it) {
      const int k = k0 + 512 * it;
      const bool in = k < k_end;
      const int kc = in ? k : k0;                     // clamped: loaded again, not used
      bv[it] = *(const u32x4_t*)(brow + kc);
      if (!in) bv[it] = u32x4_t{0u, 0u, 0u, 0u};
#pragma unroll
      for (int t = 0; t < 4; ++t)
        if (t < a.T) xv[t][it] = *(const u32x4_t*)(a.X + (size_t)t * a.K + kc);
    }
#pragma unroll
    for (int it = 0; it < BATCH; ++it) {
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        if (t < a.T) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const uint32_t bw = bv[it][i], xw = xv[t][it][i];
            float b0, b1, x0, x1;
            if constexpr (ACT == ACT_F16) {
              b0 = (float)__builtin_bit_cast(_Float16, (uint16_t)(bw & 0xffffu));
              b1 = (float)__builtin_bit_cast(_Float16, (uint16_t)(bw >> 16));
              x0 = (float)__builtin_bit_cast(_Float16, (uint16_t)(xw & 0xffffu));
              x1 = (float)__builtin_bit_cast(_Float16, (uint16_t)(xw >> 16));
            } else {
              b0 = __builtin_bit_cast(float, bw << 16);
              b1 = __builtin_bit_cast(float, bw & 0xffff0000u);
              x0 = __builtin_bit_cast(float, xw << 16);
              x1 = __builtin_bit_cast(float, xw & 0xffff0000u);
            }
            acc[t] = __builtin_fmaf(b0, x0, acc[t]);
            acc[t] = __builtin_fmaf(b1, x1, acc[t]);
          }
        }
      }
    }
  }
  const unsigned long long tag_hi = (launch_tag() & 0xffffffffull) << 32;
  unsigned long long* slots = (unsigned long long*)a.Rpart;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    if (t < a.T) {
      float s = acc[t];
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
      if (lane == 0)
        __hip_atomic_store(&slots[((size_t)t * a.ksplit + part) * a.r + rank],
                           tag_hi | (unsigned long long)__builtin_bit_cast(uint32_t, s),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

}  // namespace glowq
