// Weight preparation, the two inspection hooks, and the importance scores of GlowQ-S.
//
// quantize_rtn:  fp32 weights -> canonical W4A16 arrays (round to nearest, asymmetric)
// prepare:       canonical W4A16 arrays -> tiled layout the forward kernels read
// debug_unpack:  tiled layout -> q[d_out][d_in] bytes
// debug_dequant: tiled layout -> round_to_act((q - z) * s) through dequant_word(), the
//                library's reference dequantiser (the forward kernels schedule
//                instruction sequences of their own, checked through forward calls)
// importance:    g_ner = ||E_u||^2 / ||W_u||^2 and g_ec = sum_j sigma_j^2 / ||E_u||^2 of one
//                unit (paper Sec. 3.3, Eqs. 10-11), from the full-precision weights, the
//                prepared layout and the stored factors; all sums in float64
#include "common.hpp"
#include "launch.hpp"

namespace glowq {

// one thread per word of a tile record
__global__ void k_prepare(const uint32_t* __restrict__ wq, const uint16_t* __restrict__ scales,
                          const uint16_t* __restrict__ zeros, uint32_t* __restrict__ out,
                          int d_out, int d_in, int G, long long n_words) {
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_words) return;
  const int ktiles = d_in / 128;
  const int rec_words = prepared_rec_words(G);
  const int wi = (int)(idx % rec_words);
  const long long tile = idx / rec_words;
  const int kb = (int)(tile % ktiles);
  const int rb = (int)(tile / ktiles);
  uint32_t w;
  if (wi < 256) {
    const int j = wi & 3, lane = wi >> 2;
    const int row = rb * 16 + (lane & 15);
    const int k0 = kb * 128 + 32 * j + 8 * (lane >> 4);
    uint32_t c = 0;
    if (row < d_out) c = wq[(long long)row * (d_in / 8) + k0 / 8];
    w = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      w |= ((c >> (8 * i)) & 0xFu) << (4 * i);            // e = 2i     -> nibble i
      w |= ((c >> (8 * i + 4)) & 0xFu) << (4 * i + 16);   // e = 2i + 1 -> nibble i + 4
    }
  } else {
    const int row = rb * 16 + ((wi - 256) & 15);
    const int g = kb * (128 / G) + ((wi - 256) >> 4);
    const int n_groups = d_in / G;
    w = 0x3C00u;   // s = 1, z = 0 for padding rows
    if (row < d_out)
      w = (uint32_t)scales[(long long)row * n_groups + g] |
          ((uint32_t)zeros[(long long)row * n_groups + g] << 16);
  }
  out[idx] = w;
}

// Round-to-nearest asymmetric INT4 per (row, group of G channels) (Sec. 4.1: INT4 weights,
// group size 128 or 64).  One thread per packed word (8 channels); the G / 8 threads of a
// group are neighbouring lanes.  Range widened to contain 0; s = fp16(max((hi - lo) / 15,
// 2^-14)); z = clamp(rint(-lo / s), 0, 15); q = clamp(rint(w / s) + z, 0, 15); float64
// arithmetic on the fp16-rounded s, rint to even.
__global__ void __launch_bounds__(256) k_quantize_rtn(const float* __restrict__ W, int d_out, int d_in, int G,
                                                      uint32_t* __restrict__ wq, uint16_t* __restrict__ scales,
                                                      uint16_t* __restrict__ zeros) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const int words = d_in / 8;
  // (whole waves stay in the loop-free path: the total is a multiple of 16 words per row,
  // and lanes past the end only take part in the shuffles)
  const bool live = idx < (long long)d_out * words;
  const long long row = live ? idx / words : 0;
  const int j = live ? (int)(idx - row * words) : 0;
  const float4_t* src = (const float4_t*)(W + row * d_in + 8 * j);
  const float4_t w0 = src[0], w1 = src[1];
  const float w[8] = {w0[0], w0[1], w0[2], w0[3], w1[0], w1[1], w1[2], w1[3]};
  float lo = 0.f, hi = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    lo = fminf(lo, w[e]);
    hi = fmaxf(hi, w[e]);
  }
  for (int o = 1; o < G / 8; o <<= 1) {
    lo = fminf(lo, __shfl_xor(lo, o, 64));
    hi = fmaxf(hi, __shfl_xor(hi, o, 64));
  }
  const double s = fmax(((double)hi - (double)lo) / 15.0, 0x1p-14);
  const uint32_t s_bits = act16_round<ACT_F16>(s);
  const double s_hat = act16_value<ACT_F16>(s_bits);
  const double z = fmin(fmax(__builtin_rint(-(double)lo / s_hat), 0.0), 15.0) + 0.0;   // (+0, never -0)
  uint32_t word = 0;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const double q = fmin(fmax(__builtin_rint((double)w[e] / s_hat) + z, 0.0), 15.0);
    word |= (uint32_t)q << (4 * e);
  }
  if (!live) return;
  wq[idx] = word;
  if ((j & (G / 8 - 1)) == 0) {
    const long long g = row * (d_in / G) + (8 * j) / G;
    scales[g] = (uint16_t)s_bits;
    zeros[g] = (uint16_t)act16_round<ACT_F16>(z);
  }
}

__device__ inline uint32_t load_prepared_word(const PreparedView& v, int row, int k) {
  const int lane = (row & 15) + 16 * ((k >> 3) & 3);
  const int j = (k >> 5) & 3;
  return tile_record(v, row >> 4, k >> 7)[lane * 4 + j];
}

__device__ inline uint32_t load_prepared_sz(const PreparedView& v, int row, int k, int G) {
  return tile_record(v, row >> 4, k >> 7)[256 + 16 * ((k & 127) / G) + (row & 15)];
}

// one thread per (row, 8 channels)
__global__ void k_debug_unpack(const void* prepared, int d_out, int d_in, int G,
                               uint8_t* __restrict__ q_out) {
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  int words = d_in / 8;
  if (idx >= (long long)d_out * words) return;
  int row = (int)(idx / words), k = (int)(idx % words) * 8;
  PreparedView v = prepared_view(prepared, d_out, d_in, G);
  uint32_t w = load_prepared_word(v, row, k);
  uint32_t lo = 0, hi = 0;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    lo |= prepared_nibble(w, e) << (8 * e);
    hi |= prepared_nibble(w, e + 4) << (8 * e);
  }
  uint2* dst = (uint2*)(q_out + (long long)row * d_in + k);
  *dst = make_uint2(lo, hi);
}

template <int ACT>
__global__ void k_debug_dequant(const void* prepared, int d_out, int d_in, int G,
                                uint16_t* __restrict__ w_out) {
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  int words = d_in / 8;
  if (idx >= (long long)d_out * words) return;
  int row = (int)(idx / words), k = (int)(idx % words) * 8;
  PreparedView v = prepared_view(prepared, d_out, d_in, G);
  uint32_t w = load_prepared_word(v, row, k);
  GroupConst<ACT> g;
  g.set(load_prepared_sz(v, row, k, G));
  u32x4_t d = dequant_word<ACT>(w, g);
  *(u32x4_t*)(w_out + (long long)row * d_in + k) = d;
}

// adds the block's two partial sums to out[0], out[1]
__device__ inline void block_add2(double a, double b, double* out, double* lds) {
  const int tid = threadIdx.x;
  lds[tid] = a;
  lds[blockDim.x + tid] = b;
  __syncthreads();
  for (int h = blockDim.x >> 1; h > 0; h >>= 1) {
    if (tid < h) {
      lds[tid] += lds[tid + h];
      lds[blockDim.x + tid] += lds[blockDim.x + tid + h];
    }
    __syncthreads();
  }
  if (tid == 0) {
    atomicAdd(&out[0], lds[0]);
    atomicAdd(&out[1], lds[blockDim.x]);
  }
}

// Eq. 11, numerator and denominator of one module: sums[0] += sum (W - What)^2,
// sums[1] += sum W^2, What the stored weight widened from the activation type.  One wave
// per (tile record, word index j): lane l holds row l & 15, channels 32 j + 8 (l >> 4) ..+8,
// so a wave reads 16 rows x 128 contiguous bytes of the fp32 weights (the bytes that
// matter: 4 of 4.6 per weight) and a record's four waves read its 1 KiB of words between
// them.
template <int ACT>
__global__ void __launch_bounds__(256) k_error_energy(const float* __restrict__ W, const void* prepared,
                                                      int d_out, int d_in, int G, double* sums) {
  __shared__ double lds[512];
  PreparedView v = prepared_view(prepared, d_out, d_in, G);
  const int n_rec = v.rows16 * v.ktiles;          // (below 2^31: the layout's own limit)
  const int j = threadIdx.x >> 6, lane = threadIdx.x & 63;
  double e = 0.0, ww = 0.0;
  // (a block per record, grid-stride: few blocks, so that few atomic adds meet at the two
  // sums, and the record's place is scalar arithmetic)
  for (int rec = (int)blockIdx.x; rec < n_rec; rec += (int)gridDim.x) {
    const int rb = rec / v.ktiles, kt = rec - rb * v.ktiles;
    const int row = rb * 16 + (lane & 15), k = kt * 128 + 32 * j + 8 * (lane >> 4);
    if (row >= d_out) continue;
    const uint32_t* r = tile_record(v, rb, kt);
    GroupConst<ACT> g;
    g.set(r[256 + 16 * ((k & 127) / G) + (row & 15)]);
    const u32x4_t d = dequant_word<ACT>(r[lane * 4 + j], g);
    const float4_t* src = (const float4_t*)(W + (long long)row * d_in + k);
    const float4_t w0 = __builtin_nontemporal_load(src), w1 = __builtin_nontemporal_load(src + 1);
    const float w[8] = {w0[0], w0[1], w0[2], w0[3], w1[0], w1[1], w1[2], w1[3]};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint32_t word = d[i >> 1];
      const double wh = act16_value<ACT>((i & 1) ? (word >> 16) : (word & 0xffffu));
      const double x = (double)w[i];
      e += (x - wh) * (x - wh);
      ww += x * x;
    }
  }
  block_add2(e, ww, sums, lds);
}

// col_sq[j] += sum_o A[o][j]^2 over the rows of one module (A: [d_out][r])
template <int ACT>
__global__ void __launch_bounds__(256) k_factor_col_energy(const uint16_t* __restrict__ A, int d_out, int r,
                                                           double* col_sq) {
  const int j = threadIdx.x & 127, sub = threadIdx.x >> 7;     // two rows per pass
  if (j >= r) return;
  double s = 0.0;
  for (int o = blockIdx.x * 64 + sub; o < min(d_out, (int)(blockIdx.x + 1) * 64); o += 2) {
    const double a = act16_value<ACT>(A[(long long)o * r + j]);
    s += a * a;
  }
  atomicAdd(&col_sq[j], s);
}

// row_sq[j] = sum_k B[j][k]^2 (B: [r][d_in]); one block per rank
template <int ACT>
__global__ void __launch_bounds__(256) k_factor_row_energy(const uint16_t* __restrict__ B, int d_in,
                                                           double* row_sq) {
  __shared__ double lds[512];
  const int j = blockIdx.x;
  double s = 0.0;
  for (int k = threadIdx.x; k < d_in; k += blockDim.x) {
    const double b = act16_value<ACT>(B[(long long)j * d_in + k]);
    s += b * b;
  }
  block_add2(s, 0.0, row_sq + 2 * j, lds);      // (pairs: the second sum is unused)
}

// scratch: [0] error energy, [1] weight energy, [2 .. 2 + r) column energies of A,
// [2 + 128 .. ) pairs {row energy of B, unused}.  scores[0] = g_ner, scores[1] = g_ec: the
// balanced factors have orthogonal columns / rows with ||a_j||^2 = ||b_j||^2 = sigma_j
// (Eqs. A.1.9a-b), so sum_j ||a_j||^2 ||b_j||^2 is the captured energy sum_j sigma_j^2.
__global__ void k_importance_finish(const double* scratch, int r, double* scores) {
  __shared__ double prod[GLOWQ_MAX_RANK];
  const int t = threadIdx.x;                    // one block of GLOWQ_MAX_RANK threads
  prod[t] = t < r ? scratch[2 + t] * scratch[2 + GLOWQ_MAX_RANK + 2 * t] : 0.0;
  __syncthreads();
  if (t != 0) return;
  const double e = scratch[0], w = scratch[1];
  double cap = 0.0;
  for (int j = 0; j < r; ++j) cap += prod[j];   // in rank order: the same sum every run
  scores[0] = w > 0.0 ? e / w : 0.0;
  scores[1] = e > 0.0 ? cap / e : 0.0;
}

hipError_t launch_importance(const glowq_unit& u, const float* const* W_modules, double* scratch,
                             double* scores, hipStream_t st) {
  hipError_t err = launch_fill_zero(scratch, GLOWQ_IMPORTANCE_SCRATCH_BYTES, st);
  if (err != hipSuccess) return err;
  const bool f16 = u.act_dtype == GLOWQ_F16;
  for (int i = 0; i < u.n_modules; ++i) {
    const glowq_module& m = u.modules[i];
    const long long blocks = (long long)((m.d_out + 15) / 16) * (u.d_in / 128);   // one per tile record
    dim3 grid((unsigned)(blocks < 512 ? blocks : 512)), block(256);   // (few blocks: see k_error_energy)
    if (f16) k_error_energy<ACT_F16><<<grid, block, 0, st>>>(W_modules[i], m.w_prepared, m.d_out, u.d_in, u.group_size, scratch);
    else k_error_energy<ACT_BF16><<<grid, block, 0, st>>>(W_modules[i], m.w_prepared, m.d_out, u.d_in, u.group_size, scratch);
    if (u.r > 0) {
      dim3 cgrid((unsigned)((m.d_out + 63) / 64));
      if (f16) k_factor_col_energy<ACT_F16><<<cgrid, block, 0, st>>>((const uint16_t*)m.A, m.d_out, u.r, scratch + 2);
      else k_factor_col_energy<ACT_BF16><<<cgrid, block, 0, st>>>((const uint16_t*)m.A, m.d_out, u.r, scratch + 2);
    }
  }
  if (u.r > 0) {
    if (f16) k_factor_row_energy<ACT_F16><<<dim3((unsigned)u.r), dim3(256), 0, st>>>((const uint16_t*)u.B, u.d_in, scratch + 2 + GLOWQ_MAX_RANK);
    else k_factor_row_energy<ACT_BF16><<<dim3((unsigned)u.r), dim3(256), 0, st>>>((const uint16_t*)u.B, u.d_in, scratch + 2 + GLOWQ_MAX_RANK);
  }
  k_importance_finish<<<1, GLOWQ_MAX_RANK, 0, st>>>(scratch, u.r, scores);
  return hipGetLastError();
}

hipError_t launch_prepare(const uint32_t* wq, const uint16_t* scales, const uint16_t* zeros,
                          int d_out, int d_in, int G, void* prepared, hipStream_t st) {
  long long n_words = (long long)(prepared_total_bytes(d_out, d_in, G) / 4);
  k_prepare<<<dim3((unsigned)((n_words + 255) / 256)), dim3(256), 0, st>>>(
      wq, scales, zeros, (uint32_t*)prepared, d_out, d_in, G, n_words);
  return hipGetLastError();
}

hipError_t launch_quantize_rtn(const float* W, int d_out, int d_in, int G, uint32_t* wq, uint16_t* scales,
                               uint16_t* zeros, hipStream_t st) {
  const long long n = (long long)d_out * (d_in / 8);
  k_quantize_rtn<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st>>>(W, d_out, d_in, G, wq, scales, zeros);
  return hipGetLastError();
}

hipError_t launch_debug_unpack(const void* prepared, int d_out, int d_in, int G, uint8_t* q_out,
                               hipStream_t st) {
  long long n = (long long)d_out * (d_in / 8);
  k_debug_unpack<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st>>>(prepared, d_out, d_in,
                                                                          G, q_out);
  return hipGetLastError();
}

hipError_t launch_debug_dequant(const void* prepared, int d_out, int d_in, int G, int act,
                                void* w_out, hipStream_t st) {
  long long n = (long long)d_out * (d_in / 8);
  dim3 grid((unsigned)((n + 255) / 256)), block(256);
  if (act == ACT_F16)
    k_debug_dequant<ACT_F16><<<grid, block, 0, st>>>(prepared, d_out, d_in, G, (uint16_t*)w_out);
  else
    k_debug_dequant<ACT_BF16><<<grid, block, 0, st>>>(prepared, d_out, d_in, G, (uint16_t*)w_out);
  return hipGetLastError();
}

}  // namespace glowq
