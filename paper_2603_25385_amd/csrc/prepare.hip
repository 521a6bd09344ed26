// Weight preparation and the two inspection hooks.
//
// prepare:       canonical W4A16 arrays -> tiled layout the forward kernels read
// debug_unpack:  tiled layout -> q[d_out][d_in] bytes
// debug_dequant: tiled layout -> round_to_act((q - z) * s) through dequant_word(), the
//                library's reference dequantiser (the forward kernels schedule
//                instruction sequences of their own, checked through forward calls)
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

__device__ inline const uint32_t* tile_record(const PreparedView& v, int rb, int kb) {
  return v.base + ((size_t)rb * v.ktiles + kb) * v.rec_words;
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

hipError_t launch_prepare(const uint32_t* wq, const uint16_t* scales, const uint16_t* zeros,
                          int d_out, int d_in, int G, void* prepared, hipStream_t st) {
  long long n_words = (long long)(prepared_total_bytes(d_out, d_in, G) / 4);
  k_prepare<<<dim3((unsigned)((n_words + 255) / 256)), dim3(256), 0, st>>>(
      wq, scales, zeros, (uint32_t*)prepared, d_out, d_in, G, n_words);
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
