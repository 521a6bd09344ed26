// Shared projection R = X B^T (paper Sec. 3.3, Eq. 8): computed once per unit and
// reused by every module of the unit.
//
// The contraction is split over K slices so that even a short call spreads the
// 2 r d_in bytes of B over many compute units.  Each workgroup owns one (16-token
// block, K slice): its waves take the slice's 32-channel steps round robin, multiply
// on the matrix cores straight from global memory (both operands are k-contiguous, so
// a lane's eight values are one 128-bit load), and fold their fp32 tiles through LDS
// into one partial sum; the slices are then added in slice order, so the result does
// not depend on timing.  (The decode path runs its own projection inside its launch,
// see decode.hip.)
#include "proj_device.hpp"
#include "launch.hpp"

namespace glowq {

// Stand-alone projection, used by glowq_shared_proj only (the forward kernels run their
// projection inside their own launch): a partial-sum kernel over (16-token block, K slice) followed by a reduce kernel.  Two
// plain launches instead of fences and arrival counters: at these sizes the second
// launch costs a few microseconds and every store stays an ordinary cached store.
template <int ACT>
__global__ void __launch_bounds__(256) k_proj_partial(ProjArgs a) {
  __shared__ float lds[4 * 8 * 256];
  const int tb = (int)blockIdx.x, kz = (int)blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nbs = (a.r + 15) >> 4;
  const int i = lane & 15, kq = lane >> 4;
  // tokens past T and ranks past r are computed from clamped (valid, finite) rows and
  // never stored: row i of D depends on row i of the first operand only, column n on
  // column n of the second only
  const int tok = min(tb * 16 + i, a.T - 1);
  float4_t acc[8];
#pragma unroll
  for (int nb = 0; nb < 8; ++nb) acc[nb] = float4_t{0.f, 0.f, 0.f, 0.f};
  const int k_begin = kz * a.kslice;
  const int k_end = min(a.K, k_begin + a.kslice);
  const uint16_t* xrow = a.X + (size_t)tok * a.K + 8 * kq;
  for (int k = k_begin + wave * 32; k < k_end; k += 4 * 32) {
    const u32x4_t xf = *(const u32x4_t*)(xrow + k);
#pragma unroll
    for (int nb = 0; nb < 8; ++nb) {
      if (nb < nbs) {
        const int rank = min(nb * 16 + i, a.r - 1);
        const u32x4_t bf = *(const u32x4_t*)(a.B + (size_t)rank * a.K + k + 8 * kq);
        acc[nb] = mfma16<ACT>(xf, bf, acc[nb]);   // D[token][rank]
      }
    }
  }
  // fold the four waves in one pass and store the slice's partial sums, rank fastest
#pragma unroll
  for (int nb = 0; nb < 8; ++nb)
    if (nb < nbs)
#pragma unroll
      for (int v = 0; v < 4; ++v) lds[((wave * 8 + nb) * 4 + v) * 64 + lane] = acc[nb][v];
  __syncthreads();
  for (int e = tid; e < 16 * a.r; e += 256) {
    const int tl = e / a.r, rank = e - tl * a.r;
    const int t = tb * 16 + tl;
    if (t < a.T) {
      const int nb = rank >> 4, ln = (rank & 15) + 16 * (tl >> 2), v = tl & 3;
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) s += lds[((w * 8 + nb) * 4 + v) * 64 + ln];
      a.Rpart[((size_t)kz * a.T + t) * a.r + rank] = s;
    }
  }
}

template <int ACT>
__global__ void __launch_bounds__(256) k_proj_reduce(ProjArgs a) {
  const size_t n = (size_t)a.T * a.r;
  const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= n) return;
  float s = 0.f;
  for (int z = 0; z < a.ksplit; ++z) s += a.Rpart[(size_t)z * n + e];   // slice order
  if (a.R32) a.R32[e] = s;
  if (a.R16) a.R16[e] = to_act16<ACT>(s);
}

__global__ void k_fill_zero(uint32_t* p, long long n_words) {
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_words) p[i] = 0u;
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st) {
  long long n = (long long)(bytes / 4);
  if (n == 0) return hipSuccess;
  k_fill_zero<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st>>>((uint32_t*)p, n);
  return hipGetLastError();
}

// Counts the unit slices whose status word (word 3) is nonzero.  One launch looks at up
// to STATUS_BATCH slices; `first` says whether this launch starts the count.
__global__ void k_status_count(const char* ws, StatusBatch b, int first, uint32_t* out) {
  __shared__ uint32_t n_bad;
  if (threadIdx.x == 0) n_bad = 0;
  __syncthreads();
  const int i = (int)threadIdx.x;
  if (i < b.n) {
    const uint32_t* slice = (const uint32_t*)(ws + ((size_t)b.off256[i] << 8));
    if (__hip_atomic_load(slice + 3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u)
      atomicAdd(&n_bad, 1u);
  }
  __syncthreads();
  if (threadIdx.x == 0) *out = (first ? 0u : *out) + n_bad;
}

hipError_t launch_status_count(const void* ws, const StatusBatch& b, bool first, uint32_t* out,
                               hipStream_t st) {
  k_status_count<<<dim3(1), dim3(STATUS_BATCH), 0, st>>>((const char*)ws, b, first ? 1 : 0, out);
  return hipGetLastError();
}

ProjArgs make_proj_args(const glowq_unit& u, const UnitWorkspace& ws, float* R32, bool want_r16) {
  ProjArgs a;
  a.X = (const uint16_t*)u.X;
  a.B = (const uint16_t*)u.B;
  a.T = u.T;
  a.K = u.d_in;
  a.r = u.r;
  a.ksplit = ws.ksplit;
  a.kslice = ws.kslice;
  a.Rpart = (float*)(ws.base + ws.off_rpart);
  a.R32 = R32;
  a.R16 = want_r16 ? (uint16_t*)(ws.base + ws.off_r16) : nullptr;
  a.ctl = (Control*)ws.base;
  a.groups = 1;
  return a;
}

hipError_t launch_proj(const glowq_unit& u, const UnitWorkspace& ws, float* R32, bool want_r16,
                       hipStream_t st) {
  ProjArgs a = make_proj_args(u, ws, R32, want_r16);
  // layout of the partial sums for this path: [slice][T][r]; slices as planned, but never
  // more than the partial-sum area (sized for the decode layout) can hold
  const size_t cap = (ws.off_r16 - ws.off_rpart) / ((size_t)u.T * u.r * sizeof(float));
  // (as many slices as the area holds, up to eight: the stand-alone projection has no other
  // work on the chip to hide its latency behind)
  int ksplit = cap < 8 ? (int)cap : 8;
  if (ksplit < 1) return hipErrorInvalidValue;
  const int steps = u.d_in / 32, per = (steps + ksplit - 1) / ksplit;
  a.kslice = per * 32;
  a.ksplit = (u.d_in + a.kslice - 1) / a.kslice;
  dim3 grid((unsigned)((u.T + 15) / 16), (unsigned)a.ksplit), block(256);
  const size_t n = (size_t)u.T * u.r;
  dim3 rgrid((unsigned)((n + 255) / 256));
  if (u.act_dtype == GLOWQ_F16) {
    k_proj_partial<ACT_F16><<<grid, block, 0, st>>>(a);
    k_proj_reduce<ACT_F16><<<rgrid, block, 0, st>>>(a);
  } else {
    k_proj_partial<ACT_BF16><<<grid, block, 0, st>>>(a);
    k_proj_reduce<ACT_BF16><<<rgrid, block, 0, st>>>(a);
  }
  return hipGetLastError();
}

}  // namespace glowq

GLOWQ_TRACE_EXPORT(glowq_debug_trace_proj)
