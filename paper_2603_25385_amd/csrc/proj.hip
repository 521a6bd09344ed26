// Shared projection R = X B^T (paper Sec. 3.3, Eq. 8): computed once per unit and
// reused by every module of the unit.
//
// The contraction is split over K slices so that even a one-token call spreads
// the 2 r d_in bytes of B over many compute units.  Each workgroup owns one
// (16-token block, K slice): its waves take the slice's 32-channel steps round
// robin, multiply on the matrix cores straight from global memory (both operands
// are k-contiguous, so a lane's eight values are one 128-bit load), and fold their
// fp32 tiles through LDS into one partial sum.  The workgroup that arrives last
// for a token block adds the partial sums in slice order -- the result does not
// depend on arrival order -- and writes R in fp32 and/or in the activation type.
#include "proj_device.hpp"
#include "launch.hpp"

namespace glowq {

template <int ACT>
__global__ void __launch_bounds__(256) k_proj(ProjArgs a) {
  extern __shared__ float proj_lds[];
  proj_workgroup<ACT>(a, (int)blockIdx.x, (int)blockIdx.y, proj_lds, PROJ_ALONE);
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

ProjArgs make_proj_args(const glowq_unit& u, const UnitWorkspace& ws, float* R32, bool want_r16) {
  ProjArgs a;
  a.X = (const uint16_t*)u.X;
  a.B = (const uint16_t*)u.B;
  a.T = u.T;
  a.K = u.d_in;
  a.r = u.r;
  a.ksplit = ws.ksplit;
  a.kslice = ws.kslice;
  a.kstride = ws.kstride;
  a.Rpart = (float*)(ws.base + ws.off_rpart);
  a.R32 = R32;
  a.R16 = want_r16 ? (uint16_t*)(ws.base + ws.off_r16) : nullptr;
  a.ctl = (Control*)ws.base;
  a.counters = (uint32_t*)(ws.base + ws.off_counters);
  a.tblocks = (u.T + 15) / 16;
  return a;
}

hipError_t launch_proj(const glowq_unit& u, const UnitWorkspace& ws, float* R32, bool want_r16,
                       hipStream_t st) {
  ProjArgs a = make_proj_args(u, ws, R32, want_r16);
  dim3 grid((unsigned)((u.T + 15) / 16), (unsigned)ws.ksplit), block(256);
  size_t lds = (size_t)(256 / 64) * 256 * sizeof(float);
  if (u.act_dtype == GLOWQ_F16)
    k_proj<ACT_F16><<<grid, block, lds, st>>>(a);
  else
    k_proj<ACT_BF16><<<grid, block, lds, st>>>(a);
  return hipGetLastError();
}

}  // namespace glowq

#ifdef GLOWQ_TRACE
extern "C" int glowq_debug_trace_proj(unsigned long long* host_out /* [8192][8] */) {
  return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(glowq::g_trace), sizeof(glowq::g_trace));
}
#endif
