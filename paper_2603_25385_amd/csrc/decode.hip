// Decode path (T <= 32 tokens): Y_i = X dequant(W_q,i)^T + R A_i^T  (paper Eq. 9)
// in one pass over the packed weights.
//
// The work is bound by the bytes of W_q, so the kernel is organised around the
// weight stream.  One workgroup of four waves owns one 16-row block of one module
// (768 workgroups for a Llama-2-7B QKV group: three per compute unit); its waves
// take the block's 1 KiB tiles (16 rows x 128 channels) round robin, and a wave
// has the loads of eight tiles in flight before it touches the first.  A lane's
// four words of a tile are the B operands of four 16x16x32 matrix-core
// instructions; the token block of X is the A operand, so all tokens ride in the
// same instructions and the weights are read exactly once whatever T is.
//
// binary16 activations: a word is turned into eight exact values (q - z) with
// seven integer/packed operations, the products x (q - z) are exact in fp32, and
// the group scale s multiplies the per-group fp32 sum once (4 fused multiply-adds
// per tile instead of a rounding multiply per weight).  This differs from
// multiplying with the rounded 16-bit weight by at most one rounding of relative
// size 2^-11 per term, far inside the output tolerance.  bfloat16 activations use
// the rounded weight itself.
//
// The correction is r more channels of the same contraction: operand [A_i]
// against [R].  R = X B^T is produced inside the same launch: the first workgroups
// of the grid run the projection (K slices, last arrival reduces), everyone else
// streams weights in the meantime and only polls a ready counter right before the
// correction -- a kernel boundary would cost as much as the whole weight stream.
// The four waves' fp32 tiles are folded through LDS and stored.
#include "decode_device.hpp"
#include "proj_device.hpp"
#include "launch.hpp"

namespace glowq {

static_assert(GLOWQ_MAX_RANK <= DEC_WAVES * 32, "one 32-rank correction step per wave");

// Grid: [n_prod projection workgroups][one workgroup per 16-row block].
template <int ACT, int TBK>
__global__ void __launch_bounds__(DEC_WAVES * 64) k_decode(DecodeArgs a, ProjArgs p, int n_prod) {
  __shared__ float lds[DEC_WAVES * TBK * 4 * 64];
  if ((int)blockIdx.x < n_prod) {
    proj_workgroup<ACT>(p, (int)blockIdx.x / p.ksplit, (int)blockIdx.x % p.ksplit, lds, PROJ_TAG);
    return;
  }
  decode_workgroup<ACT, TBK>(a, (int)blockIdx.x - n_prod, lds);
}

template <int ACT, int TM>
__global__ void __launch_bounds__(DEC_WAVES * 64) k_decode_small(DecodeArgs a, ProjArgs p,
                                                                 int n_prod) {
  __shared__ float lds[DEC_WAVES * 4 * 64];
  __shared__ __attribute__((aligned(64))) char lds_x[DEC_WAVES * DecX<TM>::WAVE_BYTES];
  __shared__ __attribute__((aligned(16))) uint32_t lds_rf[DEC_WAVES * TM * DEC_MAX_PARTS * 64];
  if ((int)blockIdx.x < n_prod) {
    GLOWQ_STAMP(0);
    proj_wave_direct<ACT>(p, (int)blockIdx.x * DEC_WAVES + (int)(threadIdx.x >> 6),
                          (int)(threadIdx.x & 63));
    GLOWQ_STAMP(1);
    return;
  }
  decode_workgroup_small<ACT, TM>(a, p, (int)blockIdx.x - n_prod, lds, lds_x, lds_rf);
}

int fill_decode_args(const glowq_unit& u, const UnitWorkspace& ws, bool restore, DecodeArgs& a) {
  int blk = 0;
  for (int i = 0; i < u.n_modules; ++i) {
    const glowq_module& m = u.modules[i];
    PreparedView v = prepared_view(m.w_prepared, m.d_out, u.d_in, u.group_size);
    a.mod[i].rec = v.base;
    a.mod[i].A = (const uint16_t*)m.A;
    a.mod[i].Y = m.Y;
    a.mod[i].d_out = m.d_out;
    a.mod[i].ldy = m.ldy;
    a.mod[i].rows16 = v.rows16;
    a.mod[i].blk_start = blk;
    blk += v.rows16;
  }
  for (int i = u.n_modules; i < GLOWQ_MAX_MODULES; ++i) a.mod[i] = a.mod[0];
  a.n_modules = u.n_modules;
  a.X = (const uint16_t*)u.X;
  a.R16 = (const uint16_t*)(ws.base + ws.off_r16);
  a.T = u.T;
  a.K = u.d_in;
  a.r = u.r;
  a.G = u.group_size;
  a.restore = restore ? 1 : 0;
  a.out_f32 = (u.out_dtype == GLOWQ_F32) ? 1 : 0;
  return blk;
}

hipError_t launch_decode(const glowq_unit& u, const UnitWorkspace& ws, bool restore,
                         hipStream_t st) {
  DecodeArgs a;
  const int blocks = fill_decode_args(u, ws, restore, a);
  ProjArgs p = {};
  int n_prod = 0;
  a.ctl = (Control*)ws.base;
  a.in_launch_proj = 0;
  if (restore) {
    p = make_proj_args(u, ws, nullptr, true);
    const int tblocks = (u.T + 15) / 16;
    if (u.T <= DEC_SMALL_T) n_prod = (u.r * ws.ksplit + DEC_WAVES - 1) / DEC_WAVES;   // one wave per (rank, part)
    else n_prod = tblocks * ws.ksplit;
    a.in_launch_proj = 1;
  }
  dim3 grid((unsigned)(n_prod + blocks)), block(DEC_WAVES * 64);
  const bool f16 = (u.act_dtype == GLOWQ_F16);
  if (u.T <= DEC_SMALL_T) {
    // the single-token instance keeps its LDS small enough for four workgroups per
    // compute unit, so that the whole grid is resident at once
    if (u.T == 1) {
      if (f16) k_decode_small<ACT_F16, 1><<<grid, block, 0, st>>>(a, p, n_prod);
      else k_decode_small<ACT_BF16, 1><<<grid, block, 0, st>>>(a, p, n_prod);
    } else if (u.T == 2) {
      if (f16) k_decode_small<ACT_F16, 2><<<grid, block, 0, st>>>(a, p, n_prod);
      else k_decode_small<ACT_BF16, 2><<<grid, block, 0, st>>>(a, p, n_prod);
    } else {
      if (f16) k_decode_small<ACT_F16, DEC_SMALL_T><<<grid, block, 0, st>>>(a, p, n_prod);
      else k_decode_small<ACT_BF16, DEC_SMALL_T><<<grid, block, 0, st>>>(a, p, n_prod);
    }
  } else if (u.T <= 16) {
    if (f16) k_decode<ACT_F16, 1><<<grid, block, 0, st>>>(a, p, n_prod);
    else k_decode<ACT_BF16, 1><<<grid, block, 0, st>>>(a, p, n_prod);
  } else {
    if (f16) k_decode<ACT_F16, 2><<<grid, block, 0, st>>>(a, p, n_prod);
    else k_decode<ACT_BF16, 2><<<grid, block, 0, st>>>(a, p, n_prod);
  }
  return hipGetLastError();
}

}  // namespace glowq

#ifdef GLOWQ_TRACE
// stage timestamps of the decode kernels' most recent launch (tracing builds only)
extern "C" int glowq_debug_trace(unsigned long long* host_out /* [8192][8] */) {
  return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(glowq::g_trace), sizeof(glowq::g_trace));
}
#endif
