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
// against [R], with R already reduced by the projection.  The four waves' fp32
// tiles are folded through LDS and stored.
#include "decode_device.hpp"
#include "launch.hpp"

namespace glowq {

template <int ACT, int TBK>
__global__ void __launch_bounds__(DEC_WAVES * 64) k_decode(DecodeArgs a) {
  __shared__ float lds[DEC_WAVES * TBK * 4 * 64];
  decode_workgroup<ACT, TBK>(a, (int)blockIdx.x, lds);
}

int fill_decode_args(const glowq_unit& u, const UnitWorkspace& ws, bool restore, DecodeArgs& a) {
  int blk = 0;
  for (int i = 0; i < u.n_modules; ++i) {
    const glowq_module& m = u.modules[i];
    PreparedView v = prepared_view(m.w_prepared, m.d_out, u.d_in);
    a.mod[i].tiles = v.tiles;
    a.mod[i].sz = v.sz;
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
  dim3 grid((unsigned)blocks), block(DEC_WAVES * 64);
  const bool f16 = (u.act_dtype == GLOWQ_F16);
  if (u.T <= 16) {
    if (f16) k_decode<ACT_F16, 1><<<grid, block, 0, st>>>(a);
    else k_decode<ACT_BF16, 1><<<grid, block, 0, st>>>(a);
  } else {
    if (f16) k_decode<ACT_F16, 2><<<grid, block, 0, st>>>(a);
    else k_decode<ACT_BF16, 2><<<grid, block, 0, st>>>(a);
  }
  return hipGetLastError();
}

}  // namespace glowq
