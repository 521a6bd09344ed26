// Decode path (T <= 32 tokens): Y_i = X dequant(W_q,i)^T + R A_i^T  (paper Eq. 9)
// in one pass over the packed weights.
//
// The work is bound by the bytes of W_q, so the kernel is organised around the
// weight stream: one workgroup owns one 32-row block of one module, its eight
// waves take that block's 1 KiB tiles round robin, and each wave issues the loads
// of all its tiles before it touches any of them, so that the whole unit is in
// flight at once.  A lane's four words of a tile are dequantised in registers and
// go to the matrix cores as the B operand (32 rows x 16 channels per instruction)
// against the token block of X as the A operand; all tokens ride in the same
// instruction, so the weights are read exactly once whatever T is.  The
// correction is r more channels of the same contraction: operand [What | A_i]
// against [X ; R], with R already reduced by the projection.  The eight waves'
// fp32 tiles are folded through LDS and stored.
#include "common.hpp"
#include "launch.hpp"

namespace glowq {

constexpr int DEC_WAVES = 8;
constexpr int DEC_CHUNK = 8;   // tiles a wave keeps in flight

struct ModuleArgs {
  const u32x4_t* tiles;
  const uint32_t* sz;
  const uint16_t* A;
  void* Y;
  int d_out, ldy, rows32, blk_start;
};

struct DecodeArgs {
  ModuleArgs mod[GLOWQ_MAX_MODULES];
  int n_modules;
  const uint16_t* X;
  const uint16_t* R16;
  int T, K, r, G;
  int restore, out_f32;
};

template <int ACT>
__device__ inline void decode_workgroup(const DecodeArgs& a, int blk, float* lds) {
  int mi = 0;
#pragma unroll
  for (int i = 1; i < GLOWQ_MAX_MODULES; ++i)
    if (i < a.n_modules && blk >= a.mod[i].blk_start) mi = i;
  const ModuleArgs& M = a.mod[mi];
  const int rb = blk - M.blk_start;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m = lane & 31, h = lane >> 5;
  const int ktiles = a.K >> 6;
  const int rows_pad = M.rows32 * 32;
  const bool tok_ok = m < a.T;
  const uint16_t* xrow = a.X + (size_t)m * a.K + 32 * h;
  const u32x4_t* tile0 = M.tiles + (size_t)rb * ktiles * 64 + lane;
  const uint32_t* sz0 = M.sz + rb * 32 + m;
  const int gshift = (a.G == 128) ? 1 : 0;   // tiles per group, log2

  float16_t acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;

  for (int base = wave; base < ktiles; base += DEC_WAVES * DEC_CHUNK) {
    u32x4_t wreg[DEC_CHUNK];
    uint32_t szw[DEC_CHUNK];
#pragma unroll
    for (int c = 0; c < DEC_CHUNK; ++c) {
      const int kb = base + c * DEC_WAVES;
      wreg[c] = u32x4_t{0u, 0u, 0u, 0u};
      szw[c] = 0x3C00u;
      if (kb < ktiles) {
        wreg[c] = __builtin_nontemporal_load(tile0 + (size_t)kb * 64);
        szw[c] = sz0[(size_t)(kb >> gshift) * rows_pad];
      }
    }
#pragma unroll
    for (int c = 0; c < DEC_CHUNK; ++c) {
      const int kb = base + c * DEC_WAVES;
      if (kb < ktiles) {
        u32x4_t xf[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          xf[j] = u32x4_t{0u, 0u, 0u, 0u};
          if (tok_ok) xf[j] = *(const u32x4_t*)(xrow + kb * 64 + 8 * j);
        }
        GroupConst<ACT> g;
        g.set(szw[c]);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          u32x4_t wf = dequant_word<ACT>(wreg[c][j], g);
          acc = mfma32<ACT>(xf[j], wf, acc);   // D[token][row]
        }
      }
    }
  }

  // correction: r more channels, operand [A_i] against [R]
  if (a.restore) {
    const int row = rb * 32 + m;
    for (int jj = wave; jj * 16 < a.r; jj += DEC_WAVES) {
      const int j0 = jj * 16 + 8 * h;
      u32x4_t rf = {0u, 0u, 0u, 0u}, af = {0u, 0u, 0u, 0u};
      if (j0 < a.r) {
        if (tok_ok) rf = *(const u32x4_t*)(a.R16 + (size_t)m * a.r + j0);
        if (row < M.d_out) af = *(const u32x4_t*)(M.A + (size_t)row * a.r + j0);
      }
      acc = mfma32<ACT>(rf, af, acc);
    }
  }

  // fold the eight waves' tiles and store
#pragma unroll
  for (int i = 0; i < 16; ++i) lds[(wave * 16 + i) * 64 + lane] = acc[i];
  __syncthreads();
  for (int o = tid; o < 1024; o += DEC_WAVES * 64) {
    const int i = o >> 6, ln = o & 63;
    const int t = 8 * (i >> 2) + 4 * (ln >> 5) + (i & 3);
    const int row = rb * 32 + (ln & 31);
    if (t < a.T && row < M.d_out) {
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < DEC_WAVES; ++w) s += lds[(w * 16 + i) * 64 + ln];
      const size_t off = (size_t)t * M.ldy + row;
      if (a.out_f32) ((float*)M.Y)[off] = s;
      else ((uint16_t*)M.Y)[off] = to_act16<ACT>(s);
    }
  }
}

template <int ACT>
__global__ void __launch_bounds__(DEC_WAVES * 64) k_decode(DecodeArgs a) {
  __shared__ float lds[DEC_WAVES * 16 * 64];
  decode_workgroup<ACT>(a, (int)blockIdx.x, lds);
}

hipError_t launch_decode(const glowq_unit& u, const UnitWorkspace& ws, bool restore,
                         hipStream_t st) {
  DecodeArgs a;
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
    a.mod[i].rows32 = v.rows32;
    a.mod[i].blk_start = blk;
    blk += v.rows32;
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
  dim3 grid((unsigned)blk), block(DEC_WAVES * 64);
  if (u.act_dtype == GLOWQ_F16)
    k_decode<ACT_F16><<<grid, block, 0, st>>>(a);
  else
    k_decode<ACT_BF16><<<grid, block, 0, st>>>(a);
  return hipGetLastError();
}

}  // namespace glowq
