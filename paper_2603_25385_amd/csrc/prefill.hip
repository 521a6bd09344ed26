// Prefill path (T > 32 tokens): Y_i = X dequant(W_q,i)^T + R A_i^T  (paper Eq. 9)
// as a tiled matrix-core GEMM with the correction folded in as r extra channels.
//
// Workgroup tile: (32 MB) tokens x 256 rows, four waves, each wave 64 rows x all
// tokens of the tile.  The packed weights never pass through LDS: a wave fetches
// its 32-row x 64-channel tiles with one contiguous 1 KiB load each, already in
// operand order, dequantises a word into eight 16-bit values in registers and
// feeds them to the matrix core as the A operand; because every wave covers all
// tokens of the tile, each weight is dequantised once per workgroup.  X is staged
// through LDS (double buffered, one barrier per 64 channels) and read back as the
// B operand with 128-bit reads; the row pitch of 144 bytes keeps those reads
// conflict free.  D is [row][token], so a lane ends up with four consecutive rows
// of one token and stores them with one 8- or 16-byte write.
#include "common.hpp"
#include "launch.hpp"

namespace glowq {

constexpr int PF_WAVES = 4;
constexpr int PF_PITCH = 72;   // LDS row pitch of the X stage, in 16-bit elements

struct PfModule {
  const u32x4_t* tiles;
  const uint32_t* sz;
  const uint16_t* A;
  void* Y;
  int d_out, ldy, rows32, nt_start;   // nt_start: first 256-row tile of this module
};

struct PrefillArgs {
  PfModule mod[GLOWQ_MAX_MODULES];
  int n_modules;
  const uint16_t* X;
  const uint16_t* R16;
  int T, K, r, G;
  int restore, out_f32;
  int n_mtiles;
};

template <int ACT, int MB>
__global__ void __launch_bounds__(PF_WAVES * 64) k_prefill(PrefillArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint16_t xs[];   // [2][32 MB][PF_PITCH]
  constexpr int MT = 32 * MB;

  const int mt = (int)(blockIdx.x % (unsigned)a.n_mtiles);
  const int nt = (int)(blockIdx.x / (unsigned)a.n_mtiles);
  int mi = 0;
#pragma unroll
  for (int i = 1; i < GLOWQ_MAX_MODULES; ++i)
    if (i < a.n_modules && nt >= a.mod[i].nt_start) mi = i;
  const PfModule& M = a.mod[mi];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m = lane & 31, h = lane >> 5;
  const int ktiles = a.K >> 6;
  const int rows_pad = M.rows32 * 32;
  const int gshift = (a.G == 128) ? 1 : 0;

  // this wave's two 32-row blocks
  const int nb0 = (nt - M.nt_start) * 8 + 2 * wave;
  const bool valid[2] = {nb0 < M.rows32, nb0 + 1 < M.rows32};
  const u32x4_t* wt[2];
  const uint32_t* szp[2];
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    const int nb = valid[b] ? nb0 + b : 0;
    wt[b] = M.tiles + (size_t)nb * ktiles * 64 + lane;
    szp[b] = M.sz + nb * 32 + m;
  }

  // X stage: thread -> (row = tid / 8 + 32 p, 16-byte chunk = tid % 8)
  const int xr = tid >> 3, xc = tid & 7;
  const int tok0 = mt * MT;
  const uint16_t* xg = a.X + (size_t)(tok0 + xr) * a.K + xc * 8;

  float16_t acc[2][MB];
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[b][mb][i] = 0.f;

  u32x4_t xreg[MB];
  u32x4_t wcur[2], wnext[2];
  uint32_t szcur[2] = {0x3C00u, 0x3C00u}, sznext[2] = {0x3C00u, 0x3C00u};

  auto load_stage = [&](int kt) {
#pragma unroll
    for (int p = 0; p < MB; ++p) {
      xreg[p] = u32x4_t{0u, 0u, 0u, 0u};
      if (tok0 + xr + 32 * p < a.T)
        xreg[p] = *(const u32x4_t*)(xg + (size_t)(32 * p) * a.K + kt * 64);
    }
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      wnext[b] = u32x4_t{0u, 0u, 0u, 0u};
      if (valid[b]) {
        wnext[b] = __builtin_nontemporal_load(wt[b] + (size_t)kt * 64);
        sznext[b] = szp[b][(size_t)(kt >> gshift) * rows_pad];
      }
    }
  };
  auto store_stage = [&](int buf) {
    uint16_t* dst = xs + (size_t)buf * MT * PF_PITCH + xr * PF_PITCH + xc * 8;
#pragma unroll
    for (int p = 0; p < MB; ++p) *(u32x4_t*)(dst + 32 * p * PF_PITCH) = xreg[p];
  };

  load_stage(0);
  store_stage(0);
  wcur[0] = wnext[0];
  wcur[1] = wnext[1];
  szcur[0] = sznext[0];
  szcur[1] = sznext[1];
  __syncthreads();

  for (int kt = 0; kt < ktiles; ++kt) {
    if (kt + 1 < ktiles) load_stage(kt + 1);

    const uint16_t* xb = xs + (size_t)(kt & 1) * MT * PF_PITCH + m * PF_PITCH + 32 * h;
    GroupConst<ACT> g[2];
    g[0].set(szcur[0]);
    g[1].set(szcur[1]);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      u32x4_t wf0 = dequant_word<ACT>(wcur[0][j], g[0]);
      u32x4_t wf1 = dequant_word<ACT>(wcur[1][j], g[1]);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        u32x4_t xf = *(const u32x4_t*)(xb + mb * 32 * PF_PITCH + 8 * j);
        if (valid[0]) acc[0][mb] = mfma32<ACT>(wf0, xf, acc[0][mb]);   // D[row][token]
        if (valid[1]) acc[1][mb] = mfma32<ACT>(wf1, xf, acc[1][mb]);
      }
    }

    if (kt + 1 < ktiles) {
      store_stage((kt + 1) & 1);
      wcur[0] = wnext[0];
      wcur[1] = wnext[1];
      szcur[0] = sznext[0];
      szcur[1] = sznext[1];
    }
    __syncthreads();
  }

  // correction: r more channels, operand [A_i] against [R]
  if (a.restore) {
    // the trip count is the same for every lane (matrix-core instructions must not sit
    // under a divergent branch); a half-wave past the rank contributes zeros
    for (int jj = 0; jj * 16 < a.r; ++jj) {
      const int j0 = jj * 16 + 8 * h;
      const bool j_ok = j0 < a.r;
      u32x4_t af[2];
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        af[b] = u32x4_t{0u, 0u, 0u, 0u};
        const int row = (nb0 + b) * 32 + m;
        if (j_ok && valid[b] && row < M.d_out)
          af[b] = *(const u32x4_t*)(M.A + (size_t)row * a.r + j0);
      }
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        const int tok = tok0 + mb * 32 + m;
        u32x4_t rf = {0u, 0u, 0u, 0u};
        if (j_ok && tok < a.T) rf = *(const u32x4_t*)(a.R16 + (size_t)tok * a.r + j0);
        if (valid[0]) acc[0][mb] = mfma32<ACT>(af[0], rf, acc[0][mb]);
        if (valid[1]) acc[1][mb] = mfma32<ACT>(af[1], rf, acc[1][mb]);
      }
    }
  }

  // store: lane holds token (mb, m) and rows 8 q + 4 h + {0..3} of each 32-row block
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    if (!valid[b]) continue;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int tok = tok0 + mb * 32 + m;
      if (tok >= a.T) continue;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int row = (nb0 + b) * 32 + 8 * q + 4 * h;
        if (row >= M.d_out) continue;
        const size_t off = (size_t)tok * M.ldy + row;
        const float v0 = acc[b][mb][4 * q], v1 = acc[b][mb][4 * q + 1];
        const float v2 = acc[b][mb][4 * q + 2], v3 = acc[b][mb][4 * q + 3];
        if (a.out_f32) {
          *(float4_t*)((float*)M.Y + off) = float4_t{v0, v1, v2, v3};
        } else {
          uint2 pk;
          pk.x = (uint32_t)to_act16<ACT>(v0) | ((uint32_t)to_act16<ACT>(v1) << 16);
          pk.y = (uint32_t)to_act16<ACT>(v2) | ((uint32_t)to_act16<ACT>(v3) << 16);
          *(uint2*)((uint16_t*)M.Y + off) = pk;
        }
      }
    }
  }
}

template <int ACT, int MB>
static hipError_t launch_prefill_t(const PrefillArgs& a, int n_ntiles, hipStream_t st) {
  const size_t lds = (size_t)2 * 32 * MB * PF_PITCH * sizeof(uint16_t);
  auto kern = k_prefill<ACT, MB>;
  hipError_t e = hipFuncSetAttribute((const void*)kern,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  dim3 grid((unsigned)(a.n_mtiles * n_ntiles)), block(PF_WAVES * 64);
  kern<<<grid, block, lds, st>>>(a);
  return hipGetLastError();
}

hipError_t launch_prefill(const glowq_unit& u, const UnitWorkspace& ws, bool restore,
                          hipStream_t st) {
  PrefillArgs a;
  int nt = 0;
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
    a.mod[i].nt_start = nt;
    nt += (v.rows32 + 7) / 8;
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
  const bool f16 = (u.act_dtype == GLOWQ_F16);
  if (u.T <= 64) {
    a.n_mtiles = (u.T + 63) / 64;
    return f16 ? launch_prefill_t<ACT_F16, 2>(a, nt, st) : launch_prefill_t<ACT_BF16, 2>(a, nt, st);
  }
  if (u.T <= 128) {
    a.n_mtiles = (u.T + 127) / 128;
    return f16 ? launch_prefill_t<ACT_F16, 4>(a, nt, st) : launch_prefill_t<ACT_BF16, 4>(a, nt, st);
  }
  a.n_mtiles = (u.T + 255) / 256;
  return f16 ? launch_prefill_t<ACT_F16, 8>(a, nt, st) : launch_prefill_t<ACT_BF16, 8>(a, nt, st);
}

}  // namespace glowq
