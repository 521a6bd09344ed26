// Prefill path (T > 32 tokens): Y_i = X dequant(W_q,i)^T + R A_i^T  (paper Eq. 9)
// as a tiled matrix-core GEMM with the correction folded in as r extra channels.
//
// Workgroup tile: (16 MB) tokens x 256 rows, four waves, each wave 64 rows x all
// tokens of the tile.  The packed weights never pass through LDS: a wave fetches
// its 16-row x 128-channel tiles with one contiguous 1 KiB load each, already in
// operand order, dequantises a word into eight 16-bit values in registers (one
// rounding, the stored weight exactly) and feeds them to the matrix core as the A
// operand of a 16x16x32 instruction; because every wave covers all tokens of the
// tile, each weight is dequantised once per workgroup.  X is staged through LDS in
// 64-channel stages (double buffered, one barrier per stage) and read back as the
// B operand with 128-bit reads; the row pitch of 144 bytes keeps those reads
// conflict free.  D is [row][token], so a lane ends up with four consecutive rows
// of one token and stores them with one 8- or 16-byte write.
#include "common.hpp"
#include "launch.hpp"

namespace glowq {

constexpr int PF_WAVES = 4;
constexpr int PF_PITCH = 72;   // LDS row pitch of the X stage, in 16-bit elements

struct PfModule {
  const uint32_t* rec;   // tile records (see common.hpp)
  const uint16_t* A;
  void* Y;
  int d_out, ldy, rows16, nt_start;   // nt_start: first 256-row tile of this module
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
  extern __shared__ __attribute__((aligned(16))) uint16_t xs[];   // [2][16 MB][PF_PITCH]
  constexpr int MT = 16 * MB;
  constexpr int XP = MT / 32;     // X rows per thread and stage

  const int mt = (int)(blockIdx.x % (unsigned)a.n_mtiles);
  const int nt = (int)(blockIdx.x / (unsigned)a.n_mtiles);
  int mi = 0;
#pragma unroll
  for (int i = 1; i < GLOWQ_MAX_MODULES; ++i)
    if (i < a.n_modules && nt >= a.mod[i].nt_start) mi = i;
  const PfModule& M = a.mod[mi];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 15, kq = lane >> 4;
  const int ktiles = a.K >> 7;
  const bool g128 = (a.G == 128);
  const int rw = g128 ? 272 : 288;             // words per tile record

  // this wave's four 16-row blocks
  const int nb0 = (nt - M.nt_start) * 16 + 4 * wave;
  bool valid[4];
  const uint32_t* wt[4];
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    valid[b] = nb0 + b < M.rows16;
    const int nb = valid[b] ? nb0 + b : 0;
    wt[b] = M.rec + (size_t)nb * ktiles * rw;
  }

  // X stage: thread -> (row = tid / 8 + 32 p, 16-byte chunk = tid % 8); rows past T
  // re-read the last valid token (their columns of D are never stored)
  const int xr = tid >> 3, xc = tid & 7;
  const int tok0 = mt * MT;
  const uint16_t* xg[XP];
#pragma unroll
  for (int p = 0; p < XP; ++p)
    xg[p] = a.X + (size_t)min(tok0 + xr + 32 * p, a.T - 1) * a.K + xc * 8;

  float4_t acc[4][MB];
#pragma unroll
  for (int b = 0; b < 4; ++b)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) acc[b][mb] = float4_t{0.f, 0.f, 0.f, 0.f};

  u32x4_t xreg[XP];
  u32x4_t wcur[4], wnext[4];
  uint32_t szcur[4][2], sznext[4][2];

  auto load_x = [&](int stage) {
#pragma unroll
    for (int p = 0; p < XP; ++p) xreg[p] = *(const u32x4_t*)(xg[p] + stage * 64);
  };
  auto store_x = [&](int buf) {
    uint16_t* dst = xs + (size_t)buf * MT * PF_PITCH + xr * PF_PITCH + xc * 8;
#pragma unroll
    for (int p = 0; p < XP; ++p) *(u32x4_t*)(dst + 32 * p * PF_PITCH) = xreg[p];
  };
  auto load_w = [&](int kt) {
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const uint32_t* rec = wt[b] + (size_t)kt * rw;
      wnext[b] = __builtin_nontemporal_load((const u32x4_t*)rec + lane);
      sznext[b][0] = rec[256 + n];
      sznext[b][1] = g128 ? sznext[b][0] : rec[272 + n];
    }
  };
  auto take_w = [&]() {
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      wcur[b] = wnext[b];
      szcur[b][0] = sznext[b][0];
      szcur[b][1] = sznext[b][1];
    }
  };

  load_x(0);
  load_w(0);
  store_x(0);
  take_w();
  __syncthreads();

  const int nstages = 2 * ktiles;
  for (int kt = 0; kt < ktiles; ++kt) {
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int stage = 2 * kt + half;
      if (stage + 1 < nstages) load_x(stage + 1);
      if (half == 0 && kt + 1 < ktiles) load_w(kt + 1);

      const uint16_t* xb = xs + (size_t)(stage & 1) * MT * PF_PITCH + n * PF_PITCH + 8 * kq;
      GroupConst<ACT> g[4];
#pragma unroll
      for (int b = 0; b < 4; ++b) g[b].set(szcur[b][half]);
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const int j = 2 * half + jj;
        u32x4_t wf[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) wf[b] = dequant_word<ACT>(wcur[b][j], g[b]);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
          const u32x4_t xf = *(const u32x4_t*)(xb + mb * 16 * PF_PITCH + 32 * jj);
#pragma unroll
          for (int b = 0; b < 4; ++b)
            if (valid[b]) acc[b][mb] = mfma16<ACT>(wf[b], xf, acc[b][mb]);   // D[row][token]
        }
      }

      if (stage + 1 < nstages) store_x((stage + 1) & 1);
      __syncthreads();
    }
    if (kt + 1 < ktiles) take_w();
  }

  // correction: r more channels, operand [A_i] against [R]; every lane runs the same
  // trip count, lanes past the rank contribute zeros on both sides
  if (a.restore) {
    for (int jj = 0; jj * 32 < a.r; ++jj) {
      const int j0 = jj * 32 + 8 * kq;
      const bool ok = j0 < a.r;
      const int j0c = ok ? j0 : 0;
      u32x4_t af[4];
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const int row = min((nb0 + b) * 16 + n, M.d_out - 1);
        af[b] = *(const u32x4_t*)(M.A + (size_t)row * a.r + j0c);
        if (!ok) af[b] = u32x4_t{0u, 0u, 0u, 0u};
      }
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        const int tok = min(tok0 + mb * 16 + n, a.T - 1);
        u32x4_t rf = *(const u32x4_t*)(a.R16 + (size_t)tok * a.r + j0c);
        if (!ok) rf = u32x4_t{0u, 0u, 0u, 0u};
#pragma unroll
        for (int b = 0; b < 4; ++b)
          if (valid[b]) acc[b][mb] = mfma16<ACT>(af[b], rf, acc[b][mb]);
      }
    }
  }

  // store: lane holds token (mb, n) and rows 4 kq + {0..3} of each 16-row block
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    if (!valid[b]) continue;
    const int row = (nb0 + b) * 16 + 4 * kq;
    if (row >= M.d_out) continue;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int tok = tok0 + mb * 16 + n;
      if (tok >= a.T) continue;
      const size_t off = (size_t)tok * M.ldy + row;
      const float4_t v = acc[b][mb];
      if (a.out_f32) {
        *(float4_t*)((float*)M.Y + off) = v;
      } else {
        uint2 pk;
        pk.x = (uint32_t)to_act16<ACT>(v[0]) | ((uint32_t)to_act16<ACT>(v[1]) << 16);
        pk.y = (uint32_t)to_act16<ACT>(v[2]) | ((uint32_t)to_act16<ACT>(v[3]) << 16);
        *(uint2*)((uint16_t*)M.Y + off) = pk;
      }
    }
  }
}

template <int ACT, int MB>
static hipError_t launch_prefill_t(const PrefillArgs& a, int n_ntiles, hipStream_t st) {
  const size_t lds = (size_t)2 * 16 * MB * PF_PITCH * sizeof(uint16_t);
  auto kern = k_prefill<ACT, MB>;
  if (lds > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute((const void*)kern,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
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
    PreparedView v = prepared_view(m.w_prepared, m.d_out, u.d_in, u.group_size);
    a.mod[i].rec = v.base;
    a.mod[i].A = (const uint16_t*)m.A;
    a.mod[i].Y = m.Y;
    a.mod[i].d_out = m.d_out;
    a.mod[i].ldy = m.ldy;
    a.mod[i].rows16 = v.rows16;
    a.mod[i].nt_start = nt;
    nt += (v.rows16 + 15) / 16;
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
    return f16 ? launch_prefill_t<ACT_F16, 4>(a, nt, st) : launch_prefill_t<ACT_BF16, 4>(a, nt, st);
  }
  if (u.T <= 128) {
    a.n_mtiles = (u.T + 127) / 128;
    return f16 ? launch_prefill_t<ACT_F16, 8>(a, nt, st) : launch_prefill_t<ACT_BF16, 8>(a, nt, st);
  }
  a.n_mtiles = (u.T + 255) / 256;
  return f16 ? launch_prefill_t<ACT_F16, 16>(a, nt, st) : launch_prefill_t<ACT_BF16, 16>(a, nt, st);
}

}  // namespace glowq
