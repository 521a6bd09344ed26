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
// of the grid run the projection and publish every partial sum as a self-validating
// 8-byte slot {fp32 bits, launch tag}; everyone else streams weights in the meantime and
// fetches the slots (adding the K parts) without any flag or counter in between -- a
// kernel boundary would cost as much as the whole weight stream.
// The four waves' fp32 tiles are folded through LDS and stored.
//
// Waits: every global -> LDS load of these kernels is issued as assembly (lds_dma16 /
// lds_dma4), and no load the compiler knows of sits behind a branch between a buffer's
// loads and their use; otherwise the compiler makes each buffer's first use wait for ALL
// loads in flight, the next buffer's included, and nothing overlaps.
#include "decode_device.hpp"
#include "proj_device.hpp"
#include "launch.hpp"

namespace glowq {

static_assert(GLOWQ_MAX_RANK <= DEC_WAVES * 32, "one 32-rank correction step per wave");

// Grid: [n_prod projection workgroups][one workgroup per DEC_RG 16-row blocks].
template <int ACT, int TBK, int NW>
__global__ void __launch_bounds__(NW * 64) k_decode(DecodeArgs a, ProjArgs p, int n_prod,
                                                   int n_blocks) {
  __shared__ float lds[DEC_RG * NW * TBK * 4 * 64];
  __shared__ __attribute__((aligned(16))) uint16_t r_lds[16 * TBK * GLOWQ_MAX_RANK];
  __shared__ uint32_t r_flag;
  __shared__ __attribute__((aligned(1024))) uint32_t lds_af[NW * DEC_RG * 256];
  if ((int)blockIdx.x < n_prod) {
    const int per_tb = p.ksplit * p.groups, rem = (int)blockIdx.x % per_tb;
    proj_workgroup<ACT>(p, (int)blockIdx.x / per_tb, rem % p.ksplit, rem / p.ksplit, lds);
    return;
  }
  decode_workgroup<ACT, TBK, NW>(a, p, (int)blockIdx.x - n_prod, n_blocks, lds, r_lds, &r_flag, lds_af);
}

// Up to NB units of the same kind (activation type, token class) in one launch: the grid
// is the concatenation of the units' [projection waves][row blocks].  The descriptor
// block travels as the kernel argument; its size is a template parameter because a
// one-unit call pays measurably for a block sized for many (and a whole model's stack
// gains from fewer, larger launches).
constexpr int DEC_MAX_BATCH = 32;
template <int NB> struct DecodeBatch {
  DecodeArgs a[NB];
  ProjArgs p[NB];
  int n_prod[NB];
  int wg_start[NB];
  int n;
};

// whether the projection waves ride in the first row-block workgroups (see k_decode_small)
constexpr bool decode_small_merged(int tm) { return tm > 2; }

template <int ACT, int TM, int NB>
__global__ void __launch_bounds__(DEC_WAVES * 64) k_decode_small(DecodeBatch<NB> b) {
  __shared__ __attribute__((aligned(1024))) float lds[DEC_WAVES * 4 * 64];
  __shared__ __attribute__((aligned(64))) char lds_x[DEC_WAVES * DecX<TM>::WAVE_BYTES];
  __shared__ __attribute__((aligned(16))) uint32_t lds_rf[DEC_WAVES * TM * DEC_MAX_PARTS * 64];
  // the A_i fragments land in the fold area: wave w's 1 KiB row is exactly the part of it
  // that wave w itself overwrites, and it does so only after it has taken its fragment
  uint32_t* lds_af = (uint32_t*)lds;
  // (a one-unit launch reads its descriptor at fixed offsets of the kernel argument: one
  // batch of scalar loads instead of a chain through the unit lookup)
  int ui = 0;
#pragma unroll
  for (int i = 1; i < NB; ++i)
    if (i < b.n && (int)blockIdx.x >= b.wg_start[i]) ui = i;
  const DecodeArgs& a = b.a[ui];
  const ProjArgs& p = b.p[ui];
  const int local = (int)blockIdx.x - b.wg_start[ui];
  const int n_prod = b.n_prod[ui];
  // The 3- and 4-token instance holds three workgroups per compute unit (LDS), which a
  // 7B-sized unit's row blocks fill exactly: there the projection waves are the first
  // workgroups' prologue instead of workgroups of their own, so that the whole grid is
  // resident from the start and no row block waits for a projection workgroup's slot.
  constexpr bool MERGED = decode_small_merged(TM);
  if (local < n_prod) {
    proj_wave_direct<ACT>(p, local * DEC_WAVES + (int)(threadIdx.x >> 6), (int)(threadIdx.x & 63));
    if (!MERGED) return;
  }
  const int blk = MERGED ? local : local - n_prod;
  if (MERGED && blk >= a.mod[a.n_modules - 1].blk_start + a.mod[a.n_modules - 1].rows16) return;
  decode_workgroup_small<ACT, TM>(a, p, blk, lds, lds_x, lds_rf, lds_af);
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
  a.T = u.T;
  a.K = u.d_in;
  a.r = u.r;
  a.G = u.group_size;
  a.restore = restore ? 1 : 0;
  a.out_f32 = (u.out_dtype == GLOWQ_F32) ? 1 : 0;
  return blk;
}

static int decode_small_class(int T) { return T == 1 ? 1 : T == 2 ? 2 : DEC_SMALL_T; }

bool decode_batch_compatible(const glowq_unit& a, const glowq_unit& b) {
  return a.T <= DEC_SMALL_T && b.T <= DEC_SMALL_T && a.act_dtype == b.act_dtype &&
         decode_small_class(a.T) == decode_small_class(b.T);
}
int decode_max_batch() { return DEC_MAX_BATCH; }

template <int NB>
static hipError_t launch_decode_small(const glowq_unit* const* units, const UnitWorkspace* ws,
                                      const bool* restore, int n, hipStream_t st) {
  const glowq_unit& u0 = *units[0];
  const bool f16 = (u0.act_dtype == GLOWQ_F16);
  dim3 block(DEC_WAVES * 64);
  {
    DecodeBatch<NB> b;
    int wg = 0;
    for (int i = 0; i < n; ++i) {
      const glowq_unit& u = *units[i];
      const int blocks = fill_decode_args(u, ws[i], restore[i], b.a[i]);
      b.p[i] = ProjArgs{};
      b.n_prod[i] = 0;
      b.a[i].ctl = (Control*)ws[i].base;
      if (restore[i]) {
        b.p[i] = make_proj_args(u, ws[i], nullptr, true);
        b.n_prod[i] = (u.r * ws[i].ksplit + DEC_WAVES - 1) / DEC_WAVES;   // one wave per (rank, part)
      }
      b.wg_start[i] = wg;
      if (decode_small_merged(decode_small_class(u0.T))) wg += b.n_prod[i] > blocks ? b.n_prod[i] : blocks;
      else wg += b.n_prod[i] + blocks;
    }
    for (int i = n; i < NB; ++i) {
      b.a[i] = b.a[0];
      b.p[i] = b.p[0];
      b.n_prod[i] = 0;
      b.wg_start[i] = wg;
    }
    b.n = n;
    dim3 grid((unsigned)wg);
    // the one- and two-token instances keep their LDS small enough for four workgroups
    // per compute unit, so that a unit's whole grid is resident at once
    switch (decode_small_class(u0.T)) {
      case 1:
        if (f16) k_decode_small<ACT_F16, 1, NB><<<grid, block, 0, st>>>(b);
        else k_decode_small<ACT_BF16, 1, NB><<<grid, block, 0, st>>>(b);
        break;
      case 2:
        if (f16) k_decode_small<ACT_F16, 2, NB><<<grid, block, 0, st>>>(b);
        else k_decode_small<ACT_BF16, 2, NB><<<grid, block, 0, st>>>(b);
        break;
      default:
        if (f16) k_decode_small<ACT_F16, DEC_SMALL_T, NB><<<grid, block, 0, st>>>(b);
        else k_decode_small<ACT_BF16, DEC_SMALL_T, NB><<<grid, block, 0, st>>>(b);
    }
    return hipGetLastError();
  }
}

// units[i] uses workspace slice ws[i]; all of them pass decode_batch_compatible with
// units[0] (or n == 1, any decode-sized unit).
hipError_t launch_decode_multi(const glowq_unit* const* units, const UnitWorkspace* ws,
                               const bool* restore, int n, hipStream_t st) {
  const glowq_unit& u0 = *units[0];
  const bool f16 = (u0.act_dtype == GLOWQ_F16);
  dim3 block(DEC_WAVES * 64);
  if (u0.T <= DEC_SMALL_T) {
    if (n == 1) return launch_decode_small<1>(units, ws, restore, n, st);
    if (n <= 2) return launch_decode_small<2>(units, ws, restore, n, st);
    if (n <= 8) return launch_decode_small<8>(units, ws, restore, n, st);
    return launch_decode_small<DEC_MAX_BATCH>(units, ws, restore, n, st);
  }
  // 4 < T <= 32: one unit per launch
  for (int i = 0; i < n; ++i) {
    const glowq_unit& u = *units[i];
    DecodeArgs a;
    const int blocks = fill_decode_args(u, ws[i], restore[i], a);
    ProjArgs p = {};
    int n_prod = 0;
    a.ctl = (Control*)ws[i].base;
    if (restore[i]) {
      p = make_proj_args(u, ws[i], nullptr, true);
      // (few K slices, so that the consumers gather few partial sums per rank, and two
      // workgroups per slice, so that a projection workgroup reads no more of B than before)
      p.groups = u.r > 16 ? 2 : 1;
      n_prod = ((u.T + 15) / 16) * ws[i].ksplit * p.groups;
    }
    dim3 grid((unsigned)(n_prod + (blocks + DEC_RG - 1) / DEC_RG));
    // (eight waves per workgroup, i.e. twice the tiles in flight per compute unit, were
    // measured for up to 16 tokens: the stream took as long and the correction longer)
    if (u.T <= 16) {
      if (f16) k_decode<ACT_F16, 1, DEC_WAVES><<<grid, block, 0, st>>>(a, p, n_prod, blocks);
      else k_decode<ACT_BF16, 1, DEC_WAVES><<<grid, block, 0, st>>>(a, p, n_prod, blocks);
    } else {
      if (f16) k_decode<ACT_F16, 2, DEC_WAVES><<<grid, block, 0, st>>>(a, p, n_prod, blocks);
      else k_decode<ACT_BF16, 2, DEC_WAVES><<<grid, block, 0, st>>>(a, p, n_prod, blocks);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace glowq

GLOWQ_TRACE_EXPORT(glowq_debug_trace)
GLOWQ_WTRACE_EXPORT(glowq_debug_wtrace)
