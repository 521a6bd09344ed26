// Prefill path (T > 32 tokens): Y_i = X dequant(W_q,i)^T + R A_i^T  (paper Eq. 9)
// as a tiled matrix-core GEMM with the correction folded in as r extra channels, and
// R = X B^T (paper Eq. 8) computed by the leading tiles of the same launch.
//
// Workgroup tile: (16 MB) tokens x 256 rows (192 for bfloat16), four waves, each wave
// 64 (48) rows x all tokens of the tile; at most 256 registers per lane, so two
// workgroups share a compute unit and one's barrier or memory wait leaves the matrix
// cores to the other.  Because every wave covers all tokens of the tile, each weight is
// dequantised once per workgroup (in registers: one rounding, the stored weight exactly)
// and becomes the A operand of a 16x16x32 instruction.  Everything that moves is a
// direct global->LDS load: X in 64-channel stages into a ring of three (the 16-byte
// chunks of a row XOR-swizzled by the row index on the global-address side, so that the
// 128-bit operand reads are conflict free without padding), the tile records of the next
// tile into a per-wave stage.  The operand reads, the waits and the one barrier per
// stage are placed by hand (see the kernel).  D is [row][token], so a lane ends up with
// four consecutive rows of one token and stores them with one 8- or 16-byte write.
#include <type_traits>
#include <algorithm>
#include "common.hpp"
#include "launch.hpp"

namespace glowq {

// Two waves per SIMD either way: binary16 runs two workgroups of four waves per compute
// unit (64 rows per wave; a workgroup waiting at its barrier or for memory leaves the
// matrix cores to the other one), bfloat16, whose dequantiser needs more registers, one
// workgroup of eight waves (32 rows per wave).
template <int ACT> struct PfShape {
  static constexpr int WAVES = 4;
  // 16-row blocks per wave: 256-row tiles for binary16; bfloat16, whose dequantiser
  // holds more in registers, takes 192-row tiles to stay within 256 registers per lane
  static constexpr int RB = ACT == ACT_F16 ? 4 : 3;
  static constexpr int TILE_BLOCKS = WAVES * RB;   // 16-row blocks per workgroup tile
  static constexpr int OCC = 8 / WAVES;    // workgroups per compute unit
  static constexpr int XD = 2;              // LDS operand reads in flight per wave
};

// One launch covers up to PF_MAX_UNITS units (PF_MAX_MODS modules in all) that share the
// activation type, group size, output type and token-tile size; the grid is the
// concatenation of the modules' tile lists, longest contraction first, so that the
// hardware's in-order dispatch starts the long tiles first.
constexpr int PF_MAX_UNITS = 8;
constexpr int PF_MAX_MODS = 16;
constexpr int PF_PANEL = 2;       // token tiles per panel of the tile order (see k_prefill)

struct PfUnit {
  const uint16_t* X;
  const uint16_t* B;       // shared right factor [r][K]
  uint16_t* R16;           // R = X B^T rounded to the activation type, [T][r], in the workspace
  float* Rpart;            // fp32 [parts][T][r]: the K parts' partial sums (parts > 1 only)
  uint32_t* flags;         // one word per 16-token block; word MB*mt is token tile mt's ready
                           // flag, word MB*mt + 1 counts the K parts of that tile that are done
  int parts;               // K parts of a projection tile (one workgroup each)
  int part_stages;         // 64-channel stages per part
  uint32_t* status;        // the unit's status word (see Control)
  int T, K, r, restore, n_mtiles;
  int proj_start;          // first workgroup of this unit's projection tiles in the grid
};

struct PfModule {
  const uint32_t* rec;   // tile records (see common.hpp)
  const uint16_t* A;
  void* Y;
  int d_out, ldy, rows16;
  int unit;              // index into PrefillArgs::unit
  int wg_start;          // first workgroup of this module in the grid
  int n_ntiles;          // row tiles of the module; its workgroups: n_ntiles * unit.n_mtiles
  // A module of a long contraction may stand here several times, once per slice of K: each
  // entry multiplies the K tiles [kt0, kt0 + nkt) and leaves an fp32 partial result (Y, ldy:
  // its slab of the workspace); the first entry carries the correction; k_splitk_sum adds
  // the slabs and writes the module's output.
  int kt0, nkt;
  int corr;              // this entry applies the correction (if the unit is restored)
  int out_f32;           // what Y holds: fp32, or the activation type
};

struct PrefillArgs {
  PfUnit unit[PF_MAX_UNITS];
  PfModule mod[PF_MAX_MODS];
  int n_mods;
  int n_units;
  int n_proj_wgs;          // the grid starts with this many projection tiles
  int out_f32;
};


// a pointer that is the same in every lane, moved to scalar registers
template <typename T> __device__ inline T* uniform_ptr(T* p) {
  const unsigned long long v = (unsigned long long)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (T*)(((unsigned long long)hi << 32) | lo);
}

// Projection tile of the prefill launch: R[tile] = X[tile] B^T  (paper Eq. 8), MT tokens x
// all r ranks, rounded once to the activation type and stored in the workspace; then the
// tile's flag is set to this launch's tag.  These tiles are the first workgroups of the
// grid, so they are running before any tile that needs their result has started, and
// they wait for nothing.  A long contraction is cut into K parts, one workgroup each, so
// that R is ready well before the main tiles of the same unit reach their correction:
// every part leaves its fp32 partial tile in the workspace and counts itself in; the
// part that finds all others counted adds the partial tiles in part order (so the sum
// does not depend on which one that is), rounds, stores and sets the flag.
// X takes the same path as in the main tiles (LDS ring, swizzled rows); the rows of B
// are read straight into operand registers, one stage ahead.
template <int ACT, int MB>
__device__ inline void proj_tile(const PrefillArgs& a, uint16_t* xs) {
  constexpr int PF_WAVES = PfShape<ACT>::WAVES;
  constexpr int RBP = 8 / PF_WAVES;      // 16-rank blocks per wave (r <= 128)
  constexpr int MT = 16 * MB, XR = PF_WAVES * 8, XI = MT / XR, NBUF = 3;
  constexpr uint32_t STAGE_BYTES = MT * 64 * 2;
  // units without a projection carry proj_start = -1; the others' increase with the index
  int ui = 0;
#pragma unroll
  for (int i = 0; i < PF_MAX_UNITS; ++i)
    if (i < a.n_units && a.unit[i].proj_start >= 0 && (int)blockIdx.x >= a.unit[i].proj_start) ui = i;
  const PfUnit& U = a.unit[ui];
  const int local = (int)blockIdx.x - U.proj_start;
  const int mt = local / U.parts, part = local - mt * U.parts;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 15, kq = lane >> 4;
  const int nstages = U.K >> 6;
  const int s_begin = part * U.part_stages;                    // < nstages (host)
  const int s_end = min(nstages, s_begin + U.part_stages);
  const int tok0 = mt * MT;

  const uint16_t* xsrc[XI];
#pragma unroll
  for (int i = 0; i < XI; ++i) {
    const int row = XR * i + (tid >> 3);
    const int chunk = (tid & 7) ^ ((row >> 1) & 7);
    xsrc[i] = U.X + (size_t)min(tok0 + row, U.T - 1) * U.K + chunk * 8;
  }
  auto dma_x = [&](int stage, int slot, int i) {
    const int st = min(stage, nstages - 1);
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)(xsrc[i] + st * 64),
        (__attribute__((address_space(3))) void*)(xs + slot * (MT * 64) + (XR * i + 8 * wave) * 64),
        16, 0, 0);
  };
  const uint32_t xs_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)xs;
  const int rd_row = n * 64, rd_sw = (n >> 1) & 7;
  const uint32_t rd_lane[2] = {xs_base + 2u * (uint32_t)(rd_row + (((0 + kq) ^ rd_sw) << 3)),
                               xs_base + 2u * (uint32_t)(rd_row + (((4 + kq) ^ rd_sw) << 3))};
  // rank rows of this lane, clamped (ranks past r are computed from row r-1, not stored)
  const uint16_t* bsrc[RBP];
#pragma unroll
  for (int b = 0; b < RBP; ++b)
    bsrc[b] = U.B + (size_t)min((wave * RBP + b) * 16 + n, U.r - 1) * U.K + 8 * kq;
  u32x4_t bcur[RBP][2], bnext[RBP][2];   // operand words of the two 32-channel steps of a stage
  auto load_b = [&](int stage) {
    const int st = min(stage, nstages - 1);
#pragma unroll
    for (int b = 0; b < RBP; ++b)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) vm_load(bnext[b][jj], bsrc[b] + st * 64 + jj * 32);
  };

  float4_t acc[RBP][MB];
#pragma unroll
  for (int b = 0; b < RBP; ++b)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) acc[b][mb] = float4_t{0.f, 0.f, 0.f, 0.f};

#pragma unroll
  for (int i = 0; i < XI; ++i) dma_x(s_begin, 0, i);
#pragma unroll
  for (int i = 0; i < XI; ++i) dma_x(s_begin + 1, 1, i);
  load_b(s_begin);
  vm_wait<0>();
#pragma unroll
  for (int b = 0; b < RBP; ++b)
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) { after_wait(bnext[b][jj]); bcur[b][jj] = bnext[b][jj]; }
  __builtin_amdgcn_s_barrier();

  int slot_cur = 0, slot_next2 = 2;
  for (int stage = s_begin; stage < s_end; ++stage) {
    const uint32_t xa[2] = {rd_lane[0] + (uint32_t)slot_cur * STAGE_BYTES,
                            rd_lane[1] + (uint32_t)slot_cur * STAGE_BYTES};
    u32x4_t xq[3];
    lds_read(xq[0], xa[0], 0);
    lds_read(xq[1], xa[0], 2048);
    // in this order: the next stage's B words, then X of the stage after next
    load_b(stage + 1);
#pragma unroll
    for (int i = 0; i < XI; ++i) dma_x(stage + 2, slot_next2, i);
#pragma unroll
    for (int f = 0; f < 2 * MB; ++f) {
      if (f + 2 < 2 * MB) {
        lds_read(xq[(f + 2) % 3], xa[(f + 2) / MB], ((f + 2) % MB) * 2048);
        lds_wait<2>(xq[f % 3]);
      } else if (f + 2 == 2 * MB) lds_wait<1>(xq[f % 3]);
      else lds_wait<0>(xq[f % 3]);
#pragma unroll
      for (int b = 0; b < RBP; ++b)
        acc[b][f % MB] = mfma16<ACT>(bcur[b][f / MB], xq[f % 3], acc[b][f % MB]);   // D[rank][token]
    }
    // everything older than this stage's XI X loads has completed after this: the next
    // stage's X (issued a stage ago) and the next stage's B words
    vm_wait<XI>();
#pragma unroll
    for (int b = 0; b < RBP; ++b)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) { after_wait(bnext[b][jj]); bcur[b][jj] = bnext[b][jj]; }
    __builtin_amdgcn_s_barrier();
    slot_cur = slot_cur == NBUF - 1 ? 0 : slot_cur + 1;
    slot_next2 = slot_next2 == NBUF - 1 ? 0 : slot_next2 + 1;
  }
  vm_wait<0>();   // nothing may still be on its way into LDS when the workgroup ends

  // lane holds token (mb, n) and ranks 16 blk + 4 kq + {0..3}
  if (U.parts > 1) {
    float* mine = U.Rpart + (size_t)part * U.T * U.r;
#pragma unroll
    for (int b = 0; b < RBP; ++b) {
      const int rank0 = (wave * RBP + b) * 16 + 4 * kq;
      if (rank0 >= U.r) continue;
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        const int tok = tok0 + mb * 16 + n;
        if (tok < U.T) *(float4_t*)(mine + (size_t)tok * U.r + rank0) = acc[b][mb];
      }
    }
    // count this part in (after its stores are visible device-wide); all but the last
    // one to arrive are done
    __threadfence();
    __syncthreads();
    uint32_t* lds_word = (uint32_t*)xs;      // the X ring is idle from here on
    if (tid == 0)
      *lds_word = __hip_atomic_fetch_add(U.flags + MB * mt + 1, 1u, __ATOMIC_ACQ_REL,
                                         __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const uint32_t arrived = *lds_word;
    if (arrived + 1 != (uint32_t)U.parts) return;   // uniform
    __threadfence();
#pragma unroll
    for (int b = 0; b < RBP; ++b) {
      const int rank0 = (wave * RBP + b) * 16 + 4 * kq;
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        const int tok = min(tok0 + mb * 16 + n, U.T - 1);
        float4_t sum = float4_t{0.f, 0.f, 0.f, 0.f};
        if (rank0 < U.r) {
          for (int p = 0; p < U.parts; ++p) {
            const uint32_t* q = (const uint32_t*)(U.Rpart + ((size_t)p * U.T + tok) * U.r + rank0);
#pragma unroll
            for (int v = 0; v < 4; ++v)
              sum[v] += __builtin_bit_cast(float, __hip_atomic_load(q + v, __ATOMIC_RELAXED,
                                                                    __HIP_MEMORY_SCOPE_AGENT));
          }
        }
        acc[b][mb] = sum;
      }
    }
    if (tid == 0)   // the next launch counts from zero again
      __hip_atomic_store(U.flags + MB * mt + 1, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
#pragma unroll
  for (int b = 0; b < RBP; ++b) {
    const int rank0 = (wave * RBP + b) * 16 + 4 * kq;
    if (rank0 >= U.r) continue;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int tok = tok0 + mb * 16 + n;
      if (tok >= U.T) continue;
      const float4_t v = acc[b][mb];
      uint2 pk;
      pk.x = (uint32_t)to_act16<ACT>(v[0]) | ((uint32_t)to_act16<ACT>(v[1]) << 16);
      pk.y = (uint32_t)to_act16<ACT>(v[2]) | ((uint32_t)to_act16<ACT>(v[3]) << 16);
      *(uint2*)(U.R16 + (size_t)tok * U.r + rank0) = pk;
    }
  }
  // publish: every wave makes its stores visible device-wide, then one thread sets the flag
  __threadfence();
  __syncthreads();
  if (tid == 0)
    __hip_atomic_store(U.flags + MB * mt, (uint32_t)launch_tag(), __ATOMIC_RELEASE,
                       __HIP_MEMORY_SCOPE_AGENT);
}

// Waits until token tile mt's part of R carries this launch's tag.  The projection tiles
// lead the grid and wait for nothing, so by the time a main tile has run through its
// whole contraction they have long finished; the loop is bounded all the same, and a
// wave that gives up records it in the unit's status word and leaves the correction out
// rather than hang.
__device__ inline bool wait_tile_ready(const uint32_t* flag, uint32_t* status) {
  const uint32_t tag = (uint32_t)launch_tag();
  bool ok = false;
  for (int spin = 0; spin < (1 << 20); ++spin) {
    if (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == tag) { ok = true; break; }
    __builtin_amdgcn_s_sleep(8);
  }
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
  if (!ok && (threadIdx.x & 63) == 0) atomicOr(status, 1u);
  return ok;
}
// Eight 16-bit values read with device-scope loads: they bypass whatever this compute
// unit or this XCD's L2 may still hold for the address from an earlier launch.
__device__ inline u32x4_t load16_device(const uint16_t* p) {
  const uint32_t* q = (const uint32_t*)p;
  u32x4_t v;
  v[0] = __hip_atomic_load(q + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  v[1] = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  v[2] = __hip_atomic_load(q + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  v[3] = __hip_atomic_load(q + 3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return v;
}

template <int ACT, int MB, bool G128>
__global__ void __launch_bounds__(PfShape<ACT>::WAVES * 64, PfShape<ACT>::OCC) k_prefill(PrefillArgs a) {
  constexpr int PF_WAVES = PfShape<ACT>::WAVES, RB = PfShape<ACT>::RB;
  constexpr int MT = 16 * MB;          // tokens per workgroup tile
  constexpr int XR = PF_WAVES * 8;     // X rows covered by one load instruction of the workgroup
  constexpr int XI = MT / XR;          // 16-byte X loads per thread and stage
  constexpr int RW = G128 ? 272 : 288; // words per tile record
  // one stage = MT rows x 64 channels, 128 bytes per row, no padding; a ring of three:
  // the stage being read, the next one (landed or landing), the one after (landing)
  constexpr int NBUF = 3;
  constexpr uint32_t STAGE_BYTES = MT * 64 * 2;
  __shared__ __attribute__((aligned(1024))) uint16_t xs[NBUF * MT * 64];
  // per wave: its RB tile records of the next tile (1 KiB of words each, then 512 bytes
  // for their scale/zero words), landed here by the same kind of load and taken into
  // registers once per tile
  constexpr int WSTG = RB * 1024 + 512;
  __shared__ __attribute__((aligned(1024))) uint8_t wstage[PF_WAVES * WSTG];
  // set when a wave's bounded wait for the projection expired: then no wave of the
  // workgroup applies the correction
  __shared__ uint32_t corr_failed;

  if ((int)blockIdx.x < a.n_proj_wgs) {
    proj_tile<ACT, MB>(a, xs);
    return;
  }
  int mi = 0;
#pragma unroll
  for (int i = 1; i < PF_MAX_MODS; ++i)
    if (i < a.n_mods && (int)blockIdx.x >= a.mod[i].wg_start) mi = i;
  const PfModule& M = a.mod[mi];
  const PfUnit& U = a.unit[M.unit];
  // Workgroups go to the eight XCDs round robin and each XCD has an L2 of its own, so the
  // tiles that share operands should sit in one residue class of the workgroup index: class
  // c takes the c-th eighth of the module's tile list, and the list runs through panels of
  // PF_PANEL token tiles (row tile next, token tile within the panel fastest).  The 64
  // tiles an XCD holds at a time then cover 2 token tiles x 32 row tiles whatever T is.
  // Measured (bytes fetched past the L2 per launch, 2048 tokens x 22016 rows x 4096): panels
  // of 1 / 2 / 4 / 8 / 16 token tiles fetch 0.93 / 0.57 / 0.54 / 0.79 / 1.28 GB.  The rows
  // of X lie a whole row of K channels apart, and the more token tiles an XCD streams at
  // once the less of X survives in its L2 until the neighbour tile asks for it, while a
  // single token tile leaves nobody to share the weights with.  The time follows the
  // traffic only weakly (panel 16: +6 %).
  int mt, nt;
  {
    const int local = (int)blockIdx.x - M.wg_start;
    const int n_tiles = M.n_ntiles * U.n_mtiles;
    const int c = local & 7, q = local >> 3;
    const int t = c * (n_tiles >> 3) + min(c, n_tiles & 7) + q;
    const int per_panel = PF_PANEL * M.n_ntiles;
    const int panel = t / per_panel;
    const int width = min(PF_PANEL, U.n_mtiles - panel * PF_PANEL);
    const int tl = t - panel * per_panel;
    nt = __builtin_amdgcn_readfirstlane(tl / width);   // row tile within the module
    mt = __builtin_amdgcn_readfirstlane(panel * PF_PANEL + (tl - (tl / width) * width));
  }

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 15, kq = lane >> 4;
  const int ktiles = M.nkt;            // K tiles of this entry (all of them unless K is split)

  // this wave's four 16-row blocks; blocks past the module's last one are computed from
  // a clamped (valid) block and never stored, so that the hot loop carries no branch
  const int nb0 = nt * (PF_WAVES * RB) + RB * wave;
  const uint32_t* wt[RB];
#pragma unroll
  for (int b = 0; b < RB; ++b)
    wt[b] = uniform_ptr(M.rec + ((size_t)min(nb0 + b, M.rows16 - 1) * (U.K >> 7) + M.kt0) * RW);

  // X staging, global memory straight into LDS (no registers in between): the wave's
  // load i covers rows XR i + 8 wave + (lane >> 3), one 16-byte chunk per lane, 1 KiB
  // contiguous in LDS; lane (row, slot = lane & 7) fetches channel chunk
  // slot ^ ((row >> 1) & 7), which is what makes the operand reads conflict free.  Rows
  // past T re-read the last valid token (their columns of D are never stored).
  const int tok0 = mt * MT;
  // byte offsets of this thread's rows from the tile's first row (below 2^31: MT rows of
  // at most 2^16 channels)
  const uint16_t* xtile = uniform_ptr(U.X + (size_t)tok0 * U.K + (size_t)M.kt0 * 128);
  uint32_t xoff[XI];
#pragma unroll
  for (int i = 0; i < XI; ++i) {
    const int row = XR * i + (tid >> 3);
    const int chunk = (tid & 7) ^ ((row >> 1) & 7);
    xoff[i] = (uint32_t)(min(tok0 + row, U.T - 1) - tok0) * (uint32_t)U.K * 2u + chunk * 16;
  }
  const int nstages = 2 * ktiles;
  // stage indices past the end re-read the last stage into a ring slot nobody reads
  auto dma_x = [&](int stage, int slot, int i) {
    const int st = min(stage, nstages - 1);
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)((const char*)(xtile + st * 64) + xoff[i]),
        (__attribute__((address_space(3))) void*)(xs + slot * (MT * 64) + (XR * i + 8 * wave) * 64),
        16, 0, 0);
  };
  // The operand reads are issued as assembly, because the compiler orders every LDS
  // read it can see behind all LDS-bound loads in flight; so the waits are placed here
  // too: lds_read leaves its result pending, lds_wait<N> makes `v` usable once at most
  // N younger reads are outstanding (LDS reads of a wave return in order).
  const uint32_t xs_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)xs;
  // operand read: token row mb*16 + n, channel chunk c = 4 jj + kq
  const int rd_row = n * 64;                    // elements
  const int rd_sw = (n >> 1) & 7;
  const uint32_t rd_lane[2] = {xs_base + 2u * (uint32_t)(rd_row + (((0 + kq) ^ rd_sw) << 3)),
                               xs_base + 2u * (uint32_t)(rd_row + (((4 + kq) ^ rd_sw) << 3))};

  float4_t acc[RB][MB];
#pragma unroll
  for (int b = 0; b < RB; ++b)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) acc[b][mb] = float4_t{0.f, 0.f, 0.f, 0.f};

  u32x4_t wcur[RB];
  uint32_t szcur[RB][2];
  uint8_t* wmine = wstage + wave * WSTG;
  const uint32_t wmine_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)wmine;
  // one load per 16-row block for its 256 words (16 bytes per lane), and one (group size
  // 128: 16 scale/zero words per block, lane -> block lane >> 4) or two (group size 64: 32
  // words per block, lane -> block lane >> 5 of a pair) for the scale/zero words of all
  // RB blocks, every lane taking part, so that the loop carries no branch (lanes past the
  // last block fetch its words once more, into the unused tail of the stage)
  constexpr int SZB = G128 ? 64 : 128;     // bytes of scale/zero words per block in the stage
  constexpr int SZI = G128 ? 1 : 2;        // instructions that fetch them
  static_assert(RB <= 4, "the scale/zero loads cover four blocks");
  const uint32_t* szsrc[SZI];              // this lane's word of K tile 0, per instruction
#pragma unroll
  for (int j = 0; j < SZI; ++j) {
    const int rsel = G128 ? (lane >> 4) : 2 * j + (lane >> 5);
    const uint32_t* base = wt[0];
#pragma unroll
    for (int b = 1; b < RB; ++b) base = rsel >= b ? wt[b] : base;
    szsrc[j] = base + 256 + (G128 ? (lane & 15) : (lane & 31));
  }
  auto dma_w = [&](int kt, int b) {
    const int k = min(kt, ktiles - 1);
    const uint32_t* rec = wt[b] + (size_t)k * RW;
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)(rec + lane * 4),
        (__attribute__((address_space(3))) void*)(wmine + b * 1024), 16, 0, 0);
  };
  auto dma_sz = [&](int kt, int j) {
    const int k = min(kt, ktiles - 1);
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)(szsrc[j] + (size_t)k * RW),
        (__attribute__((address_space(3))) void*)(wmine + RB * 1024 + j * 256), 4, 0, 0);
  };
  constexpr int NWL = RB + SZI;            // load instructions per K tile of weights
  // LDS -> registers (the loads that filled the stage must have completed: vm_wait);
  // the results are pending until an lds wait
  const uint32_t wl16 = wmine_lds + lane * 16, wl4 = wmine_lds + RB * 1024 + n * 4;
  auto take_w = [&]() {
#pragma unroll
    for (int b = 0; b < RB; ++b) {
      lds_read(wcur[b], wl16, b * 1024);
      lds_read32(szcur[b][0], wl4, b * SZB);
      if (!G128) lds_read32(szcur[b][1], wl4, b * SZB + 64);
    }
  };
  auto tie_w = [&]() {
#pragma unroll
    for (int b = 0; b < RB; ++b) {
      after_wait(wcur[b]);
      after_wait32(szcur[b][0]);
      if (!G128) after_wait32(szcur[b][1]);
      else szcur[b][1] = szcur[b][0];
    }
  };
  // operand words of step j (32 channels) of the current tile, one per 16-row block
  u32x4_t wf[2][RB];
  GroupConst<ACT> g[RB];
  // the shorter binary16 recipe where its extra registers fit
  using DQ = std::conditional_t<ACT == ACT_F16 && G128, DequantLockstepF16Shiftless<RB>, DequantLockstep<ACT, RB>>;
  DQ dq;

  GLOWQ_STAMP(0);
  if (tid == 0) corr_failed = 0;       // ordered before its readers by the loop's barriers
#pragma unroll
  for (int i = 0; i < XI; ++i) dma_x(0, 0, i);
#pragma unroll
  for (int b = 0; b < RB; ++b) dma_w(0, b);
#pragma unroll
  for (int j = 0; j < SZI; ++j) dma_sz(0, j);
#pragma unroll
  for (int i = 0; i < XI; ++i) dma_x(1, 1, i);
  vm_wait<0>();
  take_w();
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  tie_w();
#pragma unroll
  for (int b = 0; b < RB; ++b) {
    g[b].set(szcur[b][0]);
    dq.set_group(b, g[b]);
    wf[0][b] = dequant_word<ACT>(wcur[b][0], g[b]);
  }
  __builtin_amdgcn_s_barrier();
  GLOWQ_STAMP(1);

  // The loop is software-pipelined over steps of 32 channels, and scheduled by hand in
  // slices of one matrix instruction each (32 per step, fenced so that the compiler
  // keeps them apart): behind product (b, mb) of step j rides one slice of the
  // dequantisation of the operand words of step j+1; the LDS reads of the X fragments
  // run XD token blocks ahead; the direct loads run two stages (X) and one tile (W)
  // ahead and sit in the first slices of a stage.
  int slot_cur = 0, slot_next2 = 2;   // ring slots of the stage being read and of stage+2
  for (int kt = 0; kt < ktiles; ++kt) {
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int stage = 2 * kt + half;
      // X fragment f = MB jj + mb of this stage: token block mb, channel chunk 4 jj + kq
      const uint32_t xa[2] = {rd_lane[0] + (uint32_t)slot_cur * STAGE_BYTES,
                              rd_lane[1] + (uint32_t)slot_cur * STAGE_BYTES};
      // operand fragments are read XD token blocks ahead of their use
      constexpr int XD = PfShape<ACT>::XD;
      u32x4_t xq[XD + 1];
#pragma unroll
      for (int f = 0; f < XD; ++f) lds_read(xq[f], xa[f / MB], (f % MB) * 2048);
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const int j = 2 * half + jj;
        const int jn = (j + 1) & 3;                        // the step being dequantised
        const bool new_group = G128 ? (j == 3) : ((j & 1) == 1);
        const u32x4_t (&wa)[RB] = wf[j & 1];
        u32x4_t (&wn)[RB] = wf[jn & 1];
#pragma unroll
        for (int i = 0; i < RB * MB; ++i) {
          const int mb = i / RB, b = i % RB;
          const int f = MB * jj + mb;
          // memory slots
          if (j == 3 && i == 0) {
            // the next tile's words: everything this wave has asked for has landed
            // (its loads of this stage come later), so take them out of the stage,
            // issue this slot's operand read, and wait for all but that one
            vm_wait<0>();
            take_w();
            lds_read(xq[(f + XD) % (XD + 1)], xa[(f + XD) / MB], ((f + XD) % MB) * 2048);
            lds_wait<1>(xq[f % (XD + 1)]);
            tie_w();
          } else if (b == 0) {
            if (f + XD < 2 * MB) {
              lds_read(xq[(f + XD) % (XD + 1)], xa[(f + XD) / MB], ((f + XD) % MB) * 2048);
              lds_wait<XD>(xq[f % (XD + 1)]);
            } else {
              // the tail of the stage: 2 MB - 1 - f younger reads are outstanding
              if (2 * MB - 1 - f == 3) lds_wait<3>(xq[f % (XD + 1)]);
              else if (2 * MB - 1 - f == 2) lds_wait<2>(xq[f % (XD + 1)]);
              else if (2 * MB - 1 - f == 1) lds_wait<1>(xq[f % (XD + 1)]);
              else lds_wait<0>(xq[f % (XD + 1)]);
            }
          }
          // X of stage+2: in the tile's first stage right away, in its second stage
          // behind the point where the next tile's weights are taken (which waits for
          // every load in flight, and these should not be among them)
          if (jj == half && i < XI) dma_x(stage + 2, slot_next2, i);
          // the next tile's records, into this wave's stage (free since the last take)
          if (j == 0 && i >= XI && i < XI + RB) dma_w(kt + 1, i - XI);
          if (j == 0 && i >= XI + RB && i < XI + NWL) dma_sz(kt + 1, i - XI - RB);
          // the product
          acc[b][mb] = mfma16<ACT>(wa[b], xq[f % (XD + 1)], acc[b][mb]);   // D[row][token]
          // its vector-ALU shadow: word i / 8 of the next step, slice i % 8
          // its vector-ALU shadow: the next instructions of the next step's dequantisation
          {
            constexpr int NS = RB * MB;
            constexpr int NO = DQ::N_OPS;
            if (i < RB && new_group) {
              g[i].set(szcur[i][G128 ? 0 : (jn >> 1)]);
              dq.set_group(i, g[i]);
            }
            // the first RB slots carry the group constants when a new group starts; the
            // recipe's instructions are spread evenly over the slots after them
            const int lo = i < RB ? 0 : ((i - RB) * NO) / (NS - RB);
            const int hi = i < RB ? 0 : ((i - RB + 1) * NO) / (NS - RB);
#pragma unroll
            for (int o = lo; o < hi; ++o)
              dq.op(o, wcur, jn, g, wn);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      // one barrier per stage: everyone is done reading this stage, and everyone's part
      // of the next stage has landed.  Vector-memory operations complete in order, and
      // the ones issued after the next stage's loads are the XI loads of the stage after
      // it plus one tile's NWL weight loads (issued in this stage or in the one before).
      {
        constexpr int YOUNGER = XI + NWL;
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(YOUNGER) : "memory");
      }
      __builtin_amdgcn_s_barrier();
      slot_cur = slot_cur == NBUF - 1 ? 0 : slot_cur + 1;
      slot_next2 = slot_next2 == NBUF - 1 ? 0 : slot_next2 + 1;
    }
  }
  // nothing of this workgroup may still be on its way into LDS when the workgroup ends
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  GLOWQ_STAMP(4);
  // correction: r more channels in stages of 64, operand [A_i] against [R].  The A words
  // do not depend on the projection and are asked for before its flag is looked at; the
  // R tile then takes the X path (straight into the idle ring, swizzled the same way,
  // with device-coherent loads: other compute units wrote it during this launch), so
  // that nothing in here waits for memory more than twice.
  if (U.restore && M.corr) {
    const int rstages = (U.r + 63) >> 6;                       // 1 or 2
    u32x4_t af[2][2][RB];
#pragma unroll
    for (int rs = 0; rs < 2; ++rs)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int b = 0; b < RB; ++b) {
          // ranks past r: operand words of rank 0 here, R words of a valid rank below,
          // and the product left out
          const int j0 = 64 * rs + 32 * jj + 8 * kq;
          const int row = min((nb0 + b) * 16 + n, M.d_out - 1);   // clamped like the tiles
          if (rs < rstages) vm_load(af[rs][jj][b], M.A + (size_t)row * U.r + (j0 < U.r ? j0 : 0));
        }
    const bool ready = wait_tile_ready(U.flags + MB * mt, U.status);
    if (!ready && lane == 0) atomicOr(&corr_failed, 1u);
    if (ready) {
      const uint16_t* rtile = uniform_ptr(U.R16 + (size_t)tok0 * U.r);
#pragma unroll
      for (int rs = 0; rs < 2; ++rs)
#pragma unroll
        for (int i = 0; i < XI; ++i) {
          const int row = XR * i + (tid >> 3);
          const int chunk = (tid & 7) ^ ((row >> 1) & 7);
          const int rank = min(64 * rs + 8 * chunk, U.r - 8);
          const uint32_t off = (uint32_t)((min(tok0 + row, U.T - 1) - tok0) * U.r + rank) * 2u;
          if (rs < rstages)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)((const char*)rtile + off),
                (__attribute__((address_space(3))) void*)(xs + rs * (MT * 64) + (XR * i + 8 * wave) * 64),
                16, 0, /*device scope*/ 16);
        }
    }
    vm_wait<0>();
#pragma unroll
    for (int rs = 0; rs < 2; ++rs)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int b = 0; b < RB; ++b)
          if (rs < rstages) after_wait(af[rs][jj][b]);
    __builtin_amdgcn_s_barrier();
    if (corr_failed == 0) {
#pragma unroll
      for (int rs = 0; rs < 2; ++rs) {
        if (rs < rstages) {
          const uint32_t xa[2] = {rd_lane[0] + (uint32_t)rs * STAGE_BYTES, rd_lane[1] + (uint32_t)rs * STAGE_BYTES};
          u32x4_t xq[3];
          lds_read(xq[0], xa[0], 0);
          lds_read(xq[1], xa[0], 2048);
#pragma unroll
          for (int f = 0; f < 2 * MB; ++f) {
            if (f + 2 < 2 * MB) {
              lds_read(xq[(f + 2) % 3], xa[(f + 2) / MB], ((f + 2) % MB) * 2048);
              lds_wait<2>(xq[f % 3]);
            } else if (f + 2 == 2 * MB) lds_wait<1>(xq[f % 3]);
            else lds_wait<0>(xq[f % 3]);
            const int jj = f / MB, mb = f % MB;
            if (64 * rs + 32 * jj < U.r) {           // uniform
#pragma unroll
              for (int b = 0; b < RB; ++b) {
                u32x4_t aw = af[rs][jj][b];
                if (64 * rs + 32 * jj + 8 * kq >= U.r) aw = u32x4_t{0u, 0u, 0u, 0u};
                acc[b][mb] = mfma16<ACT>(aw, xq[f % 3], acc[b][mb]);
              }
            }
          }
        }
      }
    }
  }

  GLOWQ_STAMP(5);
  // store: lane holds token (mb, n) and rows 4 kq + {0..3} of each 16-row block
#pragma unroll
  for (int b = 0; b < RB; ++b) {
    const int row = (nb0 + b) * 16 + 4 * kq;
    if (nb0 + b >= M.rows16 || row >= M.d_out) continue;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int tok = tok0 + mb * 16 + n;
      if (tok >= U.T) continue;
      const size_t off = (size_t)tok * M.ldy + row;
      const float4_t v = acc[b][mb];
      if (M.out_f32) {
        *(float4_t*)((float*)M.Y + off) = v;
      } else {
        uint2 pk;
        pk.x = (uint32_t)to_act16<ACT>(v[0]) | ((uint32_t)to_act16<ACT>(v[1]) << 16);
        pk.y = (uint32_t)to_act16<ACT>(v[2]) | ((uint32_t)to_act16<ACT>(v[3]) << 16);
        *(uint2*)((uint16_t*)M.Y + off) = pk;
      }
    }
  }
  GLOWQ_STAMP(6);
}

template <int ACT, int MB>
static hipError_t launch_prefill_t(const PrefillArgs& a, int n_wgs, int G, hipStream_t st) {
  dim3 grid((unsigned)n_wgs), block(PfShape<ACT>::WAVES * 64);
  if (G == 128) k_prefill<ACT, MB, true><<<grid, block, 0, st>>>(a);
  else k_prefill<ACT, MB, false><<<grid, block, 0, st>>>(a);
  return hipGetLastError();
}

static inline int prefill_mb(int T) { return T <= 64 ? 4 : 8; }

// Slices of K for a unit whose tiles would each run a long contraction while most of the chip
// idles: at least 8192 channels on at most 128 tiles (a quarter of the workgroups the chip
// holds), cut into slices of about 4096 channels, at most 4.  A unit's own shapes decide, so
// that its workspace can be planned without knowing what else shares the launch.  Measured
// on a block of 512 tokens (4096 / 14336 / 1024): the 64 tiles of the down projection, 3.5
// times the others' contraction each, set the launch's duration.
int prefill_k_slices(const glowq_unit& u) {
  if (u.T <= 64) return 1;
  const int ktiles = u.d_in / 128;
  if (ktiles < 64) return 1;
  const int tile_blocks = u.act_dtype == GLOWQ_F16 ? PfShape<ACT_F16>::TILE_BLOCKS : PfShape<ACT_BF16>::TILE_BLOCKS;
  const long long n_mtiles = (u.T + 127) / 128;
  long long tiles = 0;
  if (!u.modules) return 1;
  for (int i = 0; i < u.n_modules; ++i)
    tiles += (((u.modules[i].d_out + 15) / 16 + tile_blocks - 1) / tile_blocks) * n_mtiles;
  if (tiles > 128) return 1;
  return std::min(4, ktiles / 32);
}
// fp32 slab of one slice: [T][ldp], ldp = d_out rounded up to 4 (16-byte stores)
static inline size_t splitk_ldp(int d_out) { return (size_t)(d_out + 3) / 4 * 4; }
size_t prefill_splitk_bytes(const glowq_unit& u) {
  const int S = prefill_k_slices(u);
  if (S <= 1) return 0;
  size_t b = 0;
  for (int i = 0; i < u.n_modules; ++i) b += (size_t)S * u.T * splitk_ldp(u.modules[i].d_out) * 4;
  return b;
}

// Y[t][row] = sum over the slices' slabs, in slice order, rounded once to the output type
template <int ACT>
__global__ void k_splitk_sum(const float* __restrict__ P, int S, int T, int d_out, int ldp, void* Y, int ldy,
                             int out_f32) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;   // (token, 4 rows)
  const int per = ldp >> 2;
  if (idx >= (long long)T * per) return;
  const int t = (int)(idx / per), row = 4 * (int)(idx - (long long)t * per);
  float4_t v = *(const float4_t*)(P + (size_t)t * ldp + row);
  for (int sl = 1; sl < S; ++sl) {
    const float4_t q = *(const float4_t*)(P + ((size_t)sl * T + t) * ldp + row);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] += q[e];
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    if (row + e < d_out) {
      if (out_f32) ((float*)Y)[(size_t)t * ldy + row + e] = v[e];
      else ((uint16_t*)Y)[(size_t)t * ldy + row + e] = to_act16<ACT>(v[e]);
    }
  }
}

bool prefill_compatible(const glowq_unit& a, const glowq_unit& b) {
  return a.act_dtype == b.act_dtype && a.out_dtype == b.out_dtype &&
         a.group_size == b.group_size && prefill_mb(a.T) == prefill_mb(b.T);
}

int prefill_max_units() { return PF_MAX_UNITS; }
int prefill_max_modules() { return PF_MAX_MODS; }

// units[i] uses workspace slice ws[i]; restore[i] says whether its R16 is valid.
hipError_t launch_prefill_multi(const glowq_unit* const* units, const UnitWorkspace* ws,
                                const bool* restore, int n_units, bool allow_split, hipStream_t st) {
  PrefillArgs a;
  const glowq_unit& u0 = *units[0];
  const int MB = prefill_mb(u0.T);
  const int tile_blocks = u0.act_dtype == GLOWQ_F16 ? PfShape<ACT_F16>::TILE_BLOCKS
                                                    : PfShape<ACT_BF16>::TILE_BLOCKS;
  // longest contraction first
  int order[PF_MAX_UNITS];
  for (int i = 0; i < n_units; ++i) order[i] = i;
  for (int i = 1; i < n_units; ++i)
    for (int j = i; j > 0 && units[order[j]]->d_in > units[order[j - 1]]->d_in; --j) {
      int t = order[j]; order[j] = order[j - 1]; order[j - 1] = t;
    }
  // projection tiles of the restored units lead the grid
  int n_proj = 0;
  for (int oi = 0; oi < n_units; ++oi) {
    const int ui = order[oi];
    const glowq_unit& u = *units[ui];
    PfUnit& pu = a.unit[oi];
    const int n_mtiles = (u.T + 16 * MB - 1) / (16 * MB);
    pu.proj_start = -1;
    pu.parts = ws[ui].pf_parts;
    pu.part_stages = ws[ui].pf_part_stages;
    if (restore[ui] && u.r > 0) {
      pu.proj_start = n_proj;
      n_proj += n_mtiles * pu.parts;
    }
  }
  a.n_proj_wgs = n_proj;
  a.n_units = n_units;
  // K slices per unit: where the unit's shapes ask for them, its workspace has the slabs and
  // the module table has room
  int slices[PF_MAX_UNITS];
  {
    int total = 0;
    for (int ui = 0; ui < n_units; ++ui) total += units[ui]->n_modules;
    for (int ui = 0; ui < n_units; ++ui) {
      const glowq_unit& u = *units[ui];
      int S = (allow_split && ws[ui].base && ws[ui].splitk_bytes > 0) ? prefill_k_slices(u) : 1;
      if (total + (S - 1) * u.n_modules > PF_MAX_MODS) S = 1;
      total += (S - 1) * u.n_modules;
      slices[ui] = S;
    }
  }
  int n_mods = 0, wg = n_proj;
  for (int oi = 0; oi < n_units; ++oi) {
    const int ui = order[oi];
    const glowq_unit& u = *units[ui];
    PfUnit& pu = a.unit[oi];
    pu.X = (const uint16_t*)u.X;
    pu.B = (const uint16_t*)u.B;
    // (a call without any restored unit may come without a workspace)
    char* wsb = ws[ui].base;
    pu.R16 = wsb ? (uint16_t*)(wsb + ws[ui].off_r16) : nullptr;
    pu.Rpart = wsb ? (float*)(wsb + ws[ui].off_rpart) : nullptr;
    pu.flags = wsb ? (uint32_t*)(wsb + ws[ui].off_counters) : nullptr;
    pu.status = wsb ? &((Control*)wsb)->status : nullptr;
    pu.T = u.T;
    pu.K = u.d_in;
    pu.r = u.r;
    pu.restore = (restore[ui] && u.r > 0) ? 1 : 0;
    pu.n_mtiles = (u.T + 16 * MB - 1) / (16 * MB);
    const int S = slices[ui], ktiles = u.d_in / 128;
    float* slab = (S > 1) ? (float*)(wsb + ws[ui].off_splitk) : nullptr;
    for (int i = 0; i < u.n_modules; ++i) {
      const glowq_module& m = u.modules[i];
      PreparedView v = prepared_view(m.w_prepared, m.d_out, u.d_in, u.group_size);
      for (int sl = 0; sl < S; ++sl) {
        PfModule& pm = a.mod[n_mods++];
        pm.rec = v.base;
        pm.A = (const uint16_t*)m.A;
        pm.d_out = m.d_out;
        pm.rows16 = v.rows16;
        pm.unit = oi;
        pm.wg_start = wg;
        pm.n_ntiles = (v.rows16 + tile_blocks - 1) / tile_blocks;
        pm.kt0 = (int)((long long)ktiles * sl / S);
        pm.nkt = (int)((long long)ktiles * (sl + 1) / S) - pm.kt0;
        pm.corr = sl == 0;
        if (S > 1) {
          const size_t ldp = splitk_ldp(m.d_out);
          pm.Y = slab + (size_t)sl * u.T * ldp;
          pm.ldy = (int)ldp;
          pm.out_f32 = 1;
        } else {
          pm.Y = m.Y;
          pm.ldy = m.ldy;
          pm.out_f32 = (u.out_dtype == GLOWQ_F32) ? 1 : 0;
        }
        wg += pu.n_mtiles * pm.n_ntiles;
      }
      if (S > 1) slab += (size_t)S * u.T * splitk_ldp(m.d_out);
    }
  }
  for (int i = n_units; i < PF_MAX_UNITS; ++i) a.unit[i] = a.unit[0];
  for (int i = n_mods; i < PF_MAX_MODS; ++i) a.mod[i] = a.mod[0];
  a.n_mods = n_mods;
  a.out_f32 = (u0.out_dtype == GLOWQ_F32) ? 1 : 0;
  const bool f16 = (u0.act_dtype == GLOWQ_F16);
  hipError_t err;
  if (MB == 4)
    err = f16 ? launch_prefill_t<ACT_F16, 4>(a, wg, u0.group_size, st)
              : launch_prefill_t<ACT_BF16, 4>(a, wg, u0.group_size, st);
  else
    err = f16 ? launch_prefill_t<ACT_F16, 8>(a, wg, u0.group_size, st)
              : launch_prefill_t<ACT_BF16, 8>(a, wg, u0.group_size, st);
  if (err != hipSuccess) return err;
  // the sliced units' outputs
  for (int ui = 0; ui < n_units; ++ui) {
    const int S = slices[ui];
    if (S <= 1) continue;
    const glowq_unit& u = *units[ui];
    const float* slab = (const float*)(ws[ui].base + ws[ui].off_splitk);
    for (int i = 0; i < u.n_modules; ++i) {
      const glowq_module& m = u.modules[i];
      const int ldp = (int)splitk_ldp(m.d_out);
      const long long n = (long long)u.T * (ldp / 4);
      dim3 grid((unsigned)((n + 255) / 256)), block(256);
      const int of32 = u.out_dtype == GLOWQ_F32 ? 1 : 0;
      if (f16) k_splitk_sum<ACT_F16><<<grid, block, 0, st>>>(slab, S, u.T, m.d_out, ldp, m.Y, m.ldy, of32);
      else k_splitk_sum<ACT_BF16><<<grid, block, 0, st>>>(slab, S, u.T, m.d_out, ldp, m.Y, m.ldy, of32);
      slab += (size_t)S * u.T * ldp;
    }
  }
  return hipGetLastError();
}

}  // namespace glowq

GLOWQ_TRACE_EXPORT(glowq_debug_trace_prefill)
