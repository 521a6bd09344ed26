// C ABI of the GlowQ group forward (declared in include/glowq.h): host-side
// argument checks, workspace planning and dispatch to the HIP kernels.  Nothing in
// this file allocates, synchronises or keeps state.
#include <algorithm>
#include <mutex>
#include <vector>
#include "common.hpp"
#include "launch.hpp"

namespace glowq {

// Scratch of glowq_group_forward_static: one array per GPU, held until the process ends.
// In host code the array's name is only a stand-in; its device address comes from
// hipGetSymbolAddress, once per device, and is what every launch is given.
static __device__ __align__(256) unsigned char g_static_scratch[GLOWQ_STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
static void* g_static_scratch_ptr[MAX_DEVICES];
static std::mutex g_static_scratch_mutex;

// device address of the current device's scratch array (null + error code on failure)
static hipError_t static_scratch(void** out) {
  *out = nullptr;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
  if (!g_static_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_static_scratch_ptr[dev] = p;
  }
  *out = g_static_scratch_ptr[dev];
  return hipSuccess;
}

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

UnitWorkspace plan_unit_workspace(const glowq_unit& u, char* base) {
  UnitWorkspace w;
  w.base = base;
  const int tblocks = (u.T + 15) / 16;
  w.off_counters = sizeof(Control);
  // (one word more than blocks: the arrival counter of a last tile of a single block)
  w.ctl_bytes = align_up(w.off_counters + (size_t)(tblocks + 1) * 4, 256);
  // K slices of the projection: prefill already has T / 16 token blocks and only needs
  // enough slices to fill the chip
  // (a handful of tokens: one wave per (rank, part) and parts of about 2048 channels, so
  // that a wave has all its loads in flight at once, at most four parts; up to 32 tokens:
  // four slices, two workgroups each (one per half of the ranks); the consumers add the
  // parts themselves)
  const bool direct = u.T <= 4;
  int ksplit = direct ? (u.d_in + 2047) / 2048 : is_decode(u.T) ? 4 : (256 + tblocks - 1) / tblocks;
  if (direct && ksplit > 4) ksplit = 4;
  if (ksplit > 32) ksplit = 32;
  if (ksplit < 1) ksplit = 1;
  int steps = u.d_in / 32;
  int per = (steps + ksplit - 1) / ksplit;
  w.kslice = per * 32;
  w.ksplit = (u.d_in + w.kslice - 1) / w.kslice;
  w.kstride = (w.ksplit + 3) / 4 * 4;
  // T > 32: the projection tiles that lead the GEMM launch take parts of about 2048
  // channels (at most 8), so that the longest contraction's R is ready as early as the
  // shortest one's
  const int stages = u.d_in / 64;
  int parts = (u.d_in + 2047) / 2048;
  if (parts > 8) parts = 8;
  w.pf_part_stages = (stages + parts - 1) / parts;
  w.pf_parts = (stages + w.pf_part_stages - 1) / w.pf_part_stages;
  w.off_rpart = w.ctl_bytes;
  // (T > 32: room for eight slices, which is what the stand-alone projection uses)
  int slabs = is_decode(u.T) ? w.kstride : (w.kstride > w.pf_parts ? w.kstride : w.pf_parts);
  if (!is_decode(u.T) && slabs < 8) slabs = 8;
  size_t rpart = (u.r > 0) ? (size_t)slabs * u.T * u.r * (is_decode(u.T) ? 8 : 4) : 0;
  w.off_r16 = align_up(w.off_rpart + rpart, 256);
  size_t r16 = (u.r > 0) ? (size_t)u.T * u.r * 2 : 0;
  w.off_splitk = align_up(w.off_r16 + r16, 256);
  w.splitk_bytes = is_decode(u.T) ? 0 : prefill_splitk_bytes(u);
  w.bytes = align_up(w.off_splitk + w.splitk_bytes, 256);
  return w;
}

// Sizes of one module's weights.  ERR_SHAPE: the sizes contradict the W4A16 storage
// format itself (no such group size, d_in not a whole number of groups, nothing to do);
// ERR_UNSUPPORTED: a well-formed request that the tile layout of this build cannot hold
// (d_in not a multiple of the 128-channel tile, d_out not a multiple of 8).
static glowq_status check_weights_shape(int d_out, int d_in, int G) {
  if (G != 64 && G != 128) return GLOWQ_ERR_SHAPE;
  if (d_in < G || d_in > (1 << 16) || d_in % G) return GLOWQ_ERR_SHAPE;
  if (d_out < 1 || d_out > (1 << 20)) return GLOWQ_ERR_SHAPE;
  if (d_in % 128 || d_out % 8) return GLOWQ_ERR_UNSUPPORTED;
  return GLOWQ_OK;
}

// ptrs: also check the pointers; corrected: the unit's correction will be applied (a unit
// that is masked off, or has r == 0, needs neither B nor any A_i)
static glowq_status validate(const glowq_unit* u, bool ptrs, bool corrected) {
  if (!u) return GLOWQ_ERR_NULL;
  if (u->n_modules < 1 || u->n_modules > GLOWQ_MAX_MODULES) return GLOWQ_ERR_SHAPE;
  if (ptrs && !u->modules) return GLOWQ_ERR_NULL;
  if (u->T < 1 || u->T > (1 << 20)) return GLOWQ_ERR_SHAPE;
  if (u->group_size != 64 && u->group_size != 128) return GLOWQ_ERR_SHAPE;
  if (u->d_in < u->group_size || u->d_in > (1 << 16) || u->d_in % u->group_size) return GLOWQ_ERR_SHAPE;
  if (u->r < 0) return GLOWQ_ERR_SHAPE;
  if (u->act_dtype != GLOWQ_F16 && u->act_dtype != GLOWQ_BF16) return GLOWQ_ERR_DTYPE;
  if (u->out_dtype != u->act_dtype && u->out_dtype != GLOWQ_F32) return GLOWQ_ERR_DTYPE;
  if (u->modules)
    for (int i = 0; i < u->n_modules; ++i) {
      const glowq_module& m = u->modules[i];
      if (m.d_out < 1 || m.d_out > (1 << 20) || m.ldy < m.d_out) return GLOWQ_ERR_SHAPE;
    }
  // well-formed from here on; what this build cannot serve
  if (u->d_in % 128 || u->r > GLOWQ_MAX_RANK || u->r % 8) return GLOWQ_ERR_UNSUPPORTED;
  if (!u->modules) return GLOWQ_OK;   // shapes only
  for (int i = 0; i < u->n_modules; ++i) {
    const glowq_module& m = u->modules[i];
    if (m.d_out % 8 || m.ldy % 8) return GLOWQ_ERR_UNSUPPORTED;
  }
  if (!ptrs) return GLOWQ_OK;
  const bool need_factors = corrected && u->r > 0;
  if (!u->X || (need_factors && !u->B)) return GLOWQ_ERR_NULL;
  for (int i = 0; i < u->n_modules; ++i) {
    const glowq_module& m = u->modules[i];
    if (!m.w_prepared || !m.Y || (need_factors && !m.A)) return GLOWQ_ERR_NULL;
  }
  if (misaligned(u->X) || (need_factors && misaligned(u->B))) return GLOWQ_ERR_ALIGN;
  for (int i = 0; i < u->n_modules; ++i) {
    const glowq_module& m = u->modules[i];
    if (misaligned(m.w_prepared) || misaligned(m.Y) || (need_factors && misaligned(m.A)))
      return GLOWQ_ERR_ALIGN;
  }
  return GLOWQ_OK;
}

static thread_local hipError_t g_last_hip_error = hipSuccess;
static inline glowq_status hip_status(hipError_t e) {
  if (e == hipSuccess) return GLOWQ_OK;
  g_last_hip_error = e;
  return GLOWQ_ERR_HIP;
}

// Enqueue all units: decode-sized units one launch each (projection inside); prefill-sized
// units in batches of compatible neighbours, projections first, then one GEMM launch.
static glowq_status forward_all(const glowq_unit* units, int n_units, const uint8_t* mask,
                                char* workspace, hipStream_t st, bool allow_split = true) {
  size_t off = 0;
  int i = 0;
  while (i < n_units) {
    const glowq_unit& u = units[i];
    if (is_decode(u.T)) {
      // consecutive few-token units of one kind share a launch
      const glowq_unit* dbatch[32];
      UnitWorkspace dws[32];
      bool dcorr[32];
      int nd = 0;
      while (i < n_units && nd < decode_max_batch() && nd < 32 && is_decode(units[i].T) &&
             (nd == 0 || decode_batch_compatible(*dbatch[0], units[i]))) {
        dbatch[nd] = &units[i];
        dws[nd] = plan_unit_workspace(units[i], workspace ? workspace + off : nullptr);
        dcorr[nd] = (!mask || mask[i]) && units[i].r > 0;
        off += dws[nd].bytes;
        ++nd;
        ++i;
      }
      hipError_t e = launch_decode_multi(dbatch, dws, dcorr, nd, st);
      if (e != hipSuccess) return hip_status(e);
      continue;
    }
    const glowq_unit* batch[8];
    UnitWorkspace bws[8];
    bool corr[8];
    int nb = 0, nmods = 0;
    while (i < n_units && nb < prefill_max_units() && nb < 8 && !is_decode(units[i].T) &&
           (nb == 0 || prefill_compatible(*batch[0], units[i])) &&
           nmods + units[i].n_modules <= prefill_max_modules()) {
      batch[nb] = &units[i];
      bws[nb] = plan_unit_workspace(units[i], workspace ? workspace + off : nullptr);
      corr[nb] = (!mask || mask[i]) && units[i].r > 0;
      off += bws[nb].bytes;
      nmods += units[i].n_modules;
      ++nb;
      ++i;
    }
    // (the projections of the batch run as the first tiles of the same launch)
    hipError_t e = launch_prefill_multi(batch, bws, corr, nb, allow_split && workspace != nullptr, st);
    if (e != hipSuccess) return hip_status(e);
  }
  return GLOWQ_OK;
}

}  // namespace glowq

using namespace glowq;

extern "C" {

const char* glowq_status_string(glowq_status s) {
  switch (s) {
    case GLOWQ_OK: return "ok";
    case GLOWQ_ERR_NULL: return "required pointer is NULL";
    case GLOWQ_ERR_SHAPE: return "size out of range or inconsistent";
    case GLOWQ_ERR_ALIGN: return "device pointer or stride misaligned";
    case GLOWQ_ERR_DTYPE: return "unsupported data type";
    case GLOWQ_ERR_UNSUPPORTED: return "unsupported request";
    case GLOWQ_ERR_WORKSPACE: return "workspace missing or too small";
    case GLOWQ_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

const char* glowq_last_hip_error(void) { return hipGetErrorString(g_last_hip_error); }

glowq_status glowq_validate_unit(const glowq_unit* u, int32_t check_pointers) {
  return validate(u, check_pointers != 0, true);
}

glowq_status glowq_prepared_bytes(int32_t d_out, int32_t d_in, int32_t group_size, size_t* bytes) {
  if (!bytes) return GLOWQ_ERR_NULL;
  glowq_status s = check_weights_shape(d_out, d_in, group_size);
  if (s != GLOWQ_OK) return s;
  *bytes = prepared_total_bytes(d_out, d_in, group_size);
  return GLOWQ_OK;
}

glowq_status glowq_prepare_weights(const uint32_t* wq, const uint16_t* scales,
                                   const uint16_t* zeros, int32_t d_out, int32_t d_in,
                                   int32_t group_size, void* w_prepared, void* stream) {
  if (!wq || !scales || !zeros || !w_prepared) return GLOWQ_ERR_NULL;
  glowq_status s = check_weights_shape(d_out, d_in, group_size);
  if (s != GLOWQ_OK) return s;
  if (misaligned(wq) || misaligned(scales) || misaligned(zeros) || misaligned(w_prepared))
    return GLOWQ_ERR_ALIGN;
  return hip_status(launch_prepare(wq, scales, zeros, d_out, d_in, group_size, w_prepared,
                                   (hipStream_t)stream));
}

glowq_status glowq_workspace_bytes(const glowq_unit* units, int32_t n_units, size_t* bytes) {
  if (!units || !bytes) return GLOWQ_ERR_NULL;
  if (n_units < 1) return GLOWQ_ERR_SHAPE;
  size_t total = 0;
  for (int i = 0; i < n_units; ++i) {
    glowq_status s = validate(&units[i], false, false);
    if (s != GLOWQ_OK) return s;
    total += plan_unit_workspace(units[i], nullptr).bytes;
  }
  *bytes = total;
  return GLOWQ_OK;
}

glowq_status glowq_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
  if (!workspace) return GLOWQ_ERR_NULL;
  if (misaligned(workspace)) return GLOWQ_ERR_ALIGN;
  if (workspace_bytes % 4) return GLOWQ_ERR_SHAPE;
  return hip_status(launch_fill_zero(workspace, workspace_bytes, (hipStream_t)stream));
}

glowq_status glowq_workspace_status(const glowq_unit* units, int32_t n_units,
                                    const void* workspace, size_t workspace_bytes,
                                    uint32_t* failed_units, void* stream) {
  if (!units || !workspace || !failed_units) return GLOWQ_ERR_NULL;
  if (n_units < 1) return GLOWQ_ERR_SHAPE;
  if (misaligned(workspace) || ((uintptr_t)failed_units & 3u)) return GLOWQ_ERR_ALIGN;
  size_t need = 0;
  for (int i = 0; i < n_units; ++i) {
    glowq_status s = validate(&units[i], false, false);
    if (s != GLOWQ_OK) return s;
    need += plan_unit_workspace(units[i], nullptr).bytes;
  }
  if (workspace_bytes < need || (need >> 8) > 0xffffffffull) return GLOWQ_ERR_WORKSPACE;
  size_t off = 0;
  bool first = true;
  for (int i0 = 0; i0 < n_units; i0 += STATUS_BATCH) {
    StatusBatch b;
    b.n = n_units - i0 < STATUS_BATCH ? n_units - i0 : STATUS_BATCH;
    for (int i = 0; i < STATUS_BATCH; ++i) {
      b.off256[i] = (uint32_t)(off >> 8);
      if (i < b.n) off += plan_unit_workspace(units[i0 + i], nullptr).bytes;
    }
    hipError_t e = launch_status_count(workspace, b, first, failed_units, (hipStream_t)stream);
    if (e != hipSuccess) return hip_status(e);
    first = false;
  }
  return GLOWQ_OK;
}

glowq_status glowq_shared_proj(const glowq_unit* u, float* R_out, void* workspace,
                               size_t workspace_bytes, void* stream) {
  glowq_status s = validate(u, true, true);
  if (s != GLOWQ_OK) return s;
  if (u->r == 0) return GLOWQ_ERR_SHAPE;
  if (!R_out) return GLOWQ_ERR_NULL;
  if (misaligned(R_out)) return GLOWQ_ERR_ALIGN;
  if (!workspace) return GLOWQ_ERR_WORKSPACE;
  if (misaligned(workspace)) return GLOWQ_ERR_ALIGN;
  UnitWorkspace ws = plan_unit_workspace(*u, (char*)workspace);
  if (workspace_bytes < ws.bytes) return GLOWQ_ERR_WORKSPACE;
  return hip_status(launch_proj(*u, ws, R_out, false, (hipStream_t)stream));
}

glowq_status glowq_group_forward(const glowq_unit* u, int32_t restore, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  uint8_t mask = restore ? 1 : 0;
  return glowq_block_forward(u, 1, &mask, workspace, workspace_bytes, stream);
}

glowq_status glowq_group_forward_static(const glowq_unit* u, int32_t restore, void* stream) {
  const bool corrected = u && u->r > 0 && restore;
  glowq_status s = validate(u, true, corrected);
  if (s != GLOWQ_OK) return s;
  uint8_t mask = restore ? 1 : 0;
  if (!corrected) return forward_all(u, 1, &mask, nullptr, (hipStream_t)stream);
  // (the static array holds the projection's words; a long contraction is not cut here)
  const UnitWorkspace plan = plan_unit_workspace(*u, nullptr);
  if (plan.off_splitk > (size_t)GLOWQ_STATIC_SCRATCH_BYTES) return GLOWQ_ERR_WORKSPACE;
  void* scratch = nullptr;
  hipError_t e = static_scratch(&scratch);
  if (e != hipSuccess) return hip_status(e);
  // the array keeps the last call's contents, laid out for that call's unit: the control
  // and flag words of THIS unit's layout must start at zero (a fill kernel, not a memset
  // node, so that the call can be captured into a graph)
  e = launch_fill_zero(scratch, plan.ctl_bytes, (hipStream_t)stream);
  if (e != hipSuccess) return hip_status(e);
  return forward_all(u, 1, &mask, (char*)scratch, (hipStream_t)stream, false);
}

glowq_status glowq_block_forward(const glowq_unit* units, int32_t n_units,
                                 const uint8_t* restore_mask, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  if (!units) return GLOWQ_ERR_NULL;
  if (n_units < 1) return GLOWQ_ERR_SHAPE;
  // check everything before anything is enqueued
  size_t need = 0;
  bool any_corr = false;
  for (int i = 0; i < n_units; ++i) {
    const bool corrected = units[i].r > 0 && (!restore_mask || restore_mask[i]);
    glowq_status s = validate(&units[i], true, corrected);
    if (s != GLOWQ_OK) return s;
    need += plan_unit_workspace(units[i], nullptr).bytes;
    if (corrected) any_corr = true;
  }
  if (any_corr) {
    if (!workspace) return GLOWQ_ERR_WORKSPACE;
    if (misaligned(workspace)) return GLOWQ_ERR_ALIGN;
    if (workspace_bytes < need) return GLOWQ_ERR_WORKSPACE;
  }
  return forward_all(units, n_units, restore_mask, (char*)workspace, (hipStream_t)stream);
}

// Every module of the units as a one-module unit, module j (counted over all units) with
// B_modules[j], or with its unit's own B when B_modules is null (sizing only).
static glowq_status split_into_solo_units(const glowq_unit* units, int n_units,
                                          const void* const* B_modules,
                                          std::vector<glowq_unit>& solo) {
  for (int i = 0; i < n_units; ++i) {
    // the shape first, so that n_modules can be trusted
    glowq_status s = validate(&units[i], false, false);
    if (s != GLOWQ_OK) return s;
    if (units[i].r < 1) return GLOWQ_ERR_SHAPE;
    for (int m = 0; m < units[i].n_modules; ++m) {
      glowq_unit v = units[i];
      v.modules = units[i].modules ? &units[i].modules[m] : nullptr;
      v.n_modules = 1;
      if (B_modules) {
        v.B = B_modules[solo.size()];
        if (!v.B) return GLOWQ_ERR_NULL;
      }
      solo.push_back(v);
    }
  }
  return GLOWQ_OK;
}

glowq_status glowq_layerwise_workspace_bytes(const glowq_unit* units, int32_t n_units,
                                             size_t* bytes) {
  if (!units || !bytes) return GLOWQ_ERR_NULL;
  if (n_units < 1) return GLOWQ_ERR_SHAPE;
  std::vector<glowq_unit> solo;
  glowq_status s = split_into_solo_units(units, n_units, nullptr, solo);
  if (s != GLOWQ_OK) return s;
  return glowq_workspace_bytes(solo.data(), (int32_t)solo.size(), bytes);
}

glowq_status glowq_layerwise_forward(const glowq_unit* units, int32_t n_units,
                                     const void* const* B_modules, void* workspace,
                                     size_t workspace_bytes, void* stream) {
  if (!units || !B_modules) return GLOWQ_ERR_NULL;
  if (n_units < 1) return GLOWQ_ERR_SHAPE;
  for (int i = 0; i < n_units; ++i)
    if (!units[i].modules) return GLOWQ_ERR_NULL;
  std::vector<glowq_unit> solo;
  glowq_status s = split_into_solo_units(units, n_units, B_modules, solo);
  if (s != GLOWQ_OK) return s;
  return glowq_block_forward(solo.data(), (int32_t)solo.size(), nullptr, workspace,
                             workspace_bytes, stream);
}

glowq_status glowq_unit_importance(const glowq_unit* u, const float* const* W_modules,
                                   void* scratch, double* scores, void* stream) {
  if (!u || !W_modules || !scratch || !scores) return GLOWQ_ERR_NULL;
  glowq_status s = validate(u, false, false);
  if (s != GLOWQ_OK) return s;
  if (!u->modules) return GLOWQ_ERR_NULL;
  static_assert(GLOWQ_IMPORTANCE_SCRATCH_BYTES >= (2 + 3 * GLOWQ_MAX_RANK) * sizeof(double), "scratch layout");
  if (((uintptr_t)scratch & 7u) || ((uintptr_t)scores & 7u)) return GLOWQ_ERR_ALIGN;
  if (u->r > 0 && (!u->B || misaligned(u->B))) return u->B ? GLOWQ_ERR_ALIGN : GLOWQ_ERR_NULL;
  for (int i = 0; i < u->n_modules; ++i) {
    const glowq_module& m = u->modules[i];
    if (!W_modules[i] || !m.w_prepared || (u->r > 0 && !m.A)) return GLOWQ_ERR_NULL;
    if (misaligned(W_modules[i]) || misaligned(m.w_prepared) || (u->r > 0 && misaligned(m.A)))
      return GLOWQ_ERR_ALIGN;
  }
  return hip_status(launch_importance(*u, W_modules, (double*)scratch, scores, (hipStream_t)stream));
}

glowq_status glowq_select_units(const double* scores, int32_t n_units, int32_t k,
                                uint8_t* restore_mask) {
  if (!scores || !restore_mask) return GLOWQ_ERR_NULL;
  if (n_units < 1 || k < 0) return GLOWQ_ERR_SHAPE;
  std::vector<int> order(n_units);
  for (int i = 0; i < n_units; ++i) order[i] = i;
  // highest score first; equal scores keep their index order
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return scores[a] > scores[b]; });
  for (int i = 0; i < n_units; ++i) restore_mask[i] = 0;
  for (int i = 0; i < k && i < n_units; ++i) restore_mask[order[i]] = 1;
  return GLOWQ_OK;
}

glowq_status glowq_quantize_rtn(const float* W, int32_t d_out, int32_t d_in, int32_t group_size,
                                uint32_t* wq, uint16_t* scales, uint16_t* zeros, void* stream) {
  if (!W || !wq || !scales || !zeros) return GLOWQ_ERR_NULL;
  glowq_status s = check_weights_shape(d_out, d_in, group_size);
  if (s != GLOWQ_OK) return s;
  if (misaligned(W) || misaligned(wq) || misaligned(scales) || misaligned(zeros)) return GLOWQ_ERR_ALIGN;
  return hip_status(launch_quantize_rtn(W, d_out, d_in, group_size, wq, scales, zeros, (hipStream_t)stream));
}

static glowq_status check_factorize(const glowq_unit* u, int32_t r, int32_t p, int32_t q) {
  glowq_status s = validate(u, false, false);
  if (s != GLOWQ_OK) return s;
  if (!u->modules) return GLOWQ_ERR_NULL;
  if (r < 1 || p < 0 || q < 0) return GLOWQ_ERR_SHAPE;
  long long m = 0;
  for (int i = 0; i < u->n_modules; ++i) m += u->modules[i].d_out;
  if (r > m || r + p > u->d_in) return GLOWQ_ERR_SHAPE;      // more directions than the stack has
  if (r > GLOWQ_MAX_RANK || r % 8 || r + p > GLOWQ_MAX_SKETCH || q > GLOWQ_MAX_POWER_STEPS ||
      m > (1 << 20))
    return GLOWQ_ERR_UNSUPPORTED;
  return GLOWQ_OK;
}

glowq_status glowq_factorize_workspace_bytes(const glowq_unit* u, int32_t r, int32_t p, size_t* bytes) {
  if (!u || !bytes) return GLOWQ_ERR_NULL;
  glowq_status s = check_factorize(u, r, p, 0);
  if (s != GLOWQ_OK) return s;
  *bytes = plan_factorize(*u, r, p).bytes;
  return GLOWQ_OK;
}

glowq_status glowq_factorize_unit(const glowq_unit* u, const float* const* W_modules,
                                  const double* sigma_x_diag, int32_t r, int32_t p, int32_t q,
                                  const double* Omega, void* workspace, size_t workspace_bytes,
                                  void* const* A_out, void* B_out, double* sigma_out, void* stream) {
  if (!u || !W_modules || !Omega || !A_out || !B_out) return GLOWQ_ERR_NULL;
  glowq_status s = check_factorize(u, r, p, q);
  if (s != GLOWQ_OK) return s;
  if (!workspace || workspace_bytes < plan_factorize(*u, r, p).bytes) return GLOWQ_ERR_WORKSPACE;
  if (((uintptr_t)workspace & 255u) || ((uintptr_t)Omega & 7u) || ((uintptr_t)sigma_x_diag & 7u) ||
      ((uintptr_t)sigma_out & 7u) || misaligned(B_out))
    return GLOWQ_ERR_ALIGN;
  for (int i = 0; i < u->n_modules; ++i) {
    if (!W_modules[i] || !u->modules[i].w_prepared || !A_out[i]) return GLOWQ_ERR_NULL;
    if (misaligned(W_modules[i]) || misaligned(u->modules[i].w_prepared) || misaligned(A_out[i]))
      return GLOWQ_ERR_ALIGN;
  }
  return hip_status(launch_factorize(*u, W_modules, sigma_x_diag, r, p, q, Omega, (char*)workspace,
                                     A_out, B_out, sigma_out, (hipStream_t)stream));
}

// ---- microscaling variant ----------------------------------------------------------------
static glowq_status check_mx_weights_shape(int d_out, int d_in) {
  if (d_in < 32 || d_in > (1 << 16) || d_in % 32) return GLOWQ_ERR_SHAPE;     // whole MX blocks
  if (d_out < 1 || d_out > (1 << 20)) return GLOWQ_ERR_SHAPE;
  if (d_in % 128 || d_out % 8) return GLOWQ_ERR_UNSUPPORTED;
  return GLOWQ_OK;
}

glowq_status glowq_mx_prepared_bytes(int32_t d_out, int32_t d_in, size_t* bytes) {
  if (!bytes) return GLOWQ_ERR_NULL;
  glowq_status s = check_mx_weights_shape(d_out, d_in);
  if (s != GLOWQ_OK) return s;
  *bytes = mx_prepared_bytes(d_out, d_in);
  return GLOWQ_OK;
}

glowq_status glowq_mx_prepare_weights(const uint32_t* codes, const uint8_t* scales, int32_t d_out,
                                      int32_t d_in, void* w_prepared, void* stream) {
  if (!codes || !scales || !w_prepared) return GLOWQ_ERR_NULL;
  glowq_status s = check_mx_weights_shape(d_out, d_in);
  if (s != GLOWQ_OK) return s;
  if (misaligned(codes) || misaligned(w_prepared)) return GLOWQ_ERR_ALIGN;
  return hip_status(launch_mx_prepare(codes, scales, d_out, d_in, w_prepared, (hipStream_t)stream));
}

glowq_status glowq_mx_quantize_activations(const void* X, int32_t T, int32_t d_in, int32_t act_dtype,
                                           uint8_t* codes, uint8_t* scales, void* stream) {
  if (!X || !codes || !scales) return GLOWQ_ERR_NULL;
  if (T < 1 || T > (1 << 20) || d_in < 32 || d_in > (1 << 16) || d_in % 32) return GLOWQ_ERR_SHAPE;
  if (act_dtype != GLOWQ_F16 && act_dtype != GLOWQ_BF16) return GLOWQ_ERR_DTYPE;
  if (misaligned(X) || misaligned(codes)) return GLOWQ_ERR_ALIGN;
  return hip_status(launch_mx_quantize_x(X, T, d_in, act_dtype, codes, scales, false, (hipStream_t)stream));
}

// the unit checks of the ordinary forward without its group size (MX blocks are 32 channels)
static glowq_status validate_mx(const glowq_unit* u, bool ptrs, bool corrected) {
  if (!u) return GLOWQ_ERR_NULL;
  glowq_unit v = *u;
  v.group_size = 128;
  glowq_status s = validate(&v, ptrs, corrected);
  return s;
}

glowq_status glowq_mx_workspace_bytes(const glowq_unit* u, size_t* bytes) {
  if (!u || !bytes) return GLOWQ_ERR_NULL;
  glowq_status s = validate_mx(u, false, false);
  if (s != GLOWQ_OK) return s;
  *bytes = plan_mx_workspace(*u).bytes;
  return GLOWQ_OK;
}

glowq_status glowq_mx_group_forward(const glowq_unit* u, int32_t restore, void* workspace,
                                    size_t workspace_bytes, void* stream) {
  const bool corrected = u && u->r > 0 && restore;
  glowq_status s = validate_mx(u, true, corrected);
  if (s != GLOWQ_OK) return s;
  if (!workspace) return GLOWQ_ERR_WORKSPACE;
  if ((uintptr_t)workspace & 255u) return GLOWQ_ERR_ALIGN;
  if (workspace_bytes < plan_mx_workspace(*u).bytes) return GLOWQ_ERR_WORKSPACE;
  return hip_status(launch_mx_forward(*u, restore != 0, (char*)workspace, (hipStream_t)stream));
}

glowq_status glowq_debug_unpack(const void* w_prepared, int32_t d_out, int32_t d_in,
                                int32_t group_size, uint8_t* q_out, void* stream) {
  if (!w_prepared || !q_out) return GLOWQ_ERR_NULL;
  glowq_status s = check_weights_shape(d_out, d_in, group_size);
  if (s != GLOWQ_OK) return s;
  if (misaligned(w_prepared) || misaligned(q_out)) return GLOWQ_ERR_ALIGN;
  return hip_status(launch_debug_unpack(w_prepared, d_out, d_in, group_size, q_out, (hipStream_t)stream));
}

glowq_status glowq_debug_dequant(const void* w_prepared, int32_t d_out, int32_t d_in,
                                 int32_t group_size, int32_t act_dtype, void* w_out,
                                 void* stream) {
  if (!w_prepared || !w_out) return GLOWQ_ERR_NULL;
  glowq_status s = check_weights_shape(d_out, d_in, group_size);
  if (s != GLOWQ_OK) return s;
  if (act_dtype != GLOWQ_F16 && act_dtype != GLOWQ_BF16) return GLOWQ_ERR_DTYPE;
  if (misaligned(w_prepared) || misaligned(w_out)) return GLOWQ_ERR_ALIGN;
  return hip_status(launch_debug_dequant(w_prepared, d_out, d_in, group_size, act_dtype, w_out,
                                         (hipStream_t)stream));
}

}  // extern "C"
