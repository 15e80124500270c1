// C ABI of libtdq: argument validation on the host, workspace layout, and the
// launch sequence of each entry point.  Nothing here computes on the data.
#include <math.h>
#include <atomic>
#include <stdlib.h>
#include <string.h>

#include "tdq_internal.hpp"

namespace tdq {

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

LevelPlan make_level_plan(tdq_dtype dt, int G) {
  LevelPlan lp;
  memset(&lp, 0, sizeof(lp));
  lp.key_bits = dt == TDQ_F16 ? 15 : 31;
  int max_bits = 0;
  while ((G << (max_bits + 1)) <= kHistLdsWords && max_bits + 1 <= kMaxLevelBits) ++max_bits;
  if (max_bits < 1) max_bits = 1;
  int n = (lp.key_bits + max_bits - 1) / max_bits;
  static_assert(31 <= 5 * kMaxLevels && ((TDQ_MAX_GROUPS << 5) <= kHistLdsWords),
                "the level arrays must hold the plan of the largest set count");
  lp.n_levels = n;
  int left = lp.key_bits;
  for (int l = 0; l < n; ++l) {
    const int levels_left = n - l;
    int b = (left + levels_left - 1) / levels_left;     // spread the bits evenly
    lp.bits[l] = b;
    left -= b;
    lp.shift[l] = left;
  }
  return lp;
}

int bracket_bins(int G) {
  int w = 2048;
  while (w >= kBracketMinBins && (long long)G * w > kBracketLdsWords) w >>= 1;
  return w >= kBracketMinBins ? w : 0;
}

WorkspaceLayout make_layout(int B, int T, int G, const LevelPlan& lp) {
  WorkspaceLayout w;
  memset(&w, 0, sizeof(w));
  const size_t M = (size_t)B * T, BG = (size_t)B * G;
  size_t off = 0;
  w.status = off;   off = align256(off + 64 * sizeof(unsigned));
  w.img_flag = off; off = align256(off + (size_t)B * sizeof(unsigned));
  w.r = off;        off = align256(off + M * sizeof(float));
  w.mean = off;     off = align256(off + M * sizeof(double));
  w.m2 = off;       off = align256(off + M * sizeof(double));
  w.part = off;     off = align256(off + assign_partial_bytes(B, G));
  w.grp = off;      off = align256(off + BG * sizeof(GroupWork));
  w.hist = off;
  for (int l = 0; l < lp.n_levels; ++l) {
    w.hist_level[l] = off;
    off += BG * ((size_t)1 << lp.bits[l]) * sizeof(unsigned);   // levels are contiguous
  }
  off = align256(off);
  w.br = off;       off = align256(off + BG * sizeof(Bracket));
  w.bhist = off;    off = align256(off + BG * (size_t)bracket_bins(G) * sizeof(unsigned));
  w.total = align256(off);
  return w;
}

// blocks = false: the token-set entry points (chan_group must be 0); true: the
// per-(token, 32-channel block) entry points (chan_group must be 32).
static int check_params(const tdq_params* p, bool blocks = false) {
  if (!p) return TDQ_ERR_NULL;
  if (p->n_groups < 1 || p->n_groups > TDQ_MAX_GROUPS) return TDQ_ERR_PARAM;
  if (p->act_bits != 4) return p->act_bits == 8 ? TDQ_ERR_UNSUPPORTED : TDQ_ERR_PARAM;
  if (p->flags & ~(TDQ_FLAG_C1 | TDQ_FLAG_C2 | TDQ_FLAG_EXACT_SELECT)) return TDQ_ERR_PARAM;
  if (!(p->tau > 0.0) || !isfinite(p->tau)) return TDQ_ERR_PARAM;
  if (!(p->zr > 0.0 && p->zr < 1.0)) return TDQ_ERR_PARAM;
  if (!(p->eps_scale > 0.f) || !(p->eps_std >= 0.f)) return TDQ_ERR_PARAM;
  if (p->chan_group < 0) return TDQ_ERR_PARAM;
  if (p->chan_group != (blocks ? TDQ_BLOCK : 0)) return TDQ_ERR_UNSUPPORTED;
  if (!(p->base_pct >= 0.0 && p->base_pct <= 1.0)) return TDQ_ERR_PARAM;
  return TDQ_OK;
}

static int check_shape(int32_t B, int32_t T, int32_t C, int64_t ld_x) {
  if (B < 1 || T < 1 || C < 1 || B > TDQ_MAX_IMAGES) return TDQ_ERR_SHAPE;
  if (ld_x < C) return TDQ_ERR_SHAPE;
  if ((int64_t)B * T > (int64_t)1 << 30) return TDQ_ERR_SHAPE;
  return TDQ_OK;
}

// Rank ceil(frac g) among the g values of a block, padding zeros included (binary64, as
// everywhere).
static int block_rank(double frac) {
  long long k = (long long)ceil(frac * (double)TDQ_BLOCK);
  return (int)(k < 1 ? 1 : (k > TDQ_BLOCK ? TDQ_BLOCK : k));
}

static Scalars make_scalars(const tdq_params* p) {
  Scalars s;
  s.qmax = (float)kQMax;
  s.qmax_tau = (float)kQMax * (float)p->tau;   // binary32 product, as in the definition
  s.two_qmax = 2.0f * (float)kQMax;
  s.eps_scale = p->eps_scale;
  s.eps_std = (double)p->eps_std;
  s.zr = p->zr;
  s.base_pct = (p->base_pct > 0.0 && p->base_pct < 1.0) ? p->base_pct : 0.0;
  s.flags = p->flags;
  return s;
}

// Everything of tdq_calibrate_groups after the per-token statistics (which are in the
// workspace): assignment, rank select(s), projection.  X is token-major.
static int calibrate_after_stats(const void* X, tdq_dtype dt, int32_t B, int32_t T, int32_t C,
                                 int64_t ld_x, const tdq_params* p, int32_t* group_id, float* clip,
                                 float* scale, tdq_group_stats* stats, void* workspace,
                                 const LevelPlan& lp, const WorkspaceLayout& wl, hipStream_t st) {
  const int G = p->n_groups;
  char* ws = static_cast<char*>(workspace);
  unsigned* status = reinterpret_cast<unsigned*>(ws + wl.status);
  unsigned* img_flag = reinterpret_cast<unsigned*>(ws + wl.img_flag);
  float* r = reinterpret_cast<float*>(ws + wl.r);
  double* mean = reinterpret_cast<double*>(ws + wl.mean);
  double* m2 = reinterpret_cast<double*>(ws + wl.m2);
  GroupWork* grp = reinterpret_cast<GroupWork*>(ws + wl.grp);
  unsigned* hist = reinterpret_cast<unsigned*>(ws + wl.hist);
  const Scalars sc = make_scalars(p);

  void* part = ws + wl.part;
  if (launch_assign(r, mean, m2, B, T, C, G, group_id, part, img_flag, status, st) != hipSuccess)
    return TDQ_ERR_HIP;

  // One rank select per rank wanted of every set: first the base radius Q_p(|x|) when a
  // percentile is asked for (Eq. DSTG_clip), then Q_zr(|x|) with the projection.
  // binary16 input: one sweep resolves the rank of (nearly) every set exactly, and the
  // kernel that verifies it resolves the others.  binary32 input, or too many sets for
  // the interval histogram: radix levels.
  const int W = bracket_bins(G);
  const bool single_sweep = dt == TDQ_F16 && W > 0 && (long long)T * C < (1ll << 32);
  const bool exact_only = (p->flags & TDQ_FLAG_EXACT_SELECT) != 0;
  Bracket* br = reinterpret_cast<Bracket*>(ws + wl.br);
  unsigned* bhist = reinterpret_cast<unsigned*>(ws + wl.bhist);
  const bool two_passes = sc.base_pct > 0.0;
  for (int pass = two_passes ? kPassBase : kPassZr; pass >= kPassZr; --pass) {
    const bool keep_base = two_passes && pass == kPassZr;
    if (single_sweep) {
      if (!exact_only) {
        if (launch_bracket(X, B, T, C, ld_x, G, W, group_id, part, sc, pass, keep_base, grp, br,
                           bhist, st) != hipSuccess)
          return TDQ_ERR_HIP;
        if (launch_bracket_hist(X, B, T, C, ld_x, G, W, group_id, br, bhist, st) != hipSuccess)
          return TDQ_ERR_HIP;
      } else if (launch_finalize_groups(part, B, T, C, G, sc, pass, keep_base, grp, hist, lp, st) !=
                 hipSuccess) {
        return TDQ_ERR_HIP;
      }
      if (launch_bracket_finish(X, B, T, C, ld_x, G, W, group_id, bhist, exact_only, sc, pass, grp,
                                br, clip, scale, stats, img_flag, status, st) != hipSuccess)
        return TDQ_ERR_HIP;
      continue;
    }
    if (launch_finalize_groups(part, B, T, C, G, sc, pass, keep_base, grp, hist, lp, st) !=
        hipSuccess)
      return TDQ_ERR_HIP;
    for (int l = 0; l < lp.n_levels; ++l) {
      unsigned* hl = reinterpret_cast<unsigned*>(ws + wl.hist_level[l]);
      if (launch_hist(X, dt, B, T, C, ld_x, G, group_id, grp, hl, lp.shift[l], lp.bits[l], st) !=
          hipSuccess)
        return TDQ_ERR_HIP;
      if (launch_select(hl, B, G, lp.shift[l], lp.bits[l], l == lp.n_levels - 1, dt, sc, grp, clip,
                        scale, stats, img_flag, status, pass, st) != hipSuccess)
        return TDQ_ERR_HIP;
    }
  }
  return TDQ_OK;
}

// ---------------------------------------------------------------------------
// Library-owned calibration scratch for tdq_calibrate_groups_static.  In host code the
// array's name is only a handle for hipGetSymbolAddress; the device address is looked up
// once per device (each GPU has its own copy at its own address) and that pointer is what
// the kernels get.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[TDQ_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device, or nullptr (with *rc set).
static void* scratch_of_current_device(int* rc) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    *rc = TDQ_ERR_HIP;
    return nullptr;
  }
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    // two threads racing here look up the same address; either store is the right one
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      *rc = TDQ_ERR_HIP;
      return nullptr;
    }
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);
  }
  *rc = TDQ_OK;
  return ptr;
}

// The status area of the scratch, handed to the caller's buffer (a kernel, not a copy
// call: a caller may be capturing a graph).
__global__ void k_export_status(const unsigned* __restrict__ status, unsigned* __restrict__ out) {
  const int i = threadIdx.x;
  if (i < 4) out[i] = i < 3 ? status[i] : 0u;
}

}  // namespace tdq

using namespace tdq;

extern "C" {

int tdq_version(void) { return TDQ_VERSION; }

const char* tdq_status_string(int status) {
  switch (status) {
    case TDQ_OK: return "ok";
    case TDQ_ERR_NULL: return "null pointer";
    case TDQ_ERR_SHAPE: return "invalid shape or leading dimension";
    case TDQ_ERR_PARAM: return "parameter out of range";
    case TDQ_ERR_WORKSPACE: return "workspace too small or misaligned";
    case TDQ_ERR_DTYPE: return "unknown dtype";
    case TDQ_ERR_HIP: return "HIP call failed";
    case TDQ_ERR_UNSUPPORTED: return "not implemented in this build";
    case TDQ_ERR_ALIGN: return "pointer or leading dimension misaligned";
    default: return "unknown status";
  }
}

void tdq_default_params(tdq_params* p) {
  if (!p) return;
  p->n_groups = 8;
  p->chan_group = 0;
  p->act_bits = 4;
  p->flags = TDQ_FLAG_C1 | TDQ_FLAG_C2;
  p->tau = 1.0;
  p->zr = 0.2;
  p->base_pct = 0.0;
  p->eps_scale = 1e-8f;
  p->eps_std = 1e-12f;
}

size_t tdq_workspace_bytes(int32_t B, int32_t T, int32_t C, tdq_dtype dt, const tdq_params* p) {
  if (check_params(p) != TDQ_OK) return 0;
  if (check_shape(B, T, C, C) != TDQ_OK) return 0;
  if (dt != TDQ_F16 && dt != TDQ_F32) return 0;
  const LevelPlan lp = make_level_plan(dt, p->n_groups);
  return make_layout(B, T, p->n_groups, lp).total;
}

int tdq_calibrate_groups(const void* X, tdq_dtype dt, int32_t B, int32_t T, int32_t C,
                         int64_t ld_x, const tdq_params* p, int32_t* group_id, float* clip,
                         float* scale, tdq_group_stats* stats, void* workspace,
                         size_t workspace_bytes, void* stream) {
  if (!X || !p || !group_id || !clip || !scale || !workspace) return TDQ_ERR_NULL;
  if (dt != TDQ_F16 && dt != TDQ_F32) return TDQ_ERR_DTYPE;
  int rc = check_params(p);
  if (rc != TDQ_OK) return rc;
  rc = check_shape(B, T, C, ld_x);
  if (rc != TDQ_OK) return rc;
  const int G = p->n_groups;
  const LevelPlan lp = make_level_plan(dt, G);
  const WorkspaceLayout wl = make_layout(B, T, G, lp);
  if (workspace_bytes < wl.total) return TDQ_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255) return TDQ_ERR_WORKSPACE;
  const size_t esz = dt == TDQ_F16 ? 2 : 4;
  if (reinterpret_cast<uintptr_t>(X) % esz) return TDQ_ERR_ALIGN;

  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  if (launch_token_stats(X, dt, B * T, C, ld_x, reinterpret_cast<float*>(ws + wl.r),
                         reinterpret_cast<double*>(ws + wl.mean),
                         reinterpret_cast<double*>(ws + wl.m2), st) != hipSuccess)
    return TDQ_ERR_HIP;
  return calibrate_after_stats(X, dt, B, T, C, ld_x, p, group_id, clip, scale, stats, workspace, lp,
                               wl, st);
}

int tdq_calibrate_groups_static(const void* X, tdq_dtype dt, int32_t B, int32_t T, int32_t C,
                                int64_t ld_x, const tdq_params* p, int32_t* group_id, float* clip,
                                float* scale, tdq_group_stats* stats, uint32_t* status,
                                void* stream) {
  if (!X || !p || !group_id || !clip || !scale) return TDQ_ERR_NULL;
  if (dt != TDQ_F16 && dt != TDQ_F32) return TDQ_ERR_DTYPE;
  int rc = check_params(p);
  if (rc != TDQ_OK) return rc;
  rc = check_shape(B, T, C, ld_x);
  if (rc != TDQ_OK) return rc;
  if (reinterpret_cast<uintptr_t>(status) & 3) return TDQ_ERR_ALIGN;
  const LevelPlan lp = make_level_plan(dt, p->n_groups);
  const WorkspaceLayout wl = make_layout(B, T, p->n_groups, lp);
  if (wl.total > (size_t)TDQ_STATIC_SCRATCH_BYTES) return TDQ_ERR_WORKSPACE;
  void* ws = scratch_of_current_device(&rc);
  if (!ws) return rc;
  // the kernels of tdq_calibrate_groups clear every part of the workspace they add into
  // (set records, histograms, counters), so what the last call left behind does not matter
  rc = tdq_calibrate_groups(X, dt, B, T, C, ld_x, p, group_id, clip, scale, stats, ws,
                            TDQ_STATIC_SCRATCH_BYTES, stream);
  if (rc != TDQ_OK) return rc;
  if (status) {
    hipLaunchKernelGGL(k_export_status, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream),
                       reinterpret_cast<const unsigned*>(static_cast<char*>(ws) + wl.status), status);
    if (hipGetLastError() != hipSuccess) return TDQ_ERR_HIP;
  }
  return TDQ_OK;
}

int tdq_calibrate_groups_chw(const void* X, tdq_dtype dt, int32_t B, int32_t C, int32_t T,
                             int64_t ld_c, int64_t ld_b, const tdq_params* p, void* Xt,
                             int64_t ld_xt, int32_t* group_id, float* clip, float* scale,
                             tdq_group_stats* stats, void* workspace, size_t workspace_bytes,
                             void* stream) {
  if (!X || !Xt || !p || !group_id || !clip || !scale || !workspace) return TDQ_ERR_NULL;
  if (dt != TDQ_F16 && dt != TDQ_F32) return TDQ_ERR_DTYPE;
  int rc = check_params(p);
  if (rc != TDQ_OK) return rc;
  rc = check_shape(B, T, C, ld_xt);
  if (rc != TDQ_OK) return rc;
  if (B > TDQ_MAX_IMAGES) return TDQ_ERR_SHAPE;
  if (ld_c < T || ld_b < (int64_t)(C - 1) * ld_c + T) return TDQ_ERR_SHAPE;
  const int G = p->n_groups;
  const LevelPlan lp = make_level_plan(dt, G);
  const WorkspaceLayout wl = make_layout(B, T, G, lp);
  if (workspace_bytes < wl.total) return TDQ_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255) return TDQ_ERR_WORKSPACE;
  const size_t esz = dt == TDQ_F16 ? 2 : 4;
  if (reinterpret_cast<uintptr_t>(X) % esz || reinterpret_cast<uintptr_t>(Xt) % esz)
    return TDQ_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  if (launch_tokenize_stats_chw(X, dt, B, C, T, ld_c, ld_b, Xt, ld_xt,
                                reinterpret_cast<float*>(ws + wl.r),
                                reinterpret_cast<double*>(ws + wl.mean),
                                reinterpret_cast<double*>(ws + wl.m2), st) != hipSuccess)
    return TDQ_ERR_HIP;
  return calibrate_after_stats(Xt, dt, B, T, C, ld_xt, p, group_id, clip, scale, stats, workspace,
                               lp, wl, st);
}

int tdq_quantize_act(const void* X, tdq_dtype dt, int32_t B, int32_t T, int32_t C, int64_t ld_x,
                     const tdq_params* p, const int32_t* group_id, const float* clip,
                     const float* scale, uint8_t* Qx, int64_t ld_q, void* stream) {
  if (!X || !p || !clip || !scale || !Qx) return TDQ_ERR_NULL;
  if (dt != TDQ_F16 && dt != TDQ_F32) return TDQ_ERR_DTYPE;
  int rc = check_params(p);
  if (rc != TDQ_OK) return rc;
  rc = check_shape(B, T, C, ld_x);
  if (rc != TDQ_OK) return rc;
  if (!group_id && p->n_groups != 1) return TDQ_ERR_NULL;
  if (ld_q < (C + 1) / 2) return TDQ_ERR_SHAPE;
  const size_t esz = dt == TDQ_F16 ? 2 : 4;
  if (reinterpret_cast<uintptr_t>(X) % esz) return TDQ_ERR_ALIGN;
  if (launch_quantize(X, dt, B, T, C, ld_x, p->n_groups, group_id, clip, scale, Qx, ld_q,
                      static_cast<hipStream_t>(stream)) != hipSuccess)
    return TDQ_ERR_HIP;
  return TDQ_OK;
}

int tdq_calibrate_quantize_fused(const void* X, tdq_dtype dt, int32_t B, int32_t T, int32_t C,
                                 int64_t ld_x, const tdq_params* p, int32_t* group_id, float* clip,
                                 float* scale, tdq_group_stats* stats, uint32_t* image_flags,
                                 uint8_t* Qx, int64_t ld_q, void* workspace, size_t workspace_bytes,
                                 void* stream) {
  if (!X || !p || !group_id || !clip || !scale || !Qx || !workspace) return TDQ_ERR_NULL;
  if (dt != TDQ_F16 && dt != TDQ_F32) return TDQ_ERR_DTYPE;
  int rc = check_params(p);
  if (rc != TDQ_OK) return rc;
  rc = check_shape(B, T, C, ld_x);
  if (rc != TDQ_OK) return rc;
  const int G = p->n_groups;
  if (G > TDQ_FUSED_MAX_GROUPS) return TDQ_ERR_UNSUPPORTED;
  if (ld_q < (C + 1) / 2) return TDQ_ERR_SHAPE;
  const WorkspaceLayout wl = make_layout(B, T, G, make_level_plan(dt, G));
  if (workspace_bytes < wl.total) return TDQ_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255) return TDQ_ERR_WORKSPACE;
  const size_t esz = dt == TDQ_F16 ? 2 : 4;
  if (reinterpret_cast<uintptr_t>(X) % esz) return TDQ_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(image_flags) & 3) return TDQ_ERR_ALIGN;
  char* ws = static_cast<char*>(workspace);
  if (launch_fused_small(X, dt, B, T, C, ld_x, G, make_scalars(p),
                         reinterpret_cast<float*>(ws + wl.r), reinterpret_cast<double*>(ws + wl.mean),
                         reinterpret_cast<double*>(ws + wl.m2), group_id, clip, scale, stats,
                         image_flags, Qx, ld_q, static_cast<hipStream_t>(stream)) != hipSuccess)
    return TDQ_ERR_HIP;
  return TDQ_OK;
}

int tdq_range_disparity(const void* X, tdq_dtype dt, int32_t B, int32_t T, int32_t C, int64_t ld_x,
                        float* token_median, float* token_max, float* disparity, float* max_abs,
                        void* stream) {
  if (!X || !token_median || !token_max || !disparity || !max_abs) return TDQ_ERR_NULL;
  if (dt != TDQ_F16 && dt != TDQ_F32) return TDQ_ERR_DTYPE;
  const int rc = check_shape(B, T, C, ld_x);
  if (rc != TDQ_OK) return rc;
  const size_t esz = dt == TDQ_F16 ? 2 : 4;
  if (reinterpret_cast<uintptr_t>(X) % esz) return TDQ_ERR_ALIGN;
  if ((reinterpret_cast<uintptr_t>(token_median) | reinterpret_cast<uintptr_t>(token_max) |
       reinterpret_cast<uintptr_t>(disparity) | reinterpret_cast<uintptr_t>(max_abs)) & 3)
    return TDQ_ERR_ALIGN;
  if (launch_range_disparity(X, dt, B, T, C, ld_x, token_median, token_max, disparity, max_abs,
                             static_cast<hipStream_t>(stream)) != hipSuccess)
    return TDQ_ERR_HIP;
  return TDQ_OK;
}

int tdq_tokenize_chw(const void* X, tdq_dtype dt, int32_t B, int32_t C, int32_t T, int64_t ld_c,
                     int64_t ld_b, void* Xt, int64_t ld_xt, void* stream) {
  if (!X || !Xt) return TDQ_ERR_NULL;
  if (dt != TDQ_F16 && dt != TDQ_F32) return TDQ_ERR_DTYPE;
  if (B < 1 || T < 1 || C < 1 || B > TDQ_MAX_IMAGES) return TDQ_ERR_SHAPE;
  if ((int64_t)B * T > (int64_t)1 << 30) return TDQ_ERR_SHAPE;
  if (ld_c < T || ld_b < (int64_t)(C - 1) * ld_c + T || ld_xt < C) return TDQ_ERR_SHAPE;
  const size_t esz = dt == TDQ_F16 ? 2 : 4;
  if (reinterpret_cast<uintptr_t>(X) % esz || reinterpret_cast<uintptr_t>(Xt) % esz)
    return TDQ_ERR_ALIGN;
  if (launch_tokenize_chw(X, dt, B, C, T, ld_c, ld_b, Xt, ld_xt,
                          static_cast<hipStream_t>(stream)) != hipSuccess)
    return TDQ_ERR_HIP;
  return TDQ_OK;
}

int tdq_quantize_act_blocks(const void* X, tdq_dtype dt, int32_t B, int32_t T, int32_t C,
                            int64_t ld_x, const tdq_params* p, uint8_t* Qx, int64_t ld_q,
                            float* block_scale, float* block_clip, int64_t ld_s, void* stream) {
  if (!X || !p || !Qx || !block_scale) return TDQ_ERR_NULL;
  if (dt != TDQ_F16 && dt != TDQ_F32) return TDQ_ERR_DTYPE;
  int rc = check_params(p, true);
  if (rc != TDQ_OK) return rc;
  rc = check_shape(B, T, C, ld_x);
  if (rc != TDQ_OK) return rc;
  const int64_t KB = ((int64_t)C + TDQ_BLOCK - 1) / TDQ_BLOCK;
  if (ld_q < (C + 1) / 2 || ld_s < KB) return TDQ_ERR_SHAPE;
  if ((int64_t)B * T * KB >= (int64_t)1 << 31) return TDQ_ERR_SHAPE;
  const size_t esz = dt == TDQ_F16 ? 2 : 4;
  if (reinterpret_cast<uintptr_t>(X) % esz) return TDQ_ERR_ALIGN;
  if ((reinterpret_cast<uintptr_t>(block_scale) | reinterpret_cast<uintptr_t>(block_clip)) & 3)
    return TDQ_ERR_ALIGN;
  const int kq = block_rank(p->zr);
  const int kp = (p->base_pct > 0.0 && p->base_pct < 1.0) ? block_rank(p->base_pct) : TDQ_BLOCK;
  if (launch_quantize_blocks(X, dt, (long long)B * T, C, ld_x, kq, kp, make_scalars(p), Qx, ld_q,
                             block_scale, block_clip, ld_s,
                             static_cast<hipStream_t>(stream)) != hipSuccess)
    return TDQ_ERR_HIP;
  return TDQ_OK;
}

int tdq_quantize_act_blocks_f6(const void* X, tdq_dtype dt, int32_t B, int32_t T, int32_t C,
                               int64_t ld_x, const tdq_params* p, uint8_t* Qx6, float* block_scale,
                               float* block_clip, int64_t ld_s, void* stream) {
  if (!X || !p || !Qx6 || !block_scale) return TDQ_ERR_NULL;
  if (dt != TDQ_F16 && dt != TDQ_F32) return TDQ_ERR_DTYPE;
  int rc = check_params(p, true);
  if (rc != TDQ_OK) return rc;
  rc = check_shape(B, T, C, ld_x);
  if (rc != TDQ_OK) return rc;
  const int64_t KB = ((int64_t)C + TDQ_BLOCK - 1) / TDQ_BLOCK;
  if (ld_s < KB) return TDQ_ERR_SHAPE;
  if ((int64_t)B * T * KB >= (int64_t)1 << 31) return TDQ_ERR_SHAPE;
  const size_t esz = dt == TDQ_F16 ? 2 : 4;
  if (reinterpret_cast<uintptr_t>(X) % esz) return TDQ_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(Qx6) & 15) return TDQ_ERR_ALIGN;
  if ((reinterpret_cast<uintptr_t>(block_scale) | reinterpret_cast<uintptr_t>(block_clip)) & 3)
    return TDQ_ERR_ALIGN;
  const int kq = block_rank(p->zr);
  const int kp = (p->base_pct > 0.0 && p->base_pct < 1.0) ? block_rank(p->base_pct) : TDQ_BLOCK;
  if (launch_quantize_blocks_f6(X, dt, (long long)B * T, C, ld_x, kq, kp, make_scalars(p), Qx6,
                                block_scale, block_clip, ld_s,
                                static_cast<hipStream_t>(stream)) != hipSuccess)
    return TDQ_ERR_HIP;
  return TDQ_OK;
}

int tdq_quantize_act_blocks_chw(const void* X, tdq_dtype dt, int32_t B, int32_t C, int32_t T,
                                int64_t ld_c, int64_t ld_b, const tdq_params* p, uint8_t* Qx,
                                int64_t ld_q, float* block_scale, float* block_clip, int64_t ld_s,
                                void* stream) {
  if (!X || !p || !Qx || !block_scale) return TDQ_ERR_NULL;
  if (dt != TDQ_F16 && dt != TDQ_F32) return TDQ_ERR_DTYPE;
  int rc = check_params(p, true);
  if (rc != TDQ_OK) return rc;
  if (B < 1 || T < 1 || C < 1 || B > TDQ_MAX_IMAGES) return TDQ_ERR_SHAPE;
  if ((int64_t)B * T > (int64_t)1 << 30) return TDQ_ERR_SHAPE;
  if (ld_c < T || ld_b < (int64_t)(C - 1) * ld_c + T) return TDQ_ERR_SHAPE;
  const int64_t KB = ((int64_t)C + TDQ_BLOCK - 1) / TDQ_BLOCK;
  if (ld_q < (C + 1) / 2 || ld_s < KB) return TDQ_ERR_SHAPE;
  const size_t esz = dt == TDQ_F16 ? 2 : 4;
  if (reinterpret_cast<uintptr_t>(X) % esz) return TDQ_ERR_ALIGN;
  if ((reinterpret_cast<uintptr_t>(block_scale) | reinterpret_cast<uintptr_t>(block_clip)) & 3)
    return TDQ_ERR_ALIGN;
  const int kq = block_rank(p->zr);
  const int kp = (p->base_pct > 0.0 && p->base_pct < 1.0) ? block_rank(p->base_pct) : TDQ_BLOCK;
  if (launch_quantize_blocks_chw(X, dt, B, C, T, ld_c, ld_b, kq, kp, make_scalars(p), Qx, ld_q,
                                 block_scale, block_clip, ld_s,
                                 static_cast<hipStream_t>(stream)) != hipSuccess)
    return TDQ_ERR_HIP;
  return TDQ_OK;
}

int tdq_group_diagnostics(const void* X, tdq_dtype dt, int32_t B, int32_t T, int32_t C, int64_t ld_x,
                          const tdq_params* p, const int32_t* group_id, const float* clip,
                          const float* scale, uint64_t* zero_count, uint64_t* clipped_count,
                          void* stream) {
  if (!X || !p || !clip || !scale || !zero_count || !clipped_count) return TDQ_ERR_NULL;
  if (dt != TDQ_F16 && dt != TDQ_F32) return TDQ_ERR_DTYPE;
  int rc = check_params(p);
  if (rc != TDQ_OK) return rc;
  rc = check_shape(B, T, C, ld_x);
  if (rc != TDQ_OK) return rc;
  if (!group_id && p->n_groups != 1) return TDQ_ERR_NULL;
  const size_t esz = dt == TDQ_F16 ? 2 : 4;
  if (reinterpret_cast<uintptr_t>(X) % esz) return TDQ_ERR_ALIGN;
  if ((reinterpret_cast<uintptr_t>(zero_count) | reinterpret_cast<uintptr_t>(clipped_count)) & 7)
    return TDQ_ERR_ALIGN;
  if (launch_group_diag(X, dt, B, T, C, ld_x, p->n_groups, group_id, clip, scale,
                        reinterpret_cast<unsigned long long*>(zero_count),
                        reinterpret_cast<unsigned long long*>(clipped_count),
                        static_cast<hipStream_t>(stream)) != hipSuccess)
    return TDQ_ERR_HIP;
  return TDQ_OK;
}

int tdq_w4a4_linear(const uint8_t* Qx, int64_t ld_q, const int32_t* group_id, const float* scale,
                    int32_t B, int32_t T, int32_t K, int32_t N, int32_t G, const uint8_t* Qw,
                    int64_t ld_w, const float* w_scale, const float* bias, void* Y,
                    tdq_dtype y_dt, int64_t ld_y, int32_t* acc_dump, void* stream) {
  if (!Qx || !scale || !Qw || !w_scale || !Y) return TDQ_ERR_NULL;
  if (y_dt != TDQ_F16 && y_dt != TDQ_F32) return TDQ_ERR_DTYPE;
  if (B < 1 || T < 1 || K < 1 || N < 1) return TDQ_ERR_SHAPE;
  if ((int64_t)B * T > (int64_t)1 << 30) return TDQ_ERR_SHAPE;
  if (K > TDQ_MAX_K) return TDQ_ERR_SHAPE;  // 256 * 64 * K must stay below 2^31
  if (G < 1 || G > TDQ_MAX_GROUPS) return TDQ_ERR_PARAM;
  if (!group_id && G != 1) return TDQ_ERR_NULL;
  const int64_t row_bytes = 16 * (((int64_t)K + 31) / 32);
  if (ld_q < row_bytes || ld_w < row_bytes || ld_y < N) return TDQ_ERR_SHAPE;
  if (ld_q % 16 || ld_w % 16) return TDQ_ERR_ALIGN;
  if ((reinterpret_cast<uintptr_t>(Qx) & 15) || (reinterpret_cast<uintptr_t>(Qw) & 15))
    return TDQ_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(Y) % (y_dt == TDQ_F16 ? 2 : 4)) return TDQ_ERR_ALIGN;
  if (launch_w4a4_gemm(Qx, ld_q, group_id, scale, B * T, T, K, N, G, Qw, ld_w, w_scale, bias, Y,
                       y_dt, ld_y, acc_dump, static_cast<hipStream_t>(stream)) != hipSuccess)
    return TDQ_ERR_HIP;
  return TDQ_OK;
}

int tdq_w4a4_linear_blocks(const uint8_t* Qx, int64_t ld_q, const float* block_scale, int64_t ld_s,
                           int64_t M, int32_t K, int32_t N, const uint8_t* Qw, int64_t ld_w,
                           const float* w_scale, const float* bias, void* Y, tdq_dtype y_dt,
                           int64_t ld_y, void* stream) {
  if (!Qx || !block_scale || !Qw || !w_scale || !Y) return TDQ_ERR_NULL;
  if (y_dt != TDQ_F16 && y_dt != TDQ_F32) return TDQ_ERR_DTYPE;
  if (M < 1 || K < 1 || N < 1) return TDQ_ERR_SHAPE;
  if (M > (int64_t)1 << 30 || K > 131072) return TDQ_ERR_SHAPE;
  const int64_t KB = ((int64_t)K + TDQ_BLOCK - 1) / TDQ_BLOCK;
  const int64_t row_bytes = 16 * KB;
  if (ld_q < row_bytes || ld_w < row_bytes || ld_y < N || ld_s < KB) return TDQ_ERR_SHAPE;
  if (ld_q % 16 || ld_w % 16) return TDQ_ERR_ALIGN;
  if ((reinterpret_cast<uintptr_t>(Qx) & 15) || (reinterpret_cast<uintptr_t>(Qw) & 15))
    return TDQ_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(block_scale) & 3) return TDQ_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(Y) % (y_dt == TDQ_F16 ? 2 : 4)) return TDQ_ERR_ALIGN;
  if (launch_w4a4_gemm_blocks(Qx, ld_q, block_scale, ld_s, (int)M, K, N, Qw, ld_w, w_scale, bias, Y,
                              y_dt, ld_y, static_cast<hipStream_t>(stream)) != hipSuccess)
    return TDQ_ERR_HIP;
  return TDQ_OK;
}

int tdq_quantize_act_f6(const void* X, tdq_dtype dt, int32_t B, int32_t T, int32_t C, int64_t ld_x,
                        const tdq_params* p, const int32_t* group_id, const float* clip,
                        const float* scale, uint8_t* Qx6, void* stream) {
  if (!X || !p || !clip || !scale || !Qx6) return TDQ_ERR_NULL;
  if (dt != TDQ_F16 && dt != TDQ_F32) return TDQ_ERR_DTYPE;
  int rc = check_params(p);
  if (rc != TDQ_OK) return rc;
  rc = check_shape(B, T, C, ld_x);
  if (rc != TDQ_OK) return rc;
  if (C > 131072) return TDQ_ERR_SHAPE;
  if (!group_id && p->n_groups != 1) return TDQ_ERR_NULL;
  const size_t esz = dt == TDQ_F16 ? 2 : 4;
  if (reinterpret_cast<uintptr_t>(X) % esz) return TDQ_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(Qx6) & 15) return TDQ_ERR_ALIGN;
  if (launch_quantize_f6(X, dt, B, T, C, ld_x, p->n_groups, group_id, clip, scale, Qx6,
                         static_cast<hipStream_t>(stream)) != hipSuccess)
    return TDQ_ERR_HIP;
  return TDQ_OK;
}

size_t tdq_f6_bytes(int64_t rows, int32_t K) {
  if (rows < 1 || K < 1) return 0;
  const int64_t KB = 2 * (((int64_t)K + 127) / 128);
  return (size_t)(((rows + 31) / 32) * KB * 1536);
}

int tdq_pack_codes_f6(const uint8_t* Q, int64_t ld, int64_t rows, int32_t K, uint8_t* F, void* stream) {
  if (!Q || !F) return TDQ_ERR_NULL;
  if (rows < 1 || rows > (int64_t)1 << 30 || K < 1 || K > 131072 || ld < (K + 1) / 2) return TDQ_ERR_SHAPE;
  if (reinterpret_cast<uintptr_t>(F) & 15) return TDQ_ERR_ALIGN;
  if (launch_pack_f6(Q, ld, (int)rows, K, F, static_cast<hipStream_t>(stream)) != hipSuccess)
    return TDQ_ERR_HIP;
  return TDQ_OK;
}

int tdq_w4a4_linear_f6(const uint8_t* Qx6, const int32_t* group_id, const float* scale, int32_t B,
                       int32_t T, int32_t K, int32_t N, int32_t G, const uint8_t* Qw6,
                       const float* w_scale, const float* bias, void* Y, tdq_dtype y_dt, int64_t ld_y,
                       int32_t* acc_dump, void* stream) {
  if (!Qx6 || !scale || !Qw6 || !w_scale || !Y) return TDQ_ERR_NULL;
  if (y_dt != TDQ_F16 && y_dt != TDQ_F32) return TDQ_ERR_DTYPE;
  if (B < 1 || T < 1 || K < 1 || N < 1) return TDQ_ERR_SHAPE;
  if ((int64_t)B * T > (int64_t)1 << 30 || K > 131072 || ld_y < N) return TDQ_ERR_SHAPE;
  if (G < 1 || G > TDQ_MAX_GROUPS) return TDQ_ERR_PARAM;
  if (!group_id && G != 1) return TDQ_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(Qx6) & 15) || (reinterpret_cast<uintptr_t>(Qw6) & 15))
    return TDQ_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(Y) % (y_dt == TDQ_F16 ? 2 : 4)) return TDQ_ERR_ALIGN;
  if (launch_w4a4_gemm_f6(Qx6, Qw6, K, group_id, scale, B * T, T, N, G, w_scale, bias, Y, y_dt, ld_y,
                          acc_dump, static_cast<hipStream_t>(stream)) != hipSuccess)
    return TDQ_ERR_HIP;
  return TDQ_OK;
}

int tdq_w4a4_linear_blocks_f6(const uint8_t* Qx6, const float* block_scale, int64_t ld_s, int64_t M,
                              int32_t K, int32_t N, const uint8_t* Qw6, const float* w_scale,
                              const float* bias, void* Y, tdq_dtype y_dt, int64_t ld_y, void* stream) {
  if (!Qx6 || !block_scale || !Qw6 || !w_scale || !Y) return TDQ_ERR_NULL;
  if (y_dt != TDQ_F16 && y_dt != TDQ_F32) return TDQ_ERR_DTYPE;
  if (M < 1 || K < 1 || N < 1 || M > (int64_t)1 << 30 || K > 131072) return TDQ_ERR_SHAPE;
  const int64_t KB = ((int64_t)K + TDQ_BLOCK - 1) / TDQ_BLOCK;
  if (ld_y < N || ld_s < KB) return TDQ_ERR_SHAPE;
  if (ld_s > ((int64_t)1 << 22)) return TDQ_ERR_SHAPE;     // 128 rows of scales within 32-bit offsets
  if ((reinterpret_cast<uintptr_t>(Qx6) & 15) || (reinterpret_cast<uintptr_t>(Qw6) & 15))
    return TDQ_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(block_scale) & 3) return TDQ_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(Y) % (y_dt == TDQ_F16 ? 2 : 4)) return TDQ_ERR_ALIGN;
  if (launch_w4a4_gemm_blocks_f6(Qx6, Qw6, block_scale, ld_s, (int)M, K, N, w_scale, bias, Y, y_dt,
                                 ld_y, static_cast<hipStream_t>(stream)) != hipSuccess)
    return TDQ_ERR_HIP;
  return TDQ_OK;
}

int tdq_quantize_weight(const float* W, int32_t N, int32_t K, int64_t ld_w_in, uint8_t* Qw,
                        int64_t ld_w, float* w_scale, void* stream) {
  if (!W || !Qw || !w_scale) return TDQ_ERR_NULL;
  if (N < 1 || K < 1 || ld_w_in < K || ld_w < (K + 1) / 2) return TDQ_ERR_SHAPE;
  if (reinterpret_cast<uintptr_t>(W) & 3) return TDQ_ERR_ALIGN;
  if (launch_quantize_weight(W, N, K, ld_w_in, Qw, ld_w, w_scale,
                             static_cast<hipStream_t>(stream)) != hipSuccess)
    return TDQ_ERR_HIP;
  return TDQ_OK;
}

}  // extern "C"
