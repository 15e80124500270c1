// Host-side harness of libtdq for AddressSanitizer / UndefinedBehaviorSanitizer runs on a
// machine without a GPU (test infrastructure, not part of the product).
//
// The library's sources are compiled for the host only and linked with this file instead
// of the HIP runtime: the few runtime calls the host code makes are defined here and do
// nothing but record what was asked.  Every entry point then runs its complete host logic
// (argument checks, workspace carving, route selection, launch geometry) under the
// sanitizers, on "device" pointers that nothing on the host may dereference: they point
// into a PROT_NONE mapping, so a host access through one of them is a crash the test sees.
//
// After every call the harness checks what was recorded: a call that returns an error must
// not have launched anything, and every launch of a successful call must have a grid and
// a workgroup the hardware accepts.
#include <hip/hip_runtime_api.h>
#include <sys/mman.h>

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <string>
#include <vector>

#include "tdq.h"
#include "../../paper_2604_16855_amd/csrc/tdq_internal.hpp"

// ---------------------------------------------------------------------------
// the stand-in runtime
// ---------------------------------------------------------------------------
namespace {
struct Launch {
  std::string name;
  dim3 grid, block;
  size_t lds;
};
std::vector<Launch> g_launches;
// kernels register from static constructors of the library's objects, which may run before
// this file's: the table is built on first use
std::map<const void*, std::string>& names() {
  static std::map<const void*, std::string>* m = new std::map<const void*, std::string>();
  return *m;
}
struct {
  dim3 grid, block;
  size_t lds;
  hipStream_t st;
} g_cfg;
void* g_symbol_mem = nullptr;
int g_fail = 0;

void fail(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  fprintf(stderr, "FAIL: ");
  vfprintf(stderr, fmt, ap);
  fprintf(stderr, "\n");
  va_end(ap);
  ++g_fail;
}
}  // namespace

extern "C" {
void** __hipRegisterFatBinary(const void*) {
  static void* handle = nullptr;
  return &handle;
}
void __hipUnregisterFatBinary(void**) {}
void __hipRegisterFunction(void**, const void* host_fn, char*, const char* device_name, unsigned, void*,
                           void*, dim3*, dim3*, int*) {
  names()[host_fn] = device_name;
}
void __hipRegisterVar(void**, void*, char*, char*, int, size_t, int, int) {}
hipError_t __hipPushCallConfiguration(dim3 grid, dim3 block, size_t lds, hipStream_t st) {
  g_cfg.grid = grid;
  g_cfg.block = block;
  g_cfg.lds = lds;
  g_cfg.st = st;
  return hipSuccess;
}
hipError_t __hipPopCallConfiguration(dim3* grid, dim3* block, size_t* lds, hipStream_t* st) {
  *grid = g_cfg.grid;
  *block = g_cfg.block;
  *lds = g_cfg.lds;
  *st = g_cfg.st;
  return hipSuccess;
}
hipError_t hipLaunchKernel(const void* fn, dim3 grid, dim3 block, void**, size_t lds, hipStream_t) {
  auto it = names().find(fn);
  g_launches.push_back({it == names().end() ? std::string("?") : it->second, grid, block, lds});
  return hipSuccess;
}
hipError_t hipGetLastError(void) { return hipSuccess; }
hipError_t hipGetDevice(int* dev) {
  *dev = 0;
  return hipSuccess;
}
hipError_t hipFuncSetAttribute(const void*, hipFuncAttribute, int) { return hipSuccess; }
hipError_t hipGetSymbolAddress(void** ptr, const void*) {
  *ptr = g_symbol_mem;
  return hipSuccess;
}
hipError_t hipDeviceGetAttribute(int* v, hipDeviceAttribute_t attr, int) {
  *v = attr == hipDeviceAttributeMultiprocessorCount ? 256 : 0;
  return hipSuccess;
}
}

// ---------------------------------------------------------------------------
// checks
// ---------------------------------------------------------------------------
namespace {
int g_calls = 0;

void check_launches(const char* what) {
  for (const Launch& l : g_launches) {
    const unsigned long long threads = (unsigned long long)l.block.x * l.block.y * l.block.z;
    const bool ok = l.grid.x >= 1 && l.grid.y >= 1 && l.grid.z >= 1 && l.grid.x <= 0x7fffffffu &&
                    l.grid.y <= 65535u && l.grid.z <= 65535u && threads >= 1 && threads <= 1024 &&
                    l.lds <= 160u * 1024u;
    if (!ok)
      fail("%s: %s launched with grid (%u,%u,%u) block (%u,%u,%u) lds %zu", what, l.name.c_str(), l.grid.x,
           l.grid.y, l.grid.z, l.block.x, l.block.y, l.block.z, l.lds);
  }
}

// rc of a call that must succeed and launch something
void expect_ok(const char* what, int rc) {
  ++g_calls;
  if (rc != TDQ_OK) fail("%s: status %d (%s)", what, rc, tdq_status_string(rc));
  if (g_launches.empty()) fail("%s: no kernel launched", what);
  check_launches(what);
  g_launches.clear();
}

// rc of a call that must be refused before anything is launched
void expect_err(const char* what, int rc, int want) {
  ++g_calls;
  if (rc != want) fail("%s: status %d (%s), expected %d", what, rc, tdq_status_string(rc), want);
  if (!g_launches.empty()) fail("%s: %zu kernels launched by a refused call", what, g_launches.size());
  g_launches.clear();
}

bool launched(const char* fragment) {
  for (const Launch& l : g_launches)
    if (l.name.find(fragment) != std::string::npos) return true;
  return false;
}

// A "device" buffer: address space nothing may touch.
unsigned char* g_dev = nullptr;
const size_t kDevSpan = (size_t)1 << 40;
template <typename T>
T* dev(size_t offset_bytes) {
  return reinterpret_cast<T*>(g_dev + offset_bytes);
}

void check_layout(int B, int T, int C, tdq_dtype dt, int G) {
  tdq_params p;
  tdq_default_params(&p);
  p.n_groups = G;
  const size_t bytes = tdq_workspace_bytes(B, T, C, dt, &p);
  const tdq::LevelPlan lp = tdq::make_level_plan(dt, G);
  const tdq::WorkspaceLayout w = tdq::make_layout(B, T, G, lp);
  ++g_calls;
  if (bytes != w.total) fail("workspace_bytes %zu != layout total %zu (B=%d T=%d G=%d)", bytes, w.total, B, T, G);
  const size_t off[] = {w.status, w.img_flag, w.r, w.mean, w.m2, w.part, w.grp, w.hist, w.br, w.bhist, w.total};
  for (size_t i = 0; i + 1 < sizeof(off) / sizeof(off[0]); ++i) {
    if (off[i] % 256) fail("workspace piece %zu not 256-aligned", i);
    if (off[i] > off[i + 1]) fail("workspace pieces %zu and %zu overlap", i, i + 1);
  }
  if ((size_t)B * T * sizeof(double) > w.m2 - w.mean) fail("mean piece too small");
  if (lp.n_levels < 1 || lp.n_levels > tdq::kMaxLevels) fail("level plan: %d levels", lp.n_levels);
  int bits = 0;
  for (int l = 0; l < lp.n_levels; ++l) {
    bits += lp.bits[l];
    if (lp.bits[l] < 1 || lp.bits[l] > tdq::kMaxLevelBits) fail("level %d: %d bits", l, lp.bits[l]);
    if ((size_t)G << lp.bits[l] > (size_t)tdq::kHistLdsWords && lp.bits[l] > 1)
      fail("level %d: %d sets x %d bits exceed the LDS histogram", l, G, lp.bits[l]);
  }
  if (bits != lp.key_bits) fail("level plan covers %d of %d key bits", bits, lp.key_bits);
}

struct Shape {
  int B, T, C, G;
  tdq_dtype dt;
};

void token_set_path(const Shape& s) {
  char tag[128];
  snprintf(tag, sizeof tag, "B=%d T=%d C=%d G=%d dt=%d", s.B, s.T, s.C, s.G, (int)s.dt);
  tdq_params p;
  tdq_default_params(&p);
  p.n_groups = s.G;
  const size_t ws = tdq_workspace_bytes(s.B, s.T, s.C, s.dt, &p);
  if (ws == 0) {
    fail("%s: workspace size 0", tag);
    return;
  }
  void* X = dev<void>(0);
  int32_t* gid = dev<int32_t>((size_t)1 << 36);
  float* clip = dev<float>((size_t)2 << 36);
  float* scale = dev<float>((size_t)3 << 36);
  tdq_group_stats* st = dev<tdq_group_stats>((size_t)4 << 36);
  void* wsp = dev<void>((size_t)5 << 36);
  uint8_t* Q = dev<uint8_t>((size_t)6 << 36);
  const int64_t ld_q = (s.C + 1) / 2;
  const std::string t = tag;
  expect_ok((t + " calibrate").c_str(),
            tdq_calibrate_groups(X, s.dt, s.B, s.T, s.C, s.C, &p, gid, clip, scale, st, wsp, ws, nullptr));
  for (unsigned flags : {TDQ_FLAG_C1 | TDQ_FLAG_C2 | TDQ_FLAG_EXACT_SELECT, 0u, TDQ_FLAG_C1}) {
    tdq_params q = p;
    q.flags = flags;
    expect_ok((t + " calibrate flags").c_str(),
              tdq_calibrate_groups(X, s.dt, s.B, s.T, s.C, s.C, &q, gid, clip, scale, nullptr, wsp, ws, nullptr));
  }
  {
    tdq_params q = p;
    q.base_pct = 0.999;
    const size_t ws2 = tdq_workspace_bytes(s.B, s.T, s.C, s.dt, &q);
    expect_ok((t + " calibrate base percentile").c_str(),
              tdq_calibrate_groups(X, s.dt, s.B, s.T, s.C, s.C + 8, &q, gid, clip, scale, st, wsp, ws2, nullptr));
  }
  expect_err((t + " calibrate small workspace").c_str(),
             tdq_calibrate_groups(X, s.dt, s.B, s.T, s.C, s.C, &p, gid, clip, scale, st, wsp, ws - 1, nullptr),
             TDQ_ERR_WORKSPACE);
  expect_err((t + " calibrate misaligned workspace").c_str(),
             tdq_calibrate_groups(X, s.dt, s.B, s.T, s.C, s.C, &p, gid, clip, scale, st,
                                  static_cast<char*>(wsp) + 8, ws, nullptr),
             TDQ_ERR_WORKSPACE);
  if (ws <= TDQ_STATIC_SCRATCH_BYTES)
    expect_ok((t + " calibrate static").c_str(),
              tdq_calibrate_groups_static(X, s.dt, s.B, s.T, s.C, s.C, &p, gid, clip, scale, st,
                                          dev<uint32_t>((size_t)7 << 36), nullptr));
  else
    expect_err((t + " calibrate static, too large").c_str(),
               tdq_calibrate_groups_static(X, s.dt, s.B, s.T, s.C, s.C, &p, gid, clip, scale, st, nullptr, nullptr),
               TDQ_ERR_WORKSPACE);
  expect_ok((t + " quantize").c_str(),
            tdq_quantize_act(X, s.dt, s.B, s.T, s.C, s.C, &p, gid, clip, scale, Q, ld_q, nullptr));
  expect_ok((t + " quantize f6").c_str(),
            tdq_quantize_act_f6(X, s.dt, s.B, s.T, s.C, s.C, &p, gid, clip, scale, Q, nullptr));
  expect_ok((t + " diagnostics").c_str(),
            tdq_group_diagnostics(X, s.dt, s.B, s.T, s.C, s.C, &p, gid, clip, scale,
                                  dev<uint64_t>((size_t)7 << 36), dev<uint64_t>((size_t)8 << 36), nullptr));
  expect_ok((t + " range disparity").c_str(),
            tdq_range_disparity(X, s.dt, s.B, s.T, s.C, s.C, clip, scale, dev<float>((size_t)7 << 36),
                                dev<float>((size_t)8 << 36), nullptr));
  {
    expect_ok((t + " tokenize").c_str(),
              tdq_tokenize_chw(X, s.dt, s.B, s.C, s.T, s.T, (int64_t)s.C * s.T, dev<void>((size_t)9 << 36), s.C,
                               nullptr));
    expect_ok((t + " calibrate chw").c_str(),
              tdq_calibrate_groups_chw(X, s.dt, s.B, s.C, s.T, s.T, (int64_t)s.C * s.T, &p,
                                       dev<void>((size_t)9 << 36), s.C, gid, clip, scale, st, wsp, ws, nullptr));
  }
  if (s.G <= TDQ_FUSED_MAX_GROUPS) {
    const int rc = tdq_calibrate_quantize_fused(X, s.dt, s.B, s.T, s.C, s.C, &p, gid, clip, scale, st,
                                                dev<uint32_t>((size_t)7 << 36), Q, ld_q, wsp, ws, nullptr);
    if (rc == TDQ_ERR_UNSUPPORTED) {   // an image too large for one workgroup's LDS: the documented refusal
      expect_err((t + " fused, image too large").c_str(), rc, TDQ_ERR_UNSUPPORTED);
    } else {
      expect_ok((t + " fused").c_str(), rc);
    }
  }
  // blocks path
  tdq_params pb = p;
  pb.chan_group = TDQ_BLOCK;
  pb.n_groups = 1;
  const int64_t KB = (s.C + TDQ_BLOCK - 1) / TDQ_BLOCK;
  expect_ok((t + " quantize blocks").c_str(),
            tdq_quantize_act_blocks(X, s.dt, s.B, s.T, s.C, s.C, &pb, Q, ld_q, clip, scale, KB, nullptr));
  expect_ok((t + " quantize blocks f6").c_str(),
            tdq_quantize_act_blocks_f6(X, s.dt, s.B, s.T, s.C, s.C, &pb, Q, clip, scale, KB, nullptr));
  expect_ok((t + " quantize blocks chw").c_str(),
              tdq_quantize_act_blocks_chw(X, s.dt, s.B, s.C, s.T, s.T, (int64_t)s.C * s.T, &pb, Q, ld_q, clip,
                                          scale, KB, nullptr));
}

void linear_path(int B, int T, int K, int N, int G, tdq_dtype ydt, bool want_roll) {
  char tag[128];
  snprintf(tag, sizeof tag, "linear B=%d T=%d K=%d N=%d G=%d ydt=%d", B, T, K, N, G, (int)ydt);
  const std::string t = tag;
  const uint8_t* Qx = dev<uint8_t>(0);
  const uint8_t* Qw = dev<uint8_t>((size_t)1 << 36);
  const int32_t* gid = dev<int32_t>((size_t)2 << 36);
  const float* sc = dev<float>((size_t)3 << 36);
  const float* ws = dev<float>((size_t)4 << 36);
  const float* bias = dev<float>((size_t)5 << 36);
  void* Y = dev<void>((size_t)6 << 36);
  const int64_t ld = 16 * (((int64_t)K + 31) / 32);   // rows of whole 16-byte pieces
  ++g_calls;
  int rc = tdq_w4a4_linear(Qx, ld, gid, sc, B, T, K, N, G, Qw, ld, ws, bias, Y, ydt, N, nullptr, nullptr);
  if (rc != TDQ_OK) fail("%s: status %d", tag, rc);
  if (g_launches.size() != 1) fail("%s: %zu launches", tag, g_launches.size());
  if (want_roll != launched("gemm_roll")) fail("%s: rolling kernel %s", tag, want_roll ? "not chosen" : "chosen");
  check_launches(tag);
  g_launches.clear();
  expect_ok((t + " accumulator dump").c_str(),
            tdq_w4a4_linear(Qx, ld, gid, sc, B, T, K, N, G, Qw, ld, ws, nullptr, Y, ydt, N,
                            dev<int32_t>((size_t)7 << 36), nullptr));
  expect_ok((t + " no id array").c_str(),
            tdq_w4a4_linear(Qx, ld, nullptr, sc, B, T, K, N, 1, Qw, ld, ws, bias, Y, ydt, N, nullptr, nullptr));
  expect_ok((t + " f6").c_str(),
            tdq_w4a4_linear_f6(Qx, gid, sc, B, T, K, N, G, Qw, ws, bias, Y, ydt, N, nullptr, nullptr));
  const int64_t KB = (K + TDQ_BLOCK - 1) / TDQ_BLOCK, M = (int64_t)B * T;
  expect_ok((t + " blocks").c_str(),
            tdq_w4a4_linear_blocks(Qx, ld, sc, KB, M, K, N, Qw, ld, ws, bias, Y, ydt, N, nullptr));
  expect_ok((t + " blocks f6").c_str(),
            tdq_w4a4_linear_blocks_f6(Qx, sc, KB, M, K, N, Qw, ws, bias, Y, ydt, N, nullptr));
  expect_ok((t + " pack f6").c_str(), tdq_pack_codes_f6(Qx, ld, M, K, dev<uint8_t>((size_t)8 << 36), nullptr));
  expect_ok((t + " quantize weight").c_str(),
            tdq_quantize_weight(dev<float>((size_t)9 << 36), N, K, K, dev<uint8_t>((size_t)10 << 36), ld,
                                dev<float>((size_t)11 << 36), nullptr));
  if (tdq_f6_bytes(M, K) < (size_t)((M + 31) / 32) * ((K + 127) / 128) * 2 * 64 * 24) fail("%s: f6 bytes", tag);
}

void refusals() {
  tdq_params p;
  tdq_default_params(&p);
  void* X = dev<void>(0);
  int32_t* gid = dev<int32_t>((size_t)1 << 36);
  float* f = dev<float>((size_t)2 << 36);
  void* wsp = dev<void>((size_t)5 << 36);
  uint8_t* Q = dev<uint8_t>((size_t)6 << 36);
  const size_t ws = tdq_workspace_bytes(2, 64, 64, TDQ_F16, &p);
  expect_err("calibrate: X null", tdq_calibrate_groups(nullptr, TDQ_F16, 2, 64, 64, 64, &p, gid, f, f, nullptr, wsp, ws, nullptr), TDQ_ERR_NULL);
  expect_err("calibrate: params null", tdq_calibrate_groups(X, TDQ_F16, 2, 64, 64, 64, nullptr, gid, f, f, nullptr, wsp, ws, nullptr), TDQ_ERR_NULL);
  expect_err("calibrate: B = 0", tdq_calibrate_groups(X, TDQ_F16, 0, 64, 64, 64, &p, gid, f, f, nullptr, wsp, ws, nullptr), TDQ_ERR_SHAPE);
  expect_err("calibrate: ld < C", tdq_calibrate_groups(X, TDQ_F16, 2, 64, 64, 63, &p, gid, f, f, nullptr, wsp, ws, nullptr), TDQ_ERR_SHAPE);
  expect_err("calibrate: B > 65535", tdq_calibrate_groups(X, TDQ_F16, TDQ_MAX_IMAGES + 1, 4, 64, 64, &p, gid, f, f, nullptr, wsp, ws, nullptr), TDQ_ERR_SHAPE);
  expect_err("calibrate: B T > 2^30", tdq_calibrate_groups(X, TDQ_F16, 1 << 15, 1 << 16, 64, 64, &p, gid, f, f, nullptr, wsp, ws, nullptr), TDQ_ERR_SHAPE);
  if (tdq_workspace_bytes(1 << 15, 1 << 16, 64, TDQ_F16, &p) != 0) fail("workspace_bytes of an invalid shape is not 0");
  ++g_calls;
  for (int bad = 0; bad < 8; ++bad) {
    tdq_params q = p;
    int want = TDQ_ERR_PARAM;
    switch (bad) {
      case 0: q.n_groups = 0; break;
      case 1: q.n_groups = TDQ_MAX_GROUPS + 1; break;
      case 2: q.act_bits = 3; break;
      case 3: q.act_bits = 8; want = TDQ_ERR_UNSUPPORTED; break;
      case 4: q.tau = 0.0; break;
      case 5: q.zr = 1.0; break;
      case 6: q.flags = 8; break;
      case 7: q.chan_group = 16; want = TDQ_ERR_UNSUPPORTED; break;
    }
    expect_err("calibrate: bad params", tdq_calibrate_groups(X, TDQ_F16, 2, 64, 64, 64, &q, gid, f, f, nullptr, wsp, ws, nullptr), want);
    expect_err("quantize: bad params", tdq_quantize_act(X, TDQ_F16, 2, 64, 64, 64, &q, gid, f, f, Q, 32, nullptr), want);
  }
  expect_err("quantize: ld_q", tdq_quantize_act(X, TDQ_F16, 2, 64, 64, 64, &p, gid, f, f, Q, 31, nullptr), TDQ_ERR_SHAPE);
  expect_err("quantize: no ids for G > 1", tdq_quantize_act(X, TDQ_F16, 2, 64, 64, 64, &p, nullptr, f, f, Q, 32, nullptr), TDQ_ERR_NULL);
  const uint8_t* Qc = Q;
  expect_err("linear: K too large", tdq_w4a4_linear(Qc, 1 << 16, gid, f, 1, 8, TDQ_MAX_K + 1, 8, 4, Qc, 1 << 16, f, nullptr, X, TDQ_F32, 8, nullptr, nullptr), TDQ_ERR_SHAPE);
  expect_ok("linear: largest K", tdq_w4a4_linear(Qc, 1 << 16, gid, f, 1, 8, TDQ_MAX_K, 8, 4, Qc, 1 << 16, f, nullptr, X, TDQ_F32, 8, nullptr, nullptr));
  expect_err("linear: misaligned codes", tdq_w4a4_linear(Qc + 8, 32, gid, f, 1, 8, 64, 8, 4, Qc, 32, f, nullptr, X, TDQ_F32, 8, nullptr, nullptr), TDQ_ERR_ALIGN);
  expect_err("linear: ld_y < N", tdq_w4a4_linear(Qc, 32, gid, f, 1, 8, 64, 8, 4, Qc, 32, f, nullptr, X, TDQ_F32, 7, nullptr, nullptr), TDQ_ERR_SHAPE);
  expect_err("linear: G", tdq_w4a4_linear(Qc, 32, gid, f, 1, 8, 64, 8, 0, Qc, 32, f, nullptr, X, TDQ_F32, 8, nullptr, nullptr), TDQ_ERR_PARAM);
  expect_err("probe: kind", tdq_probe(17, X, 1 << 20, 1, 0, nullptr), TDQ_ERR_PARAM);
  expect_err("probe: no buffer", tdq_probe(TDQ_PROBE_READ, nullptr, 1 << 20, 1, 0, nullptr), TDQ_ERR_NULL);
  for (int kind = TDQ_PROBE_READ; kind <= TDQ_PROBE_FMA_4WAVES; ++kind)
    expect_ok("probe", tdq_probe(kind, X, (size_t)1 << 30, 4, 1024, nullptr));
}
}  // namespace

int main() {
  g_dev = static_cast<unsigned char*>(
      mmap(nullptr, kDevSpan, PROT_NONE, MAP_PRIVATE | MAP_ANONYMOUS | MAP_NORESERVE, -1, 0));
  if (g_dev == MAP_FAILED) {
    perror("mmap");
    return 2;
  }
  g_symbol_mem = g_dev + ((size_t)15 << 36);
  if (tdq_version() != TDQ_VERSION) fail("version");

  // the workloads of the paper's evaluation as the benchmark sizes them, small and ragged
  // shapes, the largest set count, one token per image, very many images
  const Shape shapes[] = {
      {32, 4096, 1024, 32, TDQ_F16}, {32, 4096, 4096, 32, TDQ_F32}, {4, 64, 64, 4, TDQ_F16},
      {8, 256, 320, 8, TDQ_F32},     {3, 77, 193, 5, TDQ_F16},      {1, 1, 1, 1, TDQ_F32},
      {2, 4096, 40, 256, TDQ_F16},   {2, 300, 1280, 256, TDQ_F32},  {65535, 4, 32, 2, TDQ_F16},
      {1, 1 << 20, 16, 64, TDQ_F16}, {5, 1000, 4097, 33, TDQ_F16},  {7, 129, 8200, 3, TDQ_F32},
  };
  for (const Shape& s : shapes) {
    check_layout(s.B, s.T, s.C, s.dt, s.G);
    token_set_path(s);
  }
  for (int G = 1; G <= TDQ_MAX_GROUPS; ++G) {
    check_layout(2, 100, 64, TDQ_F16, G);
    check_layout(2, 100, 64, TDQ_F32, G);
  }
  linear_path(32, 4096, 1024, 4096, 32, TDQ_F16, true);
  linear_path(32, 4096, 4096, 1024, 32, TDQ_F32, true);
  linear_path(16, 4096, 4096, 1024, 32, TDQ_F32, false);   // fewer than 8 tiles per workgroup
  linear_path(4, 64, 64, 256, 4, TDQ_F32, false);
  linear_path(3, 77, 193, 130, 5, TDQ_F16, false);
  linear_path(8, 256, 320, 1280, 8, TDQ_F16, false);
  linear_path(1, 1, 1, 1, 1, TDQ_F32, false);
  linear_path(2, 4096, 40, 40, 256, TDQ_F32, false);
  refusals();

  printf("%d calls checked, %d failures\n", g_calls, g_fail);
  return g_fail ? 1 : 0;
}
