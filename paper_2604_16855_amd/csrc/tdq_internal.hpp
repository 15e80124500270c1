// Internal declarations shared by the translation units of libtdq (host side
// launch wrappers, workspace layout).  Nothing here is part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "tdq.h"

namespace tdq {

constexpr int kQMax = 7;
constexpr int kQMin = -8;
constexpr int kOctaveFloor = 24;       // assignment: keys > 24 octaves below the top share set 0
constexpr int kMaxLevels = 6;          // radix-select levels (31-bit key / >= 6 bits per level)
constexpr int kHistLdsWords = 8192;    // 32 KiB of LDS histogram per workgroup
constexpr int kMaxLevelBits = 11;

// Per-(image, token set) working record of the calibration, kept in the workspace.
struct GroupWork {
  long long n;          // elements = tokens * C
  long long k_rem;      // rank still to be resolved below the current prefix
  unsigned prefix;      // magnitude-key bits fixed so far (high bits of thr)
  unsigned tokens;      // tokens in the set
  float c_base;         // max |x|
  float sigma;          // population std + eps_std
};

// How the magnitude key (15 bits for fp16, 31 for fp32) is split into radix levels.
struct LevelPlan {
  int n_levels;
  int bits[kMaxLevels];
  int shift[kMaxLevels];   // key >> shift gives this level's digit in the low `bits`
  int key_bits;
};

LevelPlan make_level_plan(tdq_dtype dt, int G);

// Byte offsets of the pieces of the calibration workspace (all 256-aligned).
struct WorkspaceLayout {
  size_t status;     // uint32[64]; word 0 is the device status word
  size_t img_flag;   // uint32[B]     per-image non-finite flag
  size_t r;          // float[M]      per-token range
  size_t s1;         // double[M]     per-token sum x
  size_t s2;         // double[M]     per-token sum x^2
  size_t grp;        // GroupWork[B*G]
  size_t hist;       // uint32 [levels][B*G][1 << bits[level]]
  size_t hist_level[kMaxLevels];   // offset of each level inside the workspace
  size_t total;
};

WorkspaceLayout make_layout(int B, int T, int G, const LevelPlan& lp);

struct Scalars {   // fp32 constants of the projection, rounded once on the host
  float qmax_tau;  // 7 * tau
  float two_qmax;  // 14
  float qmax;      // 7
  float eps_scale;
  double eps_std;
  double zr;
  unsigned flags;
};

// ---- launch wrappers (each returns the hipError_t of its launch) -------------
hipError_t launch_token_stats(const void* X, tdq_dtype dt, int M, int C, long long ld,
                              float* r, double* s1, double* s2, hipStream_t st);
hipError_t launch_assign(const float* r, const double* s1, const double* s2, int B, int T, int C,
                         int G, const Scalars& sc, int* gid, GroupWork* grp, unsigned* hist,
                         unsigned* img_flag, const LevelPlan& lp, hipStream_t st);
hipError_t launch_hist(const void* X, tdq_dtype dt, int B, int T, int C, long long ld, int G,
                       const int* gid, const GroupWork* grp, unsigned* hist_level, int shift,
                       int bits, hipStream_t st);
hipError_t launch_select(unsigned* hist_level, int B, int G, int shift, int bits, bool last,
                         tdq_dtype dt, const Scalars& sc, GroupWork* grp, float* clip,
                         float* scale, tdq_group_stats* stats, const unsigned* img_flag,
                         unsigned* status, hipStream_t st);
hipError_t launch_quantize(const void* X, tdq_dtype dt, int B, int T, int C, long long ld, int G,
                           const int* gid, const float* clip, const float* scale, uint8_t* Q,
                           long long ld_q, hipStream_t st);
hipError_t launch_quantize_weight(const float* W, int N, int K, long long ld_in, uint8_t* Qw,
                                  long long ld_w, float* w_scale, hipStream_t st);
hipError_t launch_w4a4_gemm(const uint8_t* Qx, long long ld_q, const int* gid, const float* scale,
                            int M, int T, int K, int N, int G, const uint8_t* Qw, long long ld_w,
                            const float* w_scale, const float* bias, void* Y, tdq_dtype y_dt,
                            long long ld_y, int* acc_dump, hipStream_t st);

}  // namespace tdq
