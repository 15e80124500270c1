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
constexpr int kMaxLevels = 7;          // radix-select levels: a 31-bit key at >= 5 bits per level
                                       // (256 sets x 2^5 bins fill the LDS histogram)
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

// Key interval [lo, lo + width) that a sample says holds the k-th smallest
// magnitude key of an (image, token set), and what the sweep counted for it.
struct Bracket {
  unsigned lo;       // first key of the interval
  unsigned width;    // keys in the interval (one histogram bin each), 0 = nothing to count
  unsigned below;    // elements of the set with key < lo
  unsigned pad;
};
constexpr int kBracketLdsWords = 16384;   // 64 KiB of LDS histogram per workgroup (128 KiB, one
                                          // workgroup per CU, made the sweep 30 % slower)
// Fewest one-key bins per set worth sampling for: with fewer the interval (half-width
// bins / 2 keys, 1024 keys per octave) misses too often, and the multi-level radix
// select over all sets at once is the cheaper route from the start.
constexpr int kBracketMinBins = 256;

// Bins per set of the interval histogram: the LDS budget shared out to G sets, rounded
// down to a power of two, at most 2048 (0 = too many sets: use the multi-level radix
// select instead).
int bracket_bins(int G);

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
  size_t status;     // uint32[64]; word 0 = device status word, words 1 and 2 = sets whose
                     // rank the last binary16 calibration's sampled key interval missed in
                     // pass kPassZr and pass kPassBase (resolved by the per-set radix select)
  size_t img_flag;   // uint32[B]     per-image non-finite flag
  size_t r;          // float[M]      per-token range
  size_t mean;       // double[M]     per-token mean
  size_t m2;         // double[M]     per-token sum (x - mean)^2
  size_t part;       // per-workgroup partial set records of the assignment
  size_t grp;        // GroupWork[B*G]
  size_t hist;       // uint32 [levels][B*G][1 << bits[level]]
  size_t hist_level[kMaxLevels];   // offset of each level inside the workspace
  size_t br;         // Bracket[B*G]
  size_t bhist;      // uint32 [B*G][bracket_bins(G)]
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
  double base_pct;   // 0 = base radius is the set's maximum; (0,1) = rank quantile Q_p (Eq. DSTG_clip)
  unsigned flags;
};

// The rank select runs once per rank wanted of every set: pass kPassBase finds the
// base radius Q_p(|x|) (only when a percentile is asked for) and leaves it in
// GroupWork::c_base; pass kPassZr finds Q_zr(|x|) and applies the projection.
constexpr int kPassZr = 0;
constexpr int kPassBase = 1;

// ---- launch wrappers (each returns the hipError_t of its launch) -------------
hipError_t launch_token_stats(const void* X, tdq_dtype dt, int M, int C, long long ld,
                              float* r, double* mean, double* m2, hipStream_t st);
// Token-set assignment.  An image is shared by assign_split(T) workgroups, each of
// which leaves one partial record per set in `part`; the records are merged into
// GroupWork either by launch_finalize_groups or, for binary16 input, by the first
// kernel of the single-sweep rank select (launch_bracket).
constexpr int kAssignSplitMax = 8;
int assign_split(int T);
size_t assign_partial_bytes(int B, int G);
hipError_t launch_assign(const float* r, const double* mean, const double* m2, int B, int T, int C,
                         int G, int* gid, void* part, unsigned* img_flag, unsigned* status,
                         hipStream_t st);
// Arms the radix levels for one pass: working record of every set (rank of this pass;
// keep_base = keep the base radius an earlier pass left) and cleared level histograms.
hipError_t launch_finalize_groups(const void* part, int B, int T, int C, int G, const Scalars& sc,
                                  int pass, bool keep_base, GroupWork* grp, unsigned* hist,
                                  const LevelPlan& lp, hipStream_t st);
// The last level of pass kPassZr projects, that of pass kPassBase stores the base radius.
hipError_t launch_hist(const void* X, tdq_dtype dt, int B, int T, int C, long long ld, int G,
                       const int* gid, const GroupWork* grp, unsigned* hist_level, int shift,
                       int bits, hipStream_t st);
hipError_t launch_select(unsigned* hist_level, int B, int G, int shift, int bits, bool last,
                         tdq_dtype dt, const Scalars& sc, GroupWork* grp, float* clip,
                         float* scale, tdq_group_stats* stats, const unsigned* img_flag,
                         unsigned* status, int pass, hipStream_t st);
// single-sweep rank select for binary16 input
hipError_t launch_bracket(const void* X, int B, int T, int C, long long ld, int G, int W,
                          const int* gid, const void* part, const Scalars& sc, int pass,
                          bool keep_base, GroupWork* grp, Bracket* br, unsigned* bhist,
                          hipStream_t st);
hipError_t launch_bracket_hist(const void* X, int B, int T, int C, long long ld, int G, int W,
                               const int* gid, Bracket* br, unsigned* bhist, hipStream_t st);
hipError_t launch_bracket_finish(const void* X, int B, int T, int C, long long ld, int G, int W,
                                 const int* gid, const unsigned* bhist, bool force_miss,
                                 const Scalars& sc, int pass, GroupWork* grp, const Bracket* br,
                                 float* clip, float* scale, tdq_group_stats* stats,
                                 const unsigned* img_flag, unsigned* status, hipStream_t st);
hipError_t launch_quantize(const void* X, tdq_dtype dt, int B, int T, int C, long long ld, int G,
                           const int* gid, const float* clip, const float* scale, uint8_t* Q,
                           long long ld_q, hipStream_t st);
hipError_t launch_quantize_blocks(const void* X, tdq_dtype dt, long long M, int C, long long ld,
                                  int kq, int kp, const Scalars& sc, uint8_t* Q, long long ld_q,
                                  float* bscale, float* bclip, long long ld_s, hipStream_t st);
hipError_t launch_w4a4_gemm_blocks(const uint8_t* Qx, long long ld_q, const float* bscale,
                                   long long ld_s, int M, int K, int N, const uint8_t* Qw,
                                   long long ld_w, const float* w_scale, const float* bias, void* Y,
                                   tdq_dtype y_dt, long long ld_y, hipStream_t st);
hipError_t launch_quantize_blocks_f6(const void* X, tdq_dtype dt, long long M, int C, long long ld,
                                     int kq, int kp, const Scalars& sc, uint8_t* F, float* bscale,
                                     float* bclip, long long ld_s, hipStream_t st);
hipError_t launch_quantize_blocks_chw(const void* X, tdq_dtype dt, int B, int C, int T, long long ld_c,
                                      long long ld_b, int kq, int kp, const Scalars& sc, uint8_t* Q,
                                      long long ld_q, float* bscale, float* bclip, long long ld_s,
                                      hipStream_t st);
hipError_t launch_fused_small(const void* X, tdq_dtype dt, int B, int T, int C, long long ld, int G,
                              const Scalars& sc, float* r, double* mean, double* m2, int* gid,
                              float* clip, float* scale, tdq_group_stats* stats,
                              unsigned* image_flags, uint8_t* Q, long long ld_q, hipStream_t st);
hipError_t launch_range_disparity(const void* X, tdq_dtype dt, int B, int T, int C, long long ld,
                                  float* token_median, float* token_max, float* disparity,
                                  float* max_abs, hipStream_t st);
hipError_t launch_tokenize_stats_chw(const void* X, tdq_dtype dt, int B, int C, int T, long long ld_c,
                                     long long ld_b, void* Xt, long long ld_xt, float* r, double* mean,
                                     double* m2, hipStream_t st);
hipError_t launch_quantize_f6(const void* X, tdq_dtype dt, int B, int T, int C, long long ld, int G,
                              const int* gid, const float* clip, const float* scale, uint8_t* F,
                              hipStream_t st);
hipError_t launch_pack_f6(const uint8_t* Q, long long ld, int R, int K, uint8_t* F, hipStream_t st);
hipError_t launch_w4a4_gemm_f6(const uint8_t* A6, const uint8_t* B6, int K, const int* gid,
                               const float* scale, int M, int T, int N, int G, const float* w_scale,
                               const float* bias, void* Y, tdq_dtype y_dt, long long ld_y,
                               int* acc_dump, hipStream_t st);
hipError_t launch_w4a4_gemm_blocks_f6(const uint8_t* A6, const uint8_t* B6, const float* bscale,
                                      long long ld_s, int M, int K, int N, const float* w_scale,
                                      const float* bias, void* Y, tdq_dtype y_dt, long long ld_y,
                                      hipStream_t st);
hipError_t launch_tokenize_chw(const void* X, tdq_dtype dt, int B, int C, int T, long long ld_c,
                               long long ld_b, void* Xt, long long ld_xt, hipStream_t st);
hipError_t launch_group_diag(const void* X, tdq_dtype dt, int B, int T, int C, long long ld, int G,
                             const int* gid, const float* clip, const float* scale,
                             unsigned long long* zero_count, unsigned long long* clipped_count,
                             hipStream_t st);
hipError_t launch_quantize_weight(const float* W, int N, int K, long long ld_in, uint8_t* Qw,
                                  long long ld_w, float* w_scale, hipStream_t st);
hipError_t launch_w4a4_gemm(const uint8_t* Qx, long long ld_q, const int* gid, const float* scale,
                            int M, int T, int K, int N, int G, const uint8_t* Qw, long long ld_w,
                            const float* w_scale, const float* bias, void* Y, tdq_dtype y_dt,
                            long long ld_y, int* acc_dump, hipStream_t st);

}  // namespace tdq
