/*
 * tdq.h — C ABI of libtdq: the DSTG + DCRP W4A4 quantized linear path of COD-TDQ
 * as hand-written HIP kernels for gfx950 (MI355X).
 *
 * Notation follows the paper: an activation tensor X[B, T, C] (B images, T tokens
 * per image, C channels), a weight W[N, C] with per-output-channel scales s[N],
 * q_max = 7, q_min = -8, step-to-dispersion bound tau, zero-bin mass bound zr.
 *
 * A quantization group here is (image b, token set S_j), j < G: every token of an
 * image is put into one of G token sets by its range, and all C channels of all
 * tokens of a set share one clip radius c[b, j] and one step Delta[b, j].
 * G = 1 is per-image ("per-tensor") quantization.
 *
 * Conventions for every entry point
 *  - All tensor pointers are DEVICE pointers owned by the caller.  The library
 *    keeps no state, allocates nothing, launches asynchronously on `stream`
 *    (a hipStream_t passed as void*, NULL = the default stream) and never
 *    synchronises.
 *  - Arguments are checked on the host before anything is launched; a bad
 *    argument returns a negative tdq_status and launches nothing.  A HIP launch
 *    error returns TDQ_ERR_HIP.  No C++ exception crosses the ABI.
 *  - Row-major; leading dimensions (ld_*) are in ELEMENTS of the array they
 *    belong to (bytes for the packed-code arrays).
 *  - Packed int4 codes: two's-complement nibbles, element 2i in bits 0-3 and
 *    element 2i+1 in bits 4-7 of byte i of the row; an odd C leaves the last high
 *    nibble zero.  (The paper leaves packing to the implementation, Sec. 3.3
 *    "Static Symmetric Weight Quantization".)
 */
#ifndef TDQ_H
#define TDQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TDQ_VERSION 110

typedef enum { TDQ_F16 = 0, TDQ_F32 = 1 } tdq_dtype;

typedef enum {
  TDQ_OK = 0,
  TDQ_ERR_NULL = -1,        /* a required pointer is NULL                        */
  TDQ_ERR_SHAPE = -2,       /* B, T, C, N, K or a leading dimension is invalid   */
  TDQ_ERR_PARAM = -3,       /* tdq_params out of range                           */
  TDQ_ERR_WORKSPACE = -4,   /* workspace too small or misaligned                 */
  TDQ_ERR_DTYPE = -5,       /* unknown tdq_dtype                                 */
  TDQ_ERR_HIP = -6,         /* a HIP call failed                                 */
  TDQ_ERR_UNSUPPORTED = -7, /* valid request that this build does not implement  */
  TDQ_ERR_ALIGN = -8        /* pointer / leading dimension alignment             */
} tdq_status;

#define TDQ_FLAG_C1 1u /* constraint C1: Delta <= tau * sigma   (Eq. tau_constraint) */
#define TDQ_FLAG_C2 2u /* constraint C2: Delta/2 <= Q_zr(|x|)   (Eq. zr_constraint)  */
/* Validation switch, no effect on the result: resolve the zr rank of every token set
 * of a binary16 input by the per-set radix select alone (the route that is
 * otherwise taken only by a set whose sampled key interval missed the rank). */
#define TDQ_FLAG_EXACT_SELECT 256u

#define TDQ_MAX_GROUPS 256
/* Largest K of the whole-K contraction: its int32 accumulator holds 256 * acc (the codes
 * enter the matrix instruction as 16 * code), and |acc| <= 64 K, so 2^14 K < 2^31:
 * tdq_w4a4_linear refuses more with TDQ_ERR_SHAPE.  (The block-scaled and the f6 entry
 * points accumulate per block or in binary32 and take K up to 131072.) */
#define TDQ_MAX_K 131071
/* Largest B: images index a 16-bit grid axis of several kernels. */
#define TDQ_MAX_IMAGES 65535
#define TDQ_FUSED_MAX_GROUPS 64 /* most token sets per image of tdq_calibrate_quantize_fused */
#define TDQ_BLOCK 32 /* channel block g of the per-(token, block) entry points (Sec. 5 setup) */

/* Hyper-parameters (Supp. "Default Hyperparameters": tau = 1.0, zr = 0.2). */
typedef struct tdq_params {
  int32_t n_groups;   /* G token sets per image, 1..TDQ_MAX_GROUPS                */
  int32_t chan_group; /* channel block g: 0 = whole row (token-set entry points),  */
                      /* TDQ_BLOCK = the *_blocks entry points; else UNSUPPORTED   */
  int32_t act_bits;   /* 4                                                        */
  uint32_t flags;     /* TDQ_FLAG_C1 | TDQ_FLAG_C2 = DCRP; 0 = base radius only   */
  double tau;         /* > 0                                                      */
  double zr;          /* in (0,1); rank k = ceil(zr * n) in binary64              */
  double base_pct;    /* 0 or 1 = max-abs base radius; p in (0,1) = rank quantile */
                      /* Q_p(|x|), the ceil(p n)-th smallest (Eq. DSTG_clip)      */
  float eps_scale;    /* floor of clip radius and step, 1e-8 (Supp. numerical conv.) */
  float eps_std;      /* added to the population std, 1e-12                       */
} tdq_params;

/* What bound the projection c = min(c_base, c_tau, c_zr) of Eq. (dcrp). */
enum { TDQ_BIND_BASE = 0, TDQ_BIND_C1 = 1, TDQ_BIND_C2 = 2, TDQ_BIND_EPS = 3, TDQ_BIND_EMPTY = 4 };

/* Per-(image, token set) record written by tdq_calibrate_groups. */
typedef struct tdq_group_stats {
  int64_t n;      /* elements in the group = tokens * C                          */
  int64_t k;      /* rank of the zr quantile, clamp(ceil(zr n), 1, n)             */
  float c_base;   /* max |x|                              (Eq. DSTG_clip)          */
  float sigma;    /* population std + eps_std                                     */
  float thr;      /* k-th smallest |x| (an element of the data)                   */
  float c_tau;    /* q_max * tau * sigma                  (Eq. tau_constraint)     */
  float c_zr;     /* 2 * q_max * thr                      (Eq. zr_constraint)      */
  float clip;     /* c   after projection and eps floor   (Eq. dcrp)               */
  float scale;    /* Delta = max(c / q_max, eps_scale)    (Eq. clipx)              */
  uint32_t bind;  /* TDQ_BIND_*                                                   */
} tdq_group_stats;

/* Bits of the device status word (first uint32 of the workspace after a call
 * to tdq_calibrate_groups; read it back after synchronising the stream). */
#define TDQ_DEV_NONFINITE 1u /* X holds an Inf or NaN: results undefined          */
/* The second uint32 of the workspace is a diagnostic: after a calibration of
 * binary16 input, the number of (image, token set) pairs whose zr rank was resolved
 * by the per-set radix select because the sampled key interval missed it (or
 * because TDQ_FLAG_EXACT_SELECT was set).  It has no bearing on the results. */

int tdq_version(void);
const char* tdq_status_string(int status);

/* Fills *p with the paper's defaults (G = 8, tau = 1, zr = 0.2, DCRP on). */
void tdq_default_params(tdq_params* p);

/* Bytes of device scratch tdq_calibrate_groups needs for this shape; 0 if the
 * shape or params are invalid.  The workspace must be 256-byte aligned. */
size_t tdq_workspace_bytes(int32_t B, int32_t T, int32_t C, tdq_dtype dt, const tdq_params* p);

/*
 * DSTG statistics + token-set assignment + DCRP projection.
 *
 *  1. per token: range r_t = max_c |x_tc|, mean and sum (x - mean)^2
 *     (Sec. 4.2: base radius and within-group dispersion);
 *  2. per image: gid[t] in [0, G) from the bit pattern of r_t — G equal-width
 *     bins between the image's smallest and largest key, the lower end raised to
 *     at most 24 octaves below the top (integer arithmetic, exact);
 *  3. per group: c_base = max r_t, sigma = population std + eps_std;
 *     thr = the ceil(zr n)-th smallest |x| of the group, exact: an order statistic
 *     of the magnitude bit patterns found with LDS histograms (binary16 input: one
 *     sweep over a key interval chosen from a sample, verified by counting, with a
 *     radix select for any set the interval missed; binary32 input: radix select);
 *  4. c = max(min(c_base, q_max tau sigma, 2 q_max thr), eps),
 *     Delta = max(c / q_max, eps)                    (Eqs. dcrp, clipx; Lemma 1).
 *
 * X        [B*T, ld_x] of dt, ld_x >= C (elements)
 * group_id [B*T] out, clip [B*G] out, scale [B*G] out, stats [B*G] out or NULL.
 * An empty token set gets clip = scale = eps_scale.
 * Every entry point that takes (B, T, C) refuses B > TDQ_MAX_IMAGES or B T > 2^30 with
 * TDQ_ERR_SHAPE (images index a 16-bit grid axis of several kernels).
 */
int tdq_calibrate_groups(const void* X, tdq_dtype dt, int32_t B, int32_t T, int32_t C,
                         int64_t ld_x, const tdq_params* p, int32_t* group_id, float* clip,
                         float* scale, tdq_group_stats* stats, void* workspace,
                         size_t workspace_bytes, void* stream);

/*
 * tdq_calibrate_groups for callers that cannot allocate or pass scratch memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * kernels, same results; the calibration scratch is a static device array of
 * TDQ_STATIC_SCRATCH_BYTES inside the library (every GPU the library runs on holds one
 * until the process ends).  The call allocates nothing and frees nothing; the first call
 * on a device looks the array's address up once.  Shapes whose
 * tdq_workspace_bytes(B, T, C, dt, p) exceeds TDQ_STATIC_SCRATCH_BYTES are refused with
 * TDQ_ERR_WORKSPACE (use tdq_calibrate_groups with a workspace of your own).  All calls
 * on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 * streams, or threads) race; calls ordered on one stream do not.
 * status [4] device out or NULL: word 0 the device status word (TDQ_DEV_*), words 1 and 2
 * the counts of token sets resolved by the per-set radix select (zr pass, base-radius
 * pass), word 3 zero.  Other arguments as tdq_calibrate_groups.
 */
#define TDQ_STATIC_SCRATCH_BYTES (16u << 20)
int tdq_calibrate_groups_static(const void* X, tdq_dtype dt, int32_t B, int32_t T, int32_t C,
                                int64_t ld_x, const tdq_params* p, int32_t* group_id, float* clip,
                                float* scale, tdq_group_stats* stats, uint32_t* status,
                                void* stream);

/*
 * Quantize + pack (Eqs. clipx, dequant): for row t of image b with j = gid,
 *   q = clamp(rint(clip(x, -c[b,j], c[b,j]) / Delta[b,j]), -8, 7)
 * with a correctly rounded binary32 quotient and ties-to-even rounding, written as
 * packed nibbles.  Qx [B*T, ld_q] bytes, ld_q >= ceil(C/2); bytes past ceil(C/2)
 * of a row are not written.
 */
int tdq_quantize_act(const void* X, tdq_dtype dt, int32_t B, int32_t T, int32_t C, int64_t ld_x,
                     const tdq_params* p, const int32_t* group_id, const float* clip,
                     const float* scale, uint8_t* Qx, int64_t ld_q, void* stream);

/*
 * Range disparity of Eq. (range_disparity), per image:
 *   D[b] = max |x| / median_t median_c |x|,
 * medians taken as the ceil(n/2)-th smallest value (the paper's rank rule k = ceil(p n) at
 * p = 1/2; the paper does not say which median it means for an even count), found exactly.
 * D is +Inf where the denominator is 0.  X [B*T, ld_x]; token_median, token_max [B*T] out
 * (the per-token median and maximum of |x|, also scratch of the call); disparity,
 * max_abs [B] out.
 */
int tdq_range_disparity(const void* X, tdq_dtype dt, int32_t B, int32_t T, int32_t C, int64_t ld_x,
                        float* token_median, float* token_max, float* disparity, float* max_abs,
                        void* stream);

/*
 * Convolutional feature maps as tokens (Supp. implementation details: the dynamic path
 * maps X[B, C, H, W] to X'[B, HW, C] and applies DSTG + DCRP along the channels).
 * Exact re-layout, element (b, c, t) of X -> row b*T + t, column c of Xt, T = H*W; every
 * token-major entry point then applies to Xt.  The paper restores the 4-D layout after its
 * quantize-dequantize; here the codes feed the contraction (a 1 x 1 convolution is
 * tdq_w4a4_linear over the channels), so nothing is restored.
 *
 * X: element (b, c, t) at X[b*ld_b + c*ld_c + t], ld_c >= T, ld_b >= (C-1)*ld_c + T.
 * Xt [B*T, ld_xt] out, ld_xt >= C; must not overlap X.  B <= 65535.
 */
int tdq_tokenize_chw(const void* X, tdq_dtype dt, int32_t B, int32_t C, int32_t T, int64_t ld_c,
                     int64_t ld_b, void* Xt, int64_t ld_xt, void* stream);

/*
 * tdq_calibrate_groups for a convolutional feature map (layout of tdq_tokenize_chw): the
 * statistics sweep reads the map in place and writes the token-major copy Xt [B*T, ld_xt]
 * as it goes; the rank select then runs on Xt, and so does tdq_quantize_act afterwards
 * (pass it Xt).  Outputs as tdq_calibrate_groups on the tokenized map.  B <= 65535.
 */
int tdq_calibrate_groups_chw(const void* X, tdq_dtype dt, int32_t B, int32_t C, int32_t T,
                             int64_t ld_c, int64_t ld_b, const tdq_params* p, void* Xt,
                             int64_t ld_xt, int32_t* group_id, float* clip, float* scale,
                             tdq_group_stats* stats, void* workspace, size_t workspace_bytes,
                             void* stream);

/*
 * The paper's own granularity (Sec. 4.2, Eq. direct_sum; Supp. Algorithm 1, steps 1-9) in
 * one sweep of X: the channel axis of every token is zero-padded to KB = ceil(C / 32)
 * blocks of g = TDQ_BLOCK channels and every (token, block) is a group of its own:
 *   c_base = max |x| of the block (or the ceil(32 p)-th smallest for base_pct = p),
 *   sigma  = population std of the block's 32 values + eps_std,
 *   thr    = the ceil(32 zr)-th smallest |x| of the block,
 *   c, Delta by Eq. (dcrp) and the eps floors, codes by Eqs. (clipx, dequant)
 * with the arithmetic of tdq_calibrate_groups / tdq_quantize_act; the padding zeros count
 * as values of the last block, as in Algorithm 1, and get no code.  p->chan_group must be
 * TDQ_BLOCK; n_groups is ignored.  X must be finite (not checked here).
 *
 * X [B*T, ld_x] of dt.  Qx [B*T, ld_q] bytes out, ld_q >= ceil(C/2), bytes past
 * ceil(C/2) of a row are not written.  block_scale [B*T, ld_s] out (Delta), block_clip
 * [B*T, ld_s] out or NULL (c), ld_s >= KB in floats.  B*T*KB < 2^31.
 */
int tdq_quantize_act_blocks(const void* X, tdq_dtype dt, int32_t B, int32_t T, int32_t C,
                            int64_t ld_x, const tdq_params* p, uint8_t* Qx, int64_t ld_q,
                            float* block_scale, float* block_clip, int64_t ld_s, void* stream);

/*
 * tdq_quantize_act_blocks reading a convolutional feature map directly (the paper's 4-D
 * branch fused into the sweep): X in the layout of tdq_tokenize_chw (element (b, c, t) at
 * X[b*ld_b + c*ld_c + t]); a group is the block of 32 channels of one pixel.  Outputs as
 * from tdq_quantize_act_blocks on the tokenized map, bit for bit: Qx [B*T, ld_q],
 * block_scale / block_clip [B*T, ld_s], row b*T + t.  B <= 65535.
 */
int tdq_quantize_act_blocks_chw(const void* X, tdq_dtype dt, int32_t B, int32_t C, int32_t T,
                                int64_t ld_c, int64_t ld_b, const tdq_params* p, uint8_t* Qx,
                                int64_t ld_q, float* block_scale, float* block_clip, int64_t ld_s,
                                void* stream);

/*
 * tdq_calibrate_groups followed by tdq_quantize_act in ONE launch, for shapes where launch
 * latency rather than bandwidth sets the time (up to a few hundred kilobytes per image;
 * it is correct for any size, one workgroup per image).  Same definitions and outputs:
 * group_id, clip, scale, stats (or NULL) as from tdq_calibrate_groups, Qx as from
 * tdq_quantize_act with those radii.  The rank of every set is found by a radix select
 * on LDS histograms (exact).  n_groups <= TDQ_FUSED_MAX_GROUPS, else
 * TDQ_ERR_UNSUPPORTED.  image_flags [B] out or NULL: TDQ_DEV_NONFINITE for an image that
 * holds an Inf or NaN (the workspace's status word is not written).  workspace as for
 * tdq_calibrate_groups (tdq_workspace_bytes).
 */
int tdq_calibrate_quantize_fused(const void* X, tdq_dtype dt, int32_t B, int32_t T, int32_t C,
                                 int64_t ld_x, const tdq_params* p, int32_t* group_id, float* clip,
                                 float* scale, tdq_group_stats* stats, uint32_t* image_flags,
                                 uint8_t* Qx, int64_t ld_q, void* workspace, size_t workspace_bytes,
                                 void* stream);

/*
 * Diagnostics of the paper's Sec. 3.1 (Preliminaries) per (image, token set), as exact element counts
 * for the radii and steps given: zero_count = elements whose code is 0 (zero-bin mass
 * rho_0 = zero_count / n, Eq. rho0_def; the code is computed exactly as
 * tdq_quantize_act computes it), clipped_count = elements with |x| > c.  The
 * step-to-dispersion ratio eta = Delta / sigma (Eq. cg_Delta_eta) follows from
 * tdq_group_stats.  One sweep of X.  zero_count, clipped_count [B*G] out, 8-byte
 * aligned; they need not be cleared.
 */
int tdq_group_diagnostics(const void* X, tdq_dtype dt, int32_t B, int32_t T, int32_t C, int64_t ld_x,
                          const tdq_params* p, const int32_t* group_id, const float* clip,
                          const float* scale, uint64_t* zero_count, uint64_t* clipped_count,
                          void* stream);

/*
 * W4A4 contraction with the dequantizing epilogue (Supp. Algorithm 1, step 10,
 * written on the integer codes):
 *   acc[m, n] = sum_i Qx[m, i] * Qw[n, i]                      (int32, exact)
 *   Y[m, n]   = (float(acc) * Delta[b(m)*G + gid[m]]) * w_scale[n] (+ bias[n])
 * each product rounded to binary32, no fused multiply-add.
 *
 * Qx [B*T, ld_q], Qw [N, ld_w] packed codes; both pointers 16-byte aligned and
 * ld_q, ld_w multiples of 16 with ld >= 16*ceil(K/32) (rows are read in 16-byte
 * pieces; bytes past ceil(K/2) are ignored).  Y [B*T, ld_y] of y_dt (fp32 or fp16).
 * acc_dump [B*T, N] int32 or NULL.  bias [N] or NULL.  group_id may be NULL when
 * G == 1.  K <= TDQ_MAX_K, else TDQ_ERR_SHAPE.
 */
int tdq_w4a4_linear(const uint8_t* Qx, int64_t ld_q, const int32_t* group_id, const float* scale,
                    int32_t B, int32_t T, int32_t K, int32_t N, int32_t G, const uint8_t* Qw,
                    int64_t ld_w, const float* w_scale, const float* bias, void* Y,
                    tdq_dtype y_dt, int64_t ld_y, int32_t* acc_dump, void* stream);

/*
 * The linear of Supp. Algorithm 1, step 10, on the codes of tdq_quantize_act_blocks:
 *   acc_kb[m, n] = sum over the 32 codes i of block kb of Qx[m, i] * Qw[n, i]   (exact)
 *   f[m, n]      = sum_kb float(acc_kb[m, n]) * Delta[m, kb]
 *   Y[m, n]      = f[m, n] * w_scale[n] (+ bias[n])
 * f is accumulated in binary32 with one fused multiply-add per block, kb ascending, so
 * the result is repeatable bit for bit and differs from the exact sum by at most
 * (KB + 2) 2^-24 sum_kb |acc_kb Delta| w_scale.
 *
 * Qx [M, ld_q], Qw [N, ld_w] packed codes with the alignment rules of tdq_w4a4_linear;
 * block_scale [M, ld_s] floats, ld_s >= KB = ceil(K / 32); Y [M, ld_y] of y_dt;
 * bias [N] or NULL.
 */
int tdq_w4a4_linear_blocks(const uint8_t* Qx, int64_t ld_q, const float* block_scale, int64_t ld_s,
                           int64_t M, int32_t K, int32_t N, const uint8_t* Qw, int64_t ld_w,
                           const float* w_scale, const float* bias, void* Y, tdq_dtype y_dt,
                           int64_t ld_y, void* stream);

/*
 * The same contraction on gfx950's 6-bit matrix format.  All sixteen int4 codes are exact
 * in bf6 (e3m2), integer sums below 2^24 are exact in the binary32 accumulator, and the
 * 6-bit matrix instruction runs at twice the int8 instruction's rate with no nibble
 * expansion: same acc, same Y, bit for bit, as tdq_w4a4_linear.
 *
 * Operands are "f6 fragments" (tdq_f6_bytes bytes, 16-byte aligned): rows in blocks of 32,
 * K zero-padded to KB = 2 ceil(K/128) blocks of 64; block (rb, kb) is the 1536 bytes at
 * (rb KB + kb) 1536 and holds, for lane l = row % 32 + 32 ((k % 64) / 32), 24 bytes with
 * code k % 32 as a bf6 pattern in bits [6 (k % 32), +6).  tdq_pack_codes_f6 converts packed
 * nibbles [rows, ld] (bytes) to fragments; tdq_quantize_act_f6 writes them directly.
 */
size_t tdq_f6_bytes(int64_t rows, int32_t K);
/* tdq_quantize_act writing f6 fragments: Qx6 holds tdq_f6_bytes(B*T, C) bytes, all written
 * (rows and codes of the padding are zero). */
int tdq_quantize_act_f6(const void* X, tdq_dtype dt, int32_t B, int32_t T, int32_t C, int64_t ld_x,
                        const tdq_params* p, const int32_t* group_id, const float* clip,
                        const float* scale, uint8_t* Qx6, void* stream);
int tdq_pack_codes_f6(const uint8_t* Q, int64_t ld, int64_t rows, int32_t K, uint8_t* F, void* stream);
int tdq_w4a4_linear_f6(const uint8_t* Qx6, const int32_t* group_id, const float* scale, int32_t B,
                       int32_t T, int32_t K, int32_t N, int32_t G, const uint8_t* Qw6,
                       const float* w_scale, const float* bias, void* Y, tdq_dtype y_dt, int64_t ld_y,
                       int32_t* acc_dump, void* stream);

/*
 * tdq_quantize_act_blocks writing f6 fragments (the operand of tdq_w4a4_linear_blocks_f6)
 * instead of packed nibbles: the same codes, steps and radii.  Qx6 holds
 * tdq_f6_bytes(B*T, C) bytes (device, 16-byte aligned), all written (rows and codes of
 * the padding are zero); the other arguments as in tdq_quantize_act_blocks.
 */
int tdq_quantize_act_blocks_f6(const void* X, tdq_dtype dt, int32_t B, int32_t T, int32_t C,
                               int64_t ld_x, const tdq_params* p, uint8_t* Qx6, float* block_scale,
                               float* block_clip, int64_t ld_s, void* stream);

/*
 * tdq_w4a4_linear_blocks on f6-fragment operands: same definition, same bits of Y.  The
 * 6-bit instruction delivers each block's sum as a float, so the per-block rescale costs
 * 16 instead of 38 vector instructions per matrix instruction.  Qx6 / Qw6: f6 fragments
 * of the [M, K] / [N, K] codes (device, 16-byte aligned); block_scale [M, ld_s] floats
 * (device), ld_s >= ceil(K / 32) and <= 2^22; w_scale [N], bias [N] or NULL; Y [M, ld_y]
 * binary32 or binary16.  Nothing is allocated; asynchronous on `stream`.
 * Errors: TDQ_ERR_NULL / _DTYPE / _SHAPE / _ALIGN / _HIP.
 */
int tdq_w4a4_linear_blocks_f6(const uint8_t* Qx6, const float* block_scale, int64_t ld_s, int64_t M,
                              int32_t K, int32_t N, const uint8_t* Qw6, const float* w_scale,
                              const float* bias, void* Y, tdq_dtype y_dt, int64_t ld_y, void* stream);

/*
 * Measurement probes (not part of the method): kernels of known traffic or known
 * arithmetic, for a benchmark that wants to measure on the device, in the same run, what
 * the memory system and the execution units sustain beside the published peaks.  One
 * launch per call, asynchronous; buf is device memory, 16-byte aligned, owned by the caller.
 *   TDQ_PROBE_READ        reads bytes - 4096 bytes of buf, 16 per thread (bytes a multiple
 *                         of 4096)
 *   TDQ_PROBE_COPY        copies the first half of buf to the second (bytes a multiple of
 *                         8192): bytes / 2 read and bytes / 2 written
 *   TDQ_PROBE_MFMA_I8     grid workgroups of 4 wavefronts, each issuing iters x 16
 *                         v_mfma_i32_32x32x32_i8 (65536 integer operations each) on four A
 *                         and four B operands taken from buf (accumulator (i, j) += A[i] B[j]
 *                         as in the contraction; the contents of buf choose the data: zeros,
 *                         random bytes, codes times 16); bytes >= 32768 grid + 4096
 *   TDQ_PROBE_FMA_1WAVE,  grid workgroups of 256 / 512 / 1024 threads (1 / 2 / 4 wavefronts
 *   _2WAVES, _4WAVES      per SIMD of a CU), every wavefront issuing iters x 16 independent
 *                         v_fma_f32; buf holds 128 floats (multiplier, addend per lane),
 *                         bytes >= 8192
 * Returns TDQ_OK or TDQ_ERR_NULL / ALIGN / SHAPE / PARAM / HIP.
 */
enum { TDQ_PROBE_READ = 0, TDQ_PROBE_COPY = 1, TDQ_PROBE_MFMA_I8 = 2, TDQ_PROBE_FMA_1WAVE = 3,
       TDQ_PROBE_FMA_2WAVES = 4, TDQ_PROBE_FMA_4WAVES = 5 };
int tdq_probe(int32_t kind, void* buf, size_t bytes, int32_t iters, int32_t grid, void* stream);

/*
 * Static symmetric per-output-channel weight quantization (Eq. weight_quant),
 * done once offline:  s_o = max(max_i |W_oi|, 1e-8) / 7,
 * Qw = clamp(rint(W / s_o), -8, 7) packed.  W [N, K] fp32 (device),
 * Qw [N, ld_w] bytes (bytes from ceil(K/2) to ld_w are zeroed), w_scale [N].
 */
int tdq_quantize_weight(const float* W, int32_t N, int32_t K, int64_t ld_w_in, uint8_t* Qw,
                        int64_t ld_w, float* w_scale, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TDQ_H */
