// Device-side helpers shared by the activation kernels of libtdq: element access
// for the two input types, DPP reductions over groups of lanes, and the DCRP
// projection that turns a group's statistics into its clip radius and step.
#pragma once

#include "tdq_internal.hpp"

namespace tdq {

// ---------------------------------------------------------------------------
// element access
// ---------------------------------------------------------------------------
typedef unsigned short u16;
typedef unsigned int u32;
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef unsigned short us2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float h2f(u32 bits16) {
  return (float)__builtin_bit_cast(_Float16, (u16)bits16);
}

template <typename T>
struct Elem;
template <>
struct Elem<u16> {                 // fp16 stored as raw bits
  static constexpr int V = 8;      // elements per 16-byte load
  static constexpr u32 kNonFinite = 0x7C00u;
  __device__ static __forceinline__ u32 key(u16 x) { return x & 0x7FFFu; }
  __device__ static __forceinline__ float val(u16 x) { return h2f(x); }
  __device__ static __forceinline__ float key_to_float(u32 k) { return h2f(k); }
  __device__ static __forceinline__ void unpack(const uint4& q, u16 out[8]) {
    out[0] = q.x & 0xFFFF; out[1] = q.x >> 16; out[2] = q.y & 0xFFFF; out[3] = q.y >> 16;
    out[4] = q.z & 0xFFFF; out[5] = q.z >> 16; out[6] = q.w & 0xFFFF; out[7] = q.w >> 16;
  }
};
template <>
struct Elem<float> {
  static constexpr int V = 4;
  static constexpr u32 kNonFinite = 0x7F800000u;
  __device__ static __forceinline__ u32 key(float x) { return __float_as_uint(x) & 0x7FFFFFFFu; }
  __device__ static __forceinline__ float val(float x) { return x; }
  __device__ static __forceinline__ float key_to_float(u32 k) { return __uint_as_float(k); }
  __device__ static __forceinline__ void unpack(const uint4& q, float out[4]) {
    out[0] = __uint_as_float(q.x); out[1] = __uint_as_float(q.y);
    out[2] = __uint_as_float(q.z); out[3] = __uint_as_float(q.w);
  }
};

// Rows are shared out to groups of L adjacent lanes (L a power of two <= 64), so a
// 64-wide wavefront covers 64/L rows; each lane reads 16-byte pieces of its row.
inline int lanes_per_row(int C, int V) {
  int nvec = (C + V - 1) / V;
  int L = 1;
  while (L < nvec && L < 64) L <<= 1;
  return L;
}

// Reductions over groups of L adjacent lanes (L a power of two <= 64) with DPP
// row shifts and row broadcasts, i.e. at vector-ALU speed instead of one LDS round
// trip per step.  The result is valid in the LAST lane of every group
// (lane % L == L - 1); the other lanes hold partial windows.
//   steps 1, 2, 4, 8: row_shr inside rows of 16 lanes (zero shifted in),
//   16: row_bcast15 into rows 1 and 3,  32: row_bcast31 into rows 2 and 3.
#define TDQ_DPP_ROW_SHR(n) (0x110 + (n))
#define TDQ_DPP_ROW_BCAST15 0x142
#define TDQ_DPP_ROW_BCAST31 0x143

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ u32 dpp_u32(u32 v) {
  return (u32)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, true);
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_f64(double v) {
  const unsigned long long b = __builtin_bit_cast(unsigned long long, v);
  const u32 lo = dpp_u32<CTRL, ROW_MASK>((u32)b), hi = dpp_u32<CTRL, ROW_MASK>((u32)(b >> 32));
  return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
}

template <int L>
__device__ __forceinline__ double group_sum_f64(double v) {
  if (L > 1) v += dpp_f64<TDQ_DPP_ROW_SHR(1), 0xF>(v);
  if (L > 2) v += dpp_f64<TDQ_DPP_ROW_SHR(2), 0xF>(v);
  if (L > 4) v += dpp_f64<TDQ_DPP_ROW_SHR(4), 0xF>(v);
  if (L > 8) v += dpp_f64<TDQ_DPP_ROW_SHR(8), 0xF>(v);
  if (L > 16) v += dpp_f64<TDQ_DPP_ROW_BCAST15, 0xA>(v);
  if (L > 32) v += dpp_f64<TDQ_DPP_ROW_BCAST31, 0xC>(v);
  return v;
}
template <int L>
__device__ __forceinline__ u32 group_max_u32(u32 v) {
  u32 o;
  if (L > 1) { o = dpp_u32<TDQ_DPP_ROW_SHR(1), 0xF>(v); v = o > v ? o : v; }
  if (L > 2) { o = dpp_u32<TDQ_DPP_ROW_SHR(2), 0xF>(v); v = o > v ? o : v; }
  if (L > 4) { o = dpp_u32<TDQ_DPP_ROW_SHR(4), 0xF>(v); v = o > v ? o : v; }
  if (L > 8) { o = dpp_u32<TDQ_DPP_ROW_SHR(8), 0xF>(v); v = o > v ? o : v; }
  if (L > 16) { o = dpp_u32<TDQ_DPP_ROW_BCAST15, 0xA>(v); v = o > v ? o : v; }
  if (L > 32) { o = dpp_u32<TDQ_DPP_ROW_BCAST31, 0xC>(v); v = o > v ? o : v; }
  return v;
}

// xor-butterfly forms (every lane gets the result), used off the hot paths
template <int L, typename F>
__device__ __forceinline__ F xor_reduce_sum(F v) {
#pragma unroll
  for (int m = L >> 1; m > 0; m >>= 1) v += __shfl_xor(v, m, 64);
  return v;
}
template <int L>
__device__ __forceinline__ u32 xor_reduce_max(u32 v) {
#pragma unroll
  for (int m = L >> 1; m > 0; m >>= 1) {
    u32 o = (u32)__shfl_xor((int)v, m, 64);
    v = o > v ? o : v;
  }
  return v;
}

template <int L>
__device__ __forceinline__ u32 group_sum_u32(u32 v) {
  if (L > 1) v += dpp_u32<TDQ_DPP_ROW_SHR(1), 0xF>(v);
  if (L > 2) v += dpp_u32<TDQ_DPP_ROW_SHR(2), 0xF>(v);
  if (L > 4) v += dpp_u32<TDQ_DPP_ROW_SHR(4), 0xF>(v);
  if (L > 8) v += dpp_u32<TDQ_DPP_ROW_SHR(8), 0xF>(v);
  if (L > 16) v += dpp_u32<TDQ_DPP_ROW_BCAST15, 0xA>(v);
  if (L > 32) v += dpp_u32<TDQ_DPP_ROW_BCAST31, 0xC>(v);
  return v;
}

// ---------------------------------------------------------------------------
// Moments.  The dispersion of a set is the population standard deviation of all its
// elements (Sec. 4.2), and the bar on it is 1e-6 relative whatever the data's offset.
// A plain sum of squares loses (mean / sigma)^2 units of its last place when it is turned
// into a variance, so nothing here is summed about zero:
//   * a token's row is summed about a pivot P taken from the row itself (S1 = sum (x - P),
//     S2 = sum (x - P)^2) and leaves the sweep as (mean, M2) = (P + S1 / C, S2 - S1^2 / C),
//     M2 = sum (x - mean)^2;
//   * the tokens of a set are merged about the mean of the image's first token, P_b:
//     a token adds C (mean - P_b) and M2 + C (mean - P_b)^2 to the set's two sums.
// Both conversions are binary64 and lose (distance to the pivot / sigma)^2 units of 2^-53.
// ---------------------------------------------------------------------------
// inv_n = 1 / C (rounded once, by the caller: a binary64 division costs a wavefront about
// thirty instructions, as much as a quarter of a short row's sweep).
__device__ __forceinline__ void pivot_to_central(double P, double S1, double S2, double inv_n,
                                                 double& mean, double& m2) {
  const double t = S1 * inv_n;               // mean - P
  mean = P + t;
  const double v = S2 - S1 * t;
  m2 = v > 0.0 ? v : 0.0;
}

// True when a row summed about P should be summed again about its mean: the pivot lies
// more than sqrt(8) row standard deviations from the mean, so the binary32 partial sums
// of a binary16 row (3 * 2^-24 relative to sum (x - P)^2 each) could cost the row's M2
// more than 1e-6.  With off = S1^2 / C = C (mean - P)^2 the test off > 8 (S2 - off) is
// 9 S1^2 > 8 C S2.  False for NaN.
__device__ __forceinline__ bool pivot_is_far(double S1, double S2, int C) {
  return 9.0 * (S1 * S1) > (8.0 * (double)C) * S2;
}

// Pivot of a binary16 row: the median of its first three values (one outlier among
// them does not become the pivot).  `wide` = the row is 8-byte aligned and C >= 4.
__device__ __forceinline__ float row_pivot(const u16* __restrict__ xp, int C, bool wide) {
  u32 w0, w1;
  if (wide) {
    const uint2 pw = *reinterpret_cast<const uint2*>(xp);
    w0 = pw.x;
    w1 = pw.y;
  } else {
    const int i1 = C > 1 ? 1 : 0, i2 = C > 2 ? 2 : i1;
    w0 = (u32)xp[0] | ((u32)xp[i1] << 16);
    w1 = xp[i2];
  }
  return __builtin_amdgcn_fmed3f(h2f(w0 & 0xFFFFu), h2f(w0 >> 16), h2f(w1 & 0xFFFFu));
}
// Pivot of a binary32 row: its first value (the row is summed in binary64, where any
// value of the row is close enough).
__device__ __forceinline__ double row_pivot(const float* __restrict__ xp, int, bool) {
  return (double)xp[0];
}

// Partial sums of one token set over part of an image's tokens, taken about a pivot of the
// record's own: the mean of the first token that went into it.
struct SetAcc {
  double s1, s2;      // sum (x - piv), sum (x - piv)^2 over the elements of the record's tokens
  double piv;
  u32 cnt, kmax;      // tokens, largest range key
};

// a += b (cn = elements per token): b's sums are re-centred on a's pivot,
//   sum (x - Pa)^2 = sum (x - Pb)^2 + 2 d sum (x - Pb) + n d^2,  d = Pb - Pa.
// Tokens with one and the same mean add exact zeros, so a set of identical values (the
// all-zero tokens of a padded image, say) ends with a variance of exactly zero, as the
// two-pass definition gives it -- sums about a pivot from outside the set would leave a
// rounding residue of 1e-8 of the pivot's distance in sigma.
__device__ inline void setacc_add(SetAcc& a, const SetAcc& b, double cn) {
  if (b.cnt == 0) return;
  const u32 km = a.kmax > b.kmax ? a.kmax : b.kmax;
  if (a.cnt == 0) {
    a = b;
  } else {
    const double d = b.piv - a.piv, nb = (double)b.cnt * cn;
    a.s1 += b.s1 + nb * d;
    a.s2 += b.s2 + 2.0 * d * b.s1 + nb * d * d;
    a.cnt += b.cnt;
  }
  a.kmax = km;
}

// Merges the S partial records of set j of image b (in index order, so the result is
// bitwise repeatable) into the set's working record: n, c_base (DSTG base radius,
// Eq. DSTG_clip), sigma = population std + eps_std (Sec. 4.2; the sums are about a pivot,
// which the variance does not depend on), and the rank this pass looks for: k = ceil(zr n),
// or ceil(p n) in the base-radius pass.
__device__ inline GroupWork merge_partials(const SetAcc* __restrict__ part, int b, int j, int S,
                                           int G, int C, const Scalars& sc, int pass) {
  SetAcc m;
  m.s1 = 0.0; m.s2 = 0.0; m.piv = 0.0; m.cnt = 0; m.kmax = 0;
  for (int s = 0; s < S; ++s) setacc_add(m, part[((long long)b * S + s) * G + j], (double)C);
  const u32 cnt = m.cnt, cmax = m.kmax;
  const double S1 = m.s1, S2 = m.s2;
  GroupWork w;
  w.tokens = cnt;
  w.n = (long long)cnt * (long long)C;
  w.prefix = 0;
  w.c_base = __uint_as_float(cmax);
  if (cnt == 0) {
    w.k_rem = 0;
    w.sigma = 0.f;
  } else {
    const double n = (double)w.n;
    const double mu = S1 / n;
    double var = S2 / n - mu * mu;
    var = var > 0.0 ? var : 0.0;
    w.sigma = (float)(sqrt(var) + sc.eps_std);
    long long k = (long long)ceil((pass == kPassBase ? sc.base_pct : sc.zr) * n);   // binary64
    k = k < 1 ? 1 : (k > w.n ? w.n : k);
    w.k_rem = k;
  }
  return w;
}

// ---------------------------------------------------------------------------
// Token -> token set, and the per-set sums of one image (or of every S-th group of its
// token batches), by ALL threads of a workgroup of NW wavefronts:
//   key_t = bits(r_t); hi = max key; lo = max(min key, hi - 24 octaves);
//   gid_t = key_t <= lo ? 0 : (key_t - lo) * G / (hi - lo + 1)      (64-bit integers)
// wacc [NW][G], s_min / s_max [NW] and s_lohi [2] are LDS; on return (after a barrier)
// wacc holds every wavefront's per-set record and s_lohi = {lo, hi}.
// ---------------------------------------------------------------------------
__device__ __forceinline__ u32 wave_max_u32(u32 v) { return xor_reduce_max<64>(v); }
__device__ __forceinline__ u32 wave_min_u32(u32 v) {
#pragma unroll
  for (int m = 32; m > 0; m >>= 1) {
    u32 o = (u32)__shfl_xor((int)v, m, 64);
    v = o < v ? o : v;
  }
  return v;
}

__device__ inline void assign_tokens(const float* __restrict__ rb, const double* __restrict__ meanb,
                                     const double* __restrict__ m2b, int T, int C, int G,
                                     int* __restrict__ gb, SetAcc* wacc, u32* s_min, u32* s_max,
                                     u32* s_lohi, int sub, int S) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int NW = blockDim.x >> 6;
  for (int i = tid; i < NW * G; i += blockDim.x) {
    SetAcc z;
    z.s1 = 0.0; z.s2 = 0.0; z.piv = 0.0; z.cnt = 0; z.kmax = 0;
    wacc[i] = z;
  }
  u32 kmin = 0xFFFFFFFFu, kmax = 0;
  for (int t = tid; t < T; t += blockDim.x) {
    const u32 k = __float_as_uint(rb[t]);
    kmin = k < kmin ? k : kmin;
    kmax = k > kmax ? k : kmax;
  }
  kmin = wave_min_u32(kmin);
  kmax = wave_max_u32(kmax);
  if (lane == 0) { s_min[wave] = kmin; s_max[wave] = kmax; }
  __syncthreads();
  if (tid == 0) {
    u32 lo = 0xFFFFFFFFu, hi = 0;
    for (int w = 0; w < NW; ++w) {
      lo = s_min[w] < lo ? s_min[w] : lo;
      hi = s_max[w] > hi ? s_max[w] : hi;
    }
    const u32 span = (u32)kOctaveFloor << 23;
    const u32 floor_key = hi > span ? hi - span : 0u;
    s_lohi[0] = lo > floor_key ? lo : floor_key;
    s_lohi[1] = hi;
  }
  __syncthreads();
  const u32 lo = s_lohi[0], hi = s_lohi[1];
  const unsigned long long width = (unsigned long long)(hi - lo) + 1ull;
  const double cn = (double)C;

  // Wavefront w of workgroup `sub` owns the token batches sub NW + w, + S NW, ... (64
  // tokens each).  Inside a batch the tokens of one set are summed with a fixed tree, about
  // the mean of the first of them, and added to the wavefront's accumulator of that set
  // (setacc_add), sets in order of first appearance: every floating-point sum has a fixed
  // order, so the result is bitwise repeatable.
  SetAcc* mine = wacc + wave * G;
  const int n_batches = (T + 63) / 64;
  // the loads of the next batch are issued before the current one is reduced
  u32 nk = 0;
  double n1 = 0.0, n2 = 0.0;
  const int bt0 = sub * NW + wave, bstep = S * NW;
  if (bt0 < n_batches && bt0 * 64 + lane < T) {
    const int t = bt0 * 64 + lane;
    nk = __float_as_uint(rb[t]);
    n1 = meanb[t];
    n2 = m2b[t];
  }
  for (int bt = bt0; bt < n_batches; bt += bstep) {
    const int t = bt * 64 + lane;
    const bool live = t < T;
    const u32 k = nk;
    const double tmean = n1, tm2 = n2;
    {
      const int tn = t + bstep * 64;
      if (bt + bstep < n_batches && tn < T) {
        nk = __float_as_uint(rb[tn]);
        n1 = meanb[tn];
        n2 = m2b[tn];
      }
    }
    int g = -1;
    if (live) {
      g = 0;
      if (G > 1 && hi != lo && k > lo)
        g = (int)(((unsigned long long)(k - lo) * (unsigned long long)G) / width);
      gb[t] = g;
    }
    unsigned long long todo = __ballot(live);
    while (todo) {
      const int leader = __ffsll((long long)todo) - 1;
      const int gg = __builtin_amdgcn_readlane(g, leader);
      const bool sel = g == gg;
      const unsigned long long m = __ballot(sel);
      // pivot of this batch's part of the set: the mean of its first token (zero if that is
      // not finite: the image's results are then undefined anyway and its flag is raised)
      const unsigned long long mb = __builtin_bit_cast(unsigned long long, tmean);
      double piv = __builtin_bit_cast(
          double, (unsigned long long)(u32)__builtin_amdgcn_readlane((int)(u32)mb, leader) |
                      ((unsigned long long)(u32)__builtin_amdgcn_readlane((int)(u32)(mb >> 32), leader) << 32));
      piv = (piv - piv == 0.0) ? piv : 0.0;
      const double dm = tmean - piv;
      const double a1 = group_sum_f64<64>(sel ? cn * dm : 0.0);            // totals land in lane 63
      const double a2 = group_sum_f64<64>(sel ? tm2 + cn * dm * dm : 0.0);
      const u32 km = group_max_u32<64>(sel ? k : 0u);
      if (lane == 63) {
        SetAcc bsum;
        bsum.s1 = a1; bsum.s2 = a2; bsum.piv = piv; bsum.cnt = (u32)__popcll(m); bsum.kmax = km;
        if (bt == bt0) {                 // uniform: the wavefront's first batch finds its records empty
          mine[gg] = bsum;
        } else {
          SetAcc a = mine[gg];
          setacc_add(a, bsum, cn);
          mine[gg] = a;
        }
      }
      todo &= ~m;
    }
  }
  __syncthreads();
}

// Clears the radix-level histograms of set idx (threads tid, tid + nthreads, ...).
__device__ inline void clear_level_hists(u32* __restrict__ hist, const LevelPlan& lp,
                                         long long groups_total, long long idx, int tid,
                                         int nthreads) {
  size_t off = 0;
  for (int l = 0; l < lp.n_levels; ++l) {
    const size_t nb = (size_t)1 << lp.bits[l];
    u32* h = hist + off + (size_t)idx * nb;
    for (size_t i = tid; i < nb; i += nthreads) h[i] = 0;
    off += (size_t)groups_total * nb;
  }
}

// DCRP projection of one (image, token set), in binary32 (Eq. dcrp with the eps
// floors of the supplementary numerical conventions): key is the magnitude bit
// pattern of the k-th smallest |x| of the set.  Called by one lane per set.
__device__ inline void project_store(int idx, const GroupWork& w, u32 key, bool is_f16,
                                     const Scalars& sc, float* __restrict__ clip,
                                     float* __restrict__ scale,
                                     tdq_group_stats* __restrict__ stats) {
  float thr = 0.f, c_tau = 0.f, c_zr = 0.f, c, d;
  u32 bind = TDQ_BIND_EMPTY;
  long long kk = 0;
  if (w.tokens == 0) {
    c = sc.eps_scale;
    d = sc.eps_scale;
  } else {
    thr = is_f16 ? h2f(key) : __uint_as_float(key);
    c_tau = sc.qmax_tau * w.sigma;            // q_max * tau * sigma
    c_zr = sc.two_qmax * thr;                 // 2 * q_max * Q_zr(|x|)
    c = w.c_base;
    bind = TDQ_BIND_BASE;
    if ((sc.flags & TDQ_FLAG_C1) && c_tau < c) { c = c_tau; bind = TDQ_BIND_C1; }
    if ((sc.flags & TDQ_FLAG_C2) && c_zr < c) { c = c_zr; bind = TDQ_BIND_C2; }
    if (!(c > sc.eps_scale)) { c = sc.eps_scale; bind = TDQ_BIND_EPS; }
    d = c / sc.qmax;
    d = d > sc.eps_scale ? d : sc.eps_scale;
    // original rank (k_rem has been consumed): recompute for the record
    const double n = (double)w.n;
    kk = (long long)ceil(sc.zr * n);
    kk = kk < 1 ? 1 : (kk > w.n ? w.n : kk);
  }
  clip[idx] = c;
  scale[idx] = d;
  if (stats) {
    tdq_group_stats s;
    s.n = w.n; s.k = kk; s.c_base = w.c_base; s.sigma = w.sigma; s.thr = thr;
    s.c_tau = c_tau; s.c_zr = c_zr; s.clip = c; s.scale = d; s.bind = bind;
    stats[idx] = s;
  }
}

// ---------------------------------------------------------------------------
// Quantization of one element.  q = clamp(rint(clip(x, +-c) / Delta), -8, 7).
// The quotient is the correctly rounded binary32 one, obtained per element as
//   y0 = x~ * r,  e = fma(-y0, Delta, x~),  y = fma(e, r, y0),   r = RN(1 / Delta)
// (one reciprocal per row instead of one division per element).  Adding
// 1.5 * 2^23 rounds y to an integer with ties to even and leaves its two's
// complement in the low mantissa bits.
// ---------------------------------------------------------------------------
__device__ __forceinline__ u32 quant_nibble(float x, float c, float d, float rcp) {
  const float xt = fminf(fmaxf(x, -c), c);
  const float y0 = xt * rcp;
  const float e = __builtin_fmaf(-y0, d, xt);
  float y = __builtin_fmaf(e, rcp, y0);
  y = fminf(fmaxf(y, (float)kQMin), (float)kQMax);
  const float m = y + 12582912.0f;
  return __float_as_uint(m) & 0xFu;
}

// Rounded quotient of one element as a float bit pattern whose low 4 bits are the
// two's-complement code (see above).  CLAMP adds the clamp to [-8, 7], needed only
// when the radii are not a projection's (c > 7.25 * Delta).
template <bool CLAMP>
__device__ __forceinline__ u32 quant_bits(float x, float c, float d, float rcp) {
  const float xt = __builtin_amdgcn_fmed3f(x, -c, c);
  const float y0 = xt * rcp;
  const float e = __builtin_fmaf(-y0, d, xt);
  float y = __builtin_fmaf(e, rcp, y0);
  if (CLAMP) y = __builtin_amdgcn_fmed3f(y, (float)kQMin, (float)kQMax);
  return __float_as_uint(y + 12582912.0f);
}

// Eight fp16 elements (one 16-byte load) -> eight packed codes.  The low bytes of
// the eight results are gathered with byte permutes into a word of the even and a
// word of the odd elements, which are then merged nibble-wise.
template <bool CLAMP>
__device__ __forceinline__ u32 quant8_f16(const uint4& q, float c, float d, float rcp) {
  const u32 w[4] = {q.x, q.y, q.z, q.w};
  u32 m[8];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const h2 h = __builtin_bit_cast(h2, w[j]);
    m[2 * j] = quant_bits<CLAMP>((float)h[0], c, d, rcp);
    m[2 * j + 1] = quant_bits<CLAMP>((float)h[1], c, d, rcp);
  }
  // v_perm_b32(s0, s1, sel): selector bytes 0-3 pick bytes of s1, 4-7 bytes of s0, 0x0c is zero
  const u32 e02 = __builtin_amdgcn_perm(m[2], m[0], 0x0c0c0400u);   // [m0.b0, m2.b0, 0, 0]
  const u32 e46 = __builtin_amdgcn_perm(m[6], m[4], 0x04000c0cu);   // [0, 0, m4.b0, m6.b0]
  const u32 o13 = __builtin_amdgcn_perm(m[3], m[1], 0x0c0c0400u);
  const u32 o57 = __builtin_amdgcn_perm(m[7], m[5], 0x04000c0cu);
  const u32 ev = e02 | e46, od = (o13 | o57) << 4;
  return (ev & 0x0F0F0F0Fu) | (od & 0xF0F0F0F0u);
}

}  // namespace tdq
