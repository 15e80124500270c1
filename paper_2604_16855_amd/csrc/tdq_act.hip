// Activation side of the W4A4 path: per-token statistics, token-set assignment,
// exact rank select of the zr quantile with LDS histograms, DCRP projection,
// quantize + pack, and the offline weight quantizer.  gfx950 only.
//
// Paper passages: Sec. 4.2 (DSTG: base radius, group dispersion, Eqs. DSTG_clip,
// clipx, dequant), Sec. 4.3 (DCRP: Eqs. tau_constraint, zr_constraint, dcrp),
// Supp. "Quantile Implementation" (rank k = ceil(p n)), Supp. numerical
// conventions (eps values, ties-to-even rounding), Eq. weight_quant.
#include "tdq_internal.hpp"

namespace tdq {

// ---------------------------------------------------------------------------
// element access
// ---------------------------------------------------------------------------
typedef unsigned short u16;
typedef unsigned int u32;

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
static int lanes_per_row(int C, int V) {
  int nvec = (C + V - 1) / V;
  int L = 1;
  while (L < nvec && L < 64) L <<= 1;
  return L;
}

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

// ---------------------------------------------------------------------------
// K_a: per-token range and moments (one sweep of X)
//   r_t = max_c |x|  (exact: integer max of the magnitude bit patterns)
//   s1_t = sum x, s2_t = sum x^2 in binary64.  For fp16 input each lane first adds
//   its 8 values / 8 squares (a square of an fp16 value is exact in binary32) in
//   binary32 and then accumulates in binary64.
// ---------------------------------------------------------------------------
template <typename T, int L>
__global__ __launch_bounds__(256) void k_token_stats(const T* __restrict__ X, long long ld, int M,
                                                     int C, int vec_ok, float* __restrict__ r,
                                                     double* __restrict__ s1,
                                                     double* __restrict__ s2) {
  constexpr int V = Elem<T>::V;
  const long long gt = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long row = gt / L;
  const int lr = (int)(gt % L);
  const bool valid = row < M;
  const T* xp = X + (valid ? row : (long long)(M - 1)) * ld;
  u32 kmax = 0;
  double a1 = 0.0, a2 = 0.0;
  const int nvec = vec_ok ? C / V : 0;
#pragma unroll 4
  for (int v = lr; v < nvec; v += L) {
    const uint4 q = *reinterpret_cast<const uint4*>(xp + (long long)v * V);
    T e[V];
    Elem<T>::unpack(q, e);
    if constexpr (sizeof(T) == 2) {
      float p1 = 0.f, p2 = 0.f;
#pragma unroll
      for (int i = 0; i < V; ++i) {
        const float f = Elem<T>::val(e[i]);
        const u32 k = Elem<T>::key(e[i]);
        kmax = k > kmax ? k : kmax;
        p1 += f;
        p2 += f * f;
      }
      a1 += (double)p1;
      a2 += (double)p2;
    } else {
#pragma unroll
      for (int i = 0; i < V; ++i) {
        const double f = (double)Elem<T>::val(e[i]);
        const u32 k = Elem<T>::key(e[i]);
        kmax = k > kmax ? k : kmax;
        a1 += f;
        a2 += f * f;
      }
    }
  }
  for (int c = nvec * V + lr; c < C; c += L) {   // ragged tail / unaligned rows
    const T x = xp[c];
    const double f = (double)Elem<T>::val(x);
    const u32 k = Elem<T>::key(x);
    kmax = k > kmax ? k : kmax;
    a1 += f;
    a2 += f * f;
  }
  kmax = xor_reduce_max<L>(kmax);
  a1 = xor_reduce_sum<L>(a1);
  a2 = xor_reduce_sum<L>(a2);
  if (lr == 0 && valid) {
    r[row] = Elem<T>::key_to_float(kmax);
    s1[row] = a1;
    s2[row] = a2;
  }
}

template <typename T>
static hipError_t token_stats_t(const T* X, int M, int C, long long ld, float* r, double* s1,
                                double* s2, hipStream_t st) {
  constexpr int V = Elem<T>::V;
  const int vec_ok = ((reinterpret_cast<uintptr_t>(X) & 15) == 0 && ld % V == 0) ? 1 : 0;
  const int L = lanes_per_row(C, V);
  const long long threads = (long long)M * L;
  const unsigned grid = (unsigned)((threads + 255) / 256);
#define TDQ_TS(LL)                                                                       \
  case LL:                                                                               \
    hipLaunchKernelGGL((k_token_stats<T, LL>), dim3(grid), dim3(256), 0, st, X, ld, M, C, \
                       vec_ok, r, s1, s2);                                               \
    break;
  switch (L) {
    TDQ_TS(1) TDQ_TS(2) TDQ_TS(4) TDQ_TS(8) TDQ_TS(16) TDQ_TS(32) TDQ_TS(64)
  }
#undef TDQ_TS
  return hipGetLastError();
}

hipError_t launch_token_stats(const void* X, tdq_dtype dt, int M, int C, long long ld, float* r,
                              double* s1, double* s2, hipStream_t st) {
  if (dt == TDQ_F16)
    return token_stats_t<u16>(static_cast<const u16*>(X), M, C, ld, r, s1, s2, st);
  return token_stats_t<float>(static_cast<const float*>(X), M, C, ld, r, s1, s2, st);
}

// ---------------------------------------------------------------------------
// K_assign: one workgroup per image.
//   key_t = bits(r_t); hi = max key; lo = max(min key, hi - 24 octaves);
//   gid_t = key_t <= lo ? 0 : (key_t - lo) * G / (hi - lo + 1)      (64-bit integers)
// then per token set: token count, c_base = max r_t, and the merged moments ->
// sigma = sqrt(S2/n - (S1/n)^2) + eps_std in binary64, rank k = ceil(zr n).
// Also clears this image's histogram slices and records whether the image holds
// a non-finite value (its largest range key is Inf/NaN).
// ---------------------------------------------------------------------------
constexpr int kAssignThreads = 1024;

__device__ __forceinline__ u32 wave_max_u32(u32 v) { return xor_reduce_max<64>(v); }
__device__ __forceinline__ u32 wave_min_u32(u32 v) {
#pragma unroll
  for (int m = 32; m > 0; m >>= 1) {
    u32 o = (u32)__shfl_xor((int)v, m, 64);
    v = o < v ? o : v;
  }
  return v;
}

__global__ __launch_bounds__(kAssignThreads) void k_assign(
    const float* __restrict__ r, const double* __restrict__ s1, const double* __restrict__ s2,
    int T, int C, int G, Scalars sc, int* __restrict__ gid, GroupWork* __restrict__ grp,
    u32* __restrict__ hist, LevelPlan lp, long long groups_total, u32* __restrict__ img_flag) {
  __shared__ u32 s_min[kAssignThreads / 64], s_max[kAssignThreads / 64];
  __shared__ u32 s_lo, s_hi;
  const int b = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int NW = kAssignThreads / 64;
  const float* rb = r + (long long)b * T;
  int* gb = gid + (long long)b * T;

  u32 kmin = 0xFFFFFFFFu, kmax = 0;
  for (int t = tid; t < T; t += kAssignThreads) {
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
    s_lo = lo > floor_key ? lo : floor_key;
    s_hi = hi;
    img_flag[b] = hi >= 0x7F800000u ? TDQ_DEV_NONFINITE : 0u;
  }
  __syncthreads();
  const u32 lo = s_lo, hi = s_hi;
  const unsigned long long width = (unsigned long long)(hi - lo) + 1ull;
  for (int t = tid; t < T; t += kAssignThreads) {
    const u32 k = __float_as_uint(rb[t]);
    int g = 0;
    if (G > 1 && hi != lo && k > lo)
      g = (int)(((unsigned long long)(k - lo) * (unsigned long long)G) / width);
    gb[t] = g;
  }
  __syncthreads();   // gid of this image visible to the whole workgroup (global, same block)

  // one wavefront per token set, fixed lane-strided order + xor tree: deterministic
  for (int g = wave; g < G; g += NW) {
    u32 cnt = 0, cmax = 0;
    double S1 = 0.0, S2 = 0.0;
    for (int t = lane; t < T; t += 64) {
      if (gb[t] == g) {
        const u32 k = __float_as_uint(rb[t]);
        cnt += 1;
        cmax = k > cmax ? k : cmax;
        S1 += s1[(long long)b * T + t];
        S2 += s2[(long long)b * T + t];
      }
    }
    cnt = (u32)xor_reduce_sum<64>((int)cnt);
    cmax = wave_max_u32(cmax);
    S1 = xor_reduce_sum<64>(S1);
    S2 = xor_reduce_sum<64>(S2);
    if (lane == 0) {
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
        long long k = (long long)ceil(sc.zr * n);   // binary64 product, then ceil
        k = k < 1 ? 1 : (k > w.n ? w.n : k);
        w.k_rem = k;
      }
      grp[(long long)b * G + g] = w;
    }
  }
  // clear this image's slice of every level's histogram
  size_t off = 0;
  for (int l = 0; l < lp.n_levels; ++l) {
    const size_t nb = (size_t)1 << lp.bits[l];
    u32* h = hist + off + (size_t)b * G * nb;
    for (size_t i = tid; i < (size_t)G * nb; i += kAssignThreads) h[i] = 0;
    off += (size_t)groups_total * nb;
  }
}

hipError_t launch_assign(const float* r, const double* s1, const double* s2, int B, int T, int C,
                         int G, const Scalars& sc, int* gid, GroupWork* grp, unsigned* hist,
                         unsigned* img_flag, const LevelPlan& lp, hipStream_t st) {
  hipLaunchKernelGGL(k_assign, dim3(B), dim3(kAssignThreads), 0, st, r, s1, s2, T, C, G, sc, gid,
                     grp, hist, lp, (long long)B * G, img_flag);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// K_hist: one radix level of the rank select.  Every element whose magnitude
// key matches its group's prefix above this level's digit adds one to the LDS
// histogram [G][1 << bits]; the workgroup then adds its non-zero bins to the
// global histogram of its image.
// ---------------------------------------------------------------------------
constexpr int kHistThreads = 1024;

template <typename T, int L>
__global__ __launch_bounds__(kHistThreads) void k_hist(const T* __restrict__ X, long long ld, int T_,
                                                       int C, int G, int vec_ok,
                                                       const int* __restrict__ gid,
                                                       const GroupWork* __restrict__ grp,
                                                       u32* __restrict__ hist, int shift, int bits,
                                                       int rows_per_block) {
  extern __shared__ u32 lds[];
  constexpr int V = Elem<T>::V;
  const int b = blockIdx.y;
  const int tid = threadIdx.x;
  const int nwords = G << bits;
  for (int i = tid; i < nwords; i += kHistThreads) lds[i] = 0;
  __syncthreads();

  const int row0 = blockIdx.x * rows_per_block;
  int nrows = T_ - row0;
  nrows = nrows < rows_per_block ? nrows : rows_per_block;
  const u32 mask = (1u << bits) - 1u;
  const int hs = shift + bits;             // bits above this level's digit
  constexpr int SLOTS = kHistThreads / L;
  const int slot = tid / L, lr = tid % L;
  const int nvec = vec_ok ? C / V : 0;
  for (int rr = slot; rr < nrows; rr += SLOTS) {
    const long long row = (long long)b * T_ + row0 + rr;
    const int g = gid[row];
    const u32 prefix = grp[(long long)b * G + g].prefix;
    u32* h = lds + (g << bits);
    const T* xp = X + row * ld;
#pragma unroll 2
    for (int v = lr; v < nvec; v += L) {
      const uint4 q = *reinterpret_cast<const uint4*>(xp + (long long)v * V);
      T e[V];
      Elem<T>::unpack(q, e);
#pragma unroll
      for (int i = 0; i < V; ++i) {
        const u32 k = Elem<T>::key(e[i]);
        if ((hs >= 32 ? 0u : (k >> hs)) == prefix) atomicAdd(&h[(k >> shift) & mask], 1u);
      }
    }
    for (int c = nvec * V + lr; c < C; c += L) {
      const u32 k = Elem<T>::key(xp[c]);
      if ((hs >= 32 ? 0u : (k >> hs)) == prefix) atomicAdd(&h[(k >> shift) & mask], 1u);
    }
  }
  __syncthreads();
  u32* gh = hist + ((size_t)b * G << bits);
  for (int i = tid; i < nwords; i += kHistThreads) {
    const u32 v = lds[i];
    if (v) atomicAdd(&gh[i], v);
  }
}

template <typename T>
static hipError_t hist_t(const T* X, int B, int T_, int C, long long ld, int G, const int* gid,
                         const GroupWork* grp, u32* hist, int shift, int bits, hipStream_t st) {
  constexpr int V = Elem<T>::V;
  const int vec_ok = ((reinterpret_cast<uintptr_t>(X) & 15) == 0 && ld % V == 0) ? 1 : 0;
  const int L = lanes_per_row(C, V);
  // enough workgroups to fill 256 CUs several times over, but at least ~32 Ki
  // elements each so the flush of G << bits bins stays small beside the sweep
  long long rows_min = (32768 + C - 1) / C;
  long long target_blocks = 2048 / (B > 0 ? B : 1);
  if (target_blocks < 1) target_blocks = 1;
  long long rpb = (T_ + target_blocks - 1) / target_blocks;
  if (rpb < rows_min) rpb = rows_min;
  if (rpb > T_) rpb = T_;
  const unsigned chunks = (unsigned)((T_ + rpb - 1) / rpb);
  const size_t lds_bytes = (size_t)(G << bits) * sizeof(u32);
#define TDQ_HIST(LL)                                                                              \
  case LL:                                                                                     \
    hipLaunchKernelGGL((k_hist<T, LL>), dim3(chunks, B), dim3(kHistThreads), lds_bytes, st, X, \
                       ld, T_, C, G, vec_ok, gid, grp, hist, shift, bits, (int)rpb);           \
    break;
  switch (L) {
    TDQ_HIST(1) TDQ_HIST(2) TDQ_HIST(4) TDQ_HIST(8) TDQ_HIST(16) TDQ_HIST(32) TDQ_HIST(64)
  }
#undef TDQ_HIST
  return hipGetLastError();
}

hipError_t launch_hist(const void* X, tdq_dtype dt, int B, int T, int C, long long ld, int G,
                       const int* gid, const GroupWork* grp, unsigned* hist_level, int shift,
                       int bits, hipStream_t st) {
  if (dt == TDQ_F16)
    return hist_t<u16>(static_cast<const u16*>(X), B, T, C, ld, G, gid, grp, hist_level, shift,
                       bits, st);
  return hist_t<float>(static_cast<const float*>(X), B, T, C, ld, G, gid, grp, hist_level, shift,
                       bits, st);
}

// ---------------------------------------------------------------------------
// K_select: one wavefront per (image, token set).  Finds the histogram bin that
// holds rank k_rem, appends its digit to the prefix and reduces the rank.  After
// the last level the prefix IS the magnitude key of the k-th smallest |x|, and the
// wavefront applies the DCRP projection (Eq. dcrp) in binary32.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void k_select(const u32* __restrict__ hist, int bits, int last,
                                               int is_f16, Scalars sc, GroupWork* __restrict__ grp,
                                               float* __restrict__ clip, float* __restrict__ scale,
                                               tdq_group_stats* __restrict__ stats,
                                               const u32* __restrict__ img_flag, int B,
                                               u32* __restrict__ status) {
  const int idx = blockIdx.x;
  const int lane = threadIdx.x;
  if (last && idx == 0) {   // fold the per-image flags into the status word
    u32 f = 0;
    for (int b = lane; b < B; b += 64) f |= img_flag[b];
    const unsigned long long any = __ballot(f != 0);
    if (lane == 0) status[0] = any ? TDQ_DEV_NONFINITE : 0u;
  }
  GroupWork w = grp[idx];
  const int nb = 1 << bits;
  u32 prefix = w.prefix;
  long long k_rem = w.k_rem;
  if (w.tokens != 0) {
    const u32* h = hist + ((size_t)idx << bits);
    const int per = nb >= 64 ? nb / 64 : 1;
    const int first = lane * per;
    unsigned long long mine = 0;
    if (first < nb)
      for (int i = 0; i < per; ++i) mine += h[first + i];
    unsigned long long incl = mine;   // inclusive scan over lanes
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const unsigned long long o = __shfl_up(incl, d, 64);
      if (lane >= d) incl += o;
    }
    const unsigned long long k = (unsigned long long)k_rem;
    const unsigned long long hit = __ballot(incl >= k);
    const int src = hit ? __ffsll((long long)hit) - 1 : 63;   // hit is never 0 for a valid rank
    int bin = 0;
    unsigned long long before = 0;
    if (lane == src) {
      unsigned long long cum = incl - mine;
      int i = 0;
      for (; i < per - 1; ++i) {
        const unsigned long long c = h[first + i];
        if (cum + c >= k) break;
        cum += c;
      }
      bin = first + i;
      before = cum;
    }
    bin = __shfl(bin, src, 64);
    before = __shfl(before, src, 64);
    prefix = (prefix << bits) | (u32)bin;
    k_rem = (long long)(k - before);
  }
  if (!last) {
    if (lane == 0) {
      grp[idx].prefix = prefix;
      grp[idx].k_rem = k_rem;
    }
    return;
  }
  if (lane != 0) return;
  float thr = 0.f, c_tau = 0.f, c_zr = 0.f, c, d;
  u32 bind = TDQ_BIND_EMPTY;
  long long kk = 0;
  if (w.tokens == 0) {
    c = sc.eps_scale;
    d = sc.eps_scale;
  } else {
    thr = is_f16 ? h2f(prefix) : __uint_as_float(prefix);
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

hipError_t launch_select(unsigned* hist_level, int B, int G, int, int bits, bool last, tdq_dtype dt,
                         const Scalars& sc, GroupWork* grp, float* clip, float* scale,
                         tdq_group_stats* stats, const unsigned* img_flag, unsigned* status,
                         hipStream_t st) {
  hipLaunchKernelGGL(k_select, dim3(B * G), dim3(64), 0, st, hist_level, bits, last ? 1 : 0,
                     dt == TDQ_F16 ? 1 : 0, sc, grp, clip, scale, stats, img_flag, B, status);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// K_c: quantize + pack.  q = clamp(rint(clip(x, +-c) / Delta), -8, 7).
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

template <typename T, int L>
__global__ __launch_bounds__(256) void k_quantize(const T* __restrict__ X, long long ld, int M, int C,
                                                  int T_, int G, int vec_ok,
                                                  const int* __restrict__ gid,
                                                  const float* __restrict__ clip,
                                                  const float* __restrict__ scale,
                                                  uint8_t* __restrict__ Q, long long ld_q) {
  constexpr int V = Elem<T>::V;
  constexpr int U = 8 / V;                 // 16-byte loads per 8 elements
  const long long gt = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long row = gt / L;
  const int lr = (int)(gt % L);
  if (row >= M) return;
  const int b = (int)(row / T_);
  const int g = gid ? gid[row] : 0;
  const float c = clip[(long long)b * G + g];
  const float d = scale[(long long)b * G + g];
  const float rcp = 1.0f / d;              // correctly rounded reciprocal
  const T* xp = X + row * ld;
  uint8_t* qp = Q + row * ld_q;
  const int n8 = vec_ok ? C / 8 : 0;       // units of 8 elements -> one 32-bit store
#pragma unroll 2
  for (int u = lr; u < n8; u += L) {
    u32 word = 0;
#pragma unroll
    for (int j = 0; j < U; ++j) {
      const uint4 q = *reinterpret_cast<const uint4*>(xp + (long long)u * 8 + j * V);
      T e[V];
      Elem<T>::unpack(q, e);
#pragma unroll
      for (int i = 0; i < V; ++i)
        word |= quant_nibble(Elem<T>::val(e[i]), c, d, rcp) << (4 * (j * V + i));
    }
    *reinterpret_cast<u32*>(qp + (long long)u * 4) = word;
  }
  // ragged tail / unaligned rows: one byte (two elements) at a time
  const int nbytes = (C + 1) / 2;
  for (int by = n8 * 4 + lr; by < nbytes; by += L) {
    const int c0 = 2 * by;
    u32 v = quant_nibble(Elem<T>::val(xp[c0]), c, d, rcp);
    if (c0 + 1 < C) v |= quant_nibble(Elem<T>::val(xp[c0 + 1]), c, d, rcp) << 4;
    qp[by] = (uint8_t)v;
  }
}

template <typename T>
static hipError_t quantize_t(const T* X, int B, int T_, int C, long long ld, int G, const int* gid,
                             const float* clip, const float* scale, uint8_t* Q, long long ld_q,
                             hipStream_t st) {
  constexpr int V = Elem<T>::V;
  const int vec_ok = ((reinterpret_cast<uintptr_t>(X) & 15) == 0 && ld % V == 0 &&
                      (reinterpret_cast<uintptr_t>(Q) & 3) == 0 && ld_q % 4 == 0)
                         ? 1 : 0;
  const int L = lanes_per_row(C, 8);
  const long long M = (long long)B * T_;
  const long long threads = M * L;
  const unsigned grid = (unsigned)((threads + 255) / 256);
#define TDQ_Q(LL)                                                                               \
  case LL:                                                                                      \
    hipLaunchKernelGGL((k_quantize<T, LL>), dim3(grid), dim3(256), 0, st, X, ld, (int)M, C, T_, \
                       G, vec_ok, gid, clip, scale, Q, ld_q);                                   \
    break;
  switch (L) {
    TDQ_Q(1) TDQ_Q(2) TDQ_Q(4) TDQ_Q(8) TDQ_Q(16) TDQ_Q(32) TDQ_Q(64)
  }
#undef TDQ_Q
  return hipGetLastError();
}

hipError_t launch_quantize(const void* X, tdq_dtype dt, int B, int T, int C, long long ld, int G,
                           const int* gid, const float* clip, const float* scale, uint8_t* Q,
                           long long ld_q, hipStream_t st) {
  if (dt == TDQ_F16)
    return quantize_t<u16>(static_cast<const u16*>(X), B, T, C, ld, G, gid, clip, scale, Q, ld_q,
                           st);
  return quantize_t<float>(static_cast<const float*>(X), B, T, C, ld, G, gid, clip, scale, Q, ld_q,
                           st);
}

// ---------------------------------------------------------------------------
// Offline weight quantizer (Eq. weight_quant): one wavefront per output channel.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void k_quantize_weight(const float* __restrict__ W, int K,
                                                        long long ld_in, uint8_t* __restrict__ Qw,
                                                        long long ld_w, float* __restrict__ w_scale) {
  const int o = blockIdx.x, lane = threadIdx.x;
  const float* wp = W + (long long)o * ld_in;
  u32 kmax = 0;
  for (int i = lane; i < K; i += 64) {
    const u32 k = __float_as_uint(wp[i]) & 0x7FFFFFFFu;
    kmax = k > kmax ? k : kmax;
  }
  kmax = wave_max_u32(kmax);
  float amax = __uint_as_float(kmax);
  amax = amax > 1e-8f ? amax : 1e-8f;
  const float s = amax / (float)kQMax;
  if (lane == 0) w_scale[o] = s;
  uint8_t* qp = Qw + (long long)o * ld_w;
  const int nbytes = (K + 1) / 2;
  for (long long by = lane; by < ld_w; by += 64) {
    u32 v = 0;
    if (by < nbytes) {
      const int c0 = 2 * (int)by;
      float y = rintf(wp[c0] / s);
      y = fminf(fmaxf(y, (float)kQMin), (float)kQMax);
      v = (u32)((int)y) & 0xFu;
      if (c0 + 1 < K) {
        float y1 = rintf(wp[c0 + 1] / s);
        y1 = fminf(fmaxf(y1, (float)kQMin), (float)kQMax);
        v |= ((u32)((int)y1) & 0xFu) << 4;
      }
    }
    qp[by] = (uint8_t)v;
  }
}

hipError_t launch_quantize_weight(const float* W, int N, int K, long long ld_in, uint8_t* Qw,
                                  long long ld_w, float* w_scale, hipStream_t st) {
  hipLaunchKernelGGL(k_quantize_weight, dim3(N), dim3(64), 0, st, W, K, ld_in, Qw, ld_w, w_scale);
  return hipGetLastError();
}

}  // namespace tdq
