// Activation side of the W4A4 path: per-token statistics, token-set assignment,
// exact rank select of the zr quantile with LDS histograms, DCRP projection,
// quantize + pack, and the offline weight quantizer.  gfx950 only.
//
// Paper passages: Sec. 4.2 (DSTG: base radius, group dispersion, Eqs. DSTG_clip,
// clipx, dequant), Sec. 4.3 (DCRP: Eqs. tau_constraint, zr_constraint, dcrp),
// Supp. "Quantile Implementation" (rank k = ceil(p n)), Supp. numerical
// conventions (eps values, ties-to-even rounding), Eq. weight_quant.
#include "tdq_device.hpp"

namespace tdq {

// ---------------------------------------------------------------------------
// K_a: per-token range and moments (one sweep of X)
//   r_t = max_c |x|  (exact: integer max of the magnitude bit patterns)
//   (mean_t, M2_t) with M2_t = sum_c (x - mean_t)^2, summed about a pivot P taken from
//   the row (see "Moments" in tdq_device.hpp).  binary16 input: a lane adds the 8
//   differences x - P of a 16-byte load and their squares in binary32, then accumulates
//   in binary64; binary32 input: binary64 throughout.
// ---------------------------------------------------------------------------
template <typename T>
struct PivotOf { typedef double type; };
template <>
struct PivotOf<u16> { typedef float type; };

// One 16-byte piece of a row added to a lane's partial sums about the pivot P.
template <typename T>
struct RowAcc;
template <>
struct RowAcc<u16> {
  us2 kpk = {0, 0};                     // running max of the magnitude keys, two at a time
  double a1 = 0.0, a2 = 0.0;
  float one, nP;
  __device__ __forceinline__ explicit RowAcc(float P) : nP(-P) {
    one = 1.0f;                         // opaque to the optimizer, so x * one - P stays ONE mixed fma
    asm volatile("" : "+v"(one));
  }
  // Per element: d = x - P as one mixed-precision fma (the fp16 -> fp32 conversion rides in
  // the instruction), one add for the sum and one fma for the sum of squares; the keys of a
  // pair of elements are maxed with one packed 16-bit instruction.
  __device__ __forceinline__ void add(const uint4& q) {
    const u32 w[4] = {q.x, q.y, q.z, q.w};
    float p1, p2;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const h2 h = __builtin_bit_cast(h2, w[j]);
      kpk = __builtin_elementwise_max(kpk, __builtin_bit_cast(us2, w[j] & 0x7FFF7FFFu));
      const float d0 = __builtin_fmaf((float)h[0], one, nP);
      const float d1 = __builtin_fmaf((float)h[1], one, nP);
      if (j == 0) {
        p1 = d0;
        p2 = d0 * d0;
      } else {
        p1 += d0;
        p2 = __builtin_fmaf(d0, d0, p2);
      }
      p1 += d1;
      p2 = __builtin_fmaf(d1, d1, p2);
    }
    a1 += (double)p1;
    a2 += (double)p2;
  }
  __device__ __forceinline__ void add_one(u16 x, u32& kmax) {
    const double d = (double)h2f(x) + (double)nP;
    const u32 k = x & 0x7FFFu;
    kmax = k > kmax ? k : kmax;
    a1 += d;
    a2 = fma(d, d, a2);
  }
  __device__ __forceinline__ u32 key_max() const { return kpk[0] > kpk[1] ? kpk[0] : kpk[1]; }
};
template <>
struct RowAcc<float> {
  u32 km = 0;
  double a1 = 0.0, a2 = 0.0;
  double P;
  __device__ __forceinline__ explicit RowAcc(double P_) : P(P_) {}
  __device__ __forceinline__ void add(const uint4& q) {
    const u32 w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const double d = (double)__uint_as_float(w[i]) - P;
      const u32 k = w[i] & 0x7FFFFFFFu;
      km = k > km ? k : km;
      a1 += d;
      a2 = fma(d, d, a2);
    }
  }
  __device__ __forceinline__ void add_one(float x, u32& kmax) {
    const double d = (double)x - P;
    const u32 k = __float_as_uint(x) & 0x7FFFFFFFu;
    kmax = k > kmax ? k : kmax;
    a1 += d;
    a2 = fma(d, d, a2);
  }
  __device__ __forceinline__ u32 key_max() const { return km; }
};

// The part of a row that one of NL cooperating lanes (index lr) sees: 16-byte pieces
// lr, lr + NL, ... and, past the last whole piece, single elements.  Every lane has
// nvec / NL whole rounds (a uniform count, so the branches below are scalar) and the
// first nvec % NL lanes one more piece; the rounds are taken four, then two, then one
// at a time with the loads of a step issued together, so a lane has several loads in
// flight however short its share of the row is.
template <typename T, int NL>
__device__ __forceinline__ void row_partial(const T* __restrict__ xp, int lr, int nvec, int C,
                                            typename PivotOf<T>::type P, u32& kmax, double& a1,
                                            double& a2) {
  constexpr int V = Elem<T>::V;
  RowAcc<T> acc(P);
  const uint4* xv = reinterpret_cast<const uint4*>(xp);
  int v = lr;
  int rounds = nvec / NL;
  for (; rounds >= 4; rounds -= 4, v += 4 * NL) {
    const uint4 q0 = xv[v], q1 = xv[v + NL], q2 = xv[v + 2 * NL], q3 = xv[v + 3 * NL];
    acc.add(q0);
    acc.add(q1);
    acc.add(q2);
    acc.add(q3);
  }
  if (rounds >= 2) {
    const uint4 q0 = xv[v], q1 = xv[v + NL];
    acc.add(q0);
    acc.add(q1);
    v += 2 * NL;
    rounds -= 2;
  }
  if (rounds >= 1) {
    acc.add(xv[v]);
    v += NL;
  }
  if (v < nvec) acc.add(xv[v]);
  kmax = acc.key_max();
  for (int c = nvec * V + lr; c < C; c += NL) acc.add_one(xp[c], kmax);   // ragged tail / unaligned rows
  a1 = acc.a1;
  a2 = acc.a2;
}

template <typename T, int L>
__global__ __launch_bounds__(256) void k_token_stats(const T* __restrict__ X, long long ld, int M,
                                                     int C, double inv_n, int vec_ok,
                                                     float* __restrict__ r,
                                                     double* __restrict__ mean,
                                                     double* __restrict__ m2) {
  constexpr int V = Elem<T>::V;
  typedef typename PivotOf<T>::type PT;
  const long long gt = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long row = gt / L;
  const int lr = (int)(gt % L);
  const bool valid = row < M;
  const T* xp = X + (valid ? row : (long long)(M - 1)) * ld;
  const int nvec = vec_ok ? C / V : 0;
  PT P = row_pivot(xp, C, nvec > 0);
  u32 kmax;
  double a1, a2;
  row_partial<T, L>(xp, lr, nvec, C, P, kmax, a1, a2);
  kmax = group_max_u32<L>(kmax);
  a1 = group_sum_f64<L>(a1);                       // totals in the row's last lane
  a2 = group_sum_f64<L>(a2);
  if constexpr (sizeof(T) == 2) {
    // A pivot far from the row's mean: all rows of this wavefront are summed again, each
    // about its own mean (uniform branch; the data comes from the cache).
    const bool far = lr == L - 1 && pivot_is_far(a1, a2, C);
    if (__ballot(far)) {
      const float pn = P + (float)(a1 * inv_n);
      P = __shfl(pn, (int)(threadIdx.x & 63) | (L - 1), 64);
      u32 k2;
      row_partial<T, L>(xp, lr, nvec, C, P, k2, a1, a2);
      a1 = group_sum_f64<L>(a1);
      a2 = group_sum_f64<L>(a2);
    }
  }
  if (lr == L - 1 && valid) {
    double mu, q;
    pivot_to_central((double)P, a1, a2, inv_n, mu, q);
    r[row] = Elem<T>::key_to_float(kmax);
    mean[row] = mu;
    m2[row] = q;
  }
}

// Wide rows (at least 256 16-byte pieces): one workgroup of four wavefronts per row,
// so every lane issues only a few loads and the chip runs many short wavefronts
// (measured faster for streaming reads than few long ones).  The four wavefront
// totals are combined through LDS in a fixed order.
template <typename T>
__global__ __launch_bounds__(256) void k_token_stats_wide(const T* __restrict__ X, long long ld, int M,
                                                          int C, double inv_n,
                                                          float* __restrict__ r,
                                                          double* __restrict__ mean,
                                                          double* __restrict__ m2) {
  constexpr int V = Elem<T>::V;
  typedef typename PivotOf<T>::type PT;
  __shared__ double sh1[2][4], sh2[2][4];
  __shared__ u32 shk[4];
  const long long row = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const T* xp = X + row * ld;
  const int nvec = C / V;
  PT P = row_pivot(xp, C, true);
  u32 kmax;
  double a1, a2;
  row_partial<T, 256>(xp, tid, nvec, C, P, kmax, a1, a2);
  kmax = group_max_u32<64>(kmax);
  a1 = group_sum_f64<64>(a1);
  a2 = group_sum_f64<64>(a2);
  if (lane == 63) { shk[wave] = kmax; sh1[0][wave] = a1; sh2[0][wave] = a2; }
  __syncthreads();
  // every thread adds the four totals in the same order: the same bits everywhere
  double t1 = sh1[0][0], t2 = sh2[0][0];
  for (int w = 1; w < 4; ++w) { t1 += sh1[0][w]; t2 += sh2[0][w]; }
  if constexpr (sizeof(T) == 2) {
    if (pivot_is_far(t1, t2, C)) {                 // uniform over the workgroup
      P = P + (float)(t1 * inv_n);
      u32 k2;
      row_partial<T, 256>(xp, tid, nvec, C, P, k2, a1, a2);
      a1 = group_sum_f64<64>(a1);
      a2 = group_sum_f64<64>(a2);
      if (lane == 63) { sh1[1][wave] = a1; sh2[1][wave] = a2; }
      __syncthreads();
      t1 = sh1[1][0];
      t2 = sh2[1][0];
      for (int w = 1; w < 4; ++w) { t1 += sh1[1][w]; t2 += sh2[1][w]; }
    }
  }
  if (tid == 0) {
    u32 k = shk[0];
    for (int w = 1; w < 4; ++w) k = shk[w] > k ? shk[w] : k;
    double mu, q;
    pivot_to_central((double)P, t1, t2, inv_n, mu, q);
    r[row] = Elem<T>::key_to_float(k);
    mean[row] = mu;
    m2[row] = q;
  }
}

// Lanes per row of the statistics sweep: enough that a wavefront's load instruction
// covers whole 128-byte lines (8 lanes), otherwise as few as leave every lane about 4
// pieces, all loaded at once -- the reduction over the row's lanes costs as many vector
// instructions as 2 pieces do, and with fewer pieces per lane it, not the memory system,
// sets the pace (C = 1024: 47.3 / 45.5 / 60.4 us at 8 / 4 / 2 pieces per lane).
static int stats_lanes_per_row(int C, int V) {
  const int nvec = (C + V - 1) / V;
  int L = 1;
  while (L < nvec && L < 8) L <<= 1;
  while (L < 64 && L * 4 < nvec) L <<= 1;
  return L;
}

template <typename T>
static hipError_t token_stats_t(const T* X, int M, int C, long long ld, float* r, double* mean,
                                double* m2, hipStream_t st) {
  constexpr int V = Elem<T>::V;
  const int vec_ok = ((reinterpret_cast<uintptr_t>(X) & 15) == 0 && ld % V == 0) ? 1 : 0;
  if (vec_ok && C / V >= 256) {
    hipLaunchKernelGGL((k_token_stats_wide<T>), dim3(M), dim3(256), 0, st, X, ld, M, C,
                       1.0 / (double)C, r, mean, m2);
    return hipGetLastError();
  }
  const int L = stats_lanes_per_row(C, V);
  const long long threads = (long long)M * L;
  const unsigned grid = (unsigned)((threads + 255) / 256);
#define TDQ_TS(LL)                                                                       \
  case LL:                                                                               \
    hipLaunchKernelGGL((k_token_stats<T, LL>), dim3(grid), dim3(256), 0, st, X, ld, M, C, \
                       1.0 / (double)C, vec_ok, r, mean, m2);                            \
    break;
  switch (L) {
    TDQ_TS(1) TDQ_TS(2) TDQ_TS(4) TDQ_TS(8) TDQ_TS(16) TDQ_TS(32) TDQ_TS(64)
  }
#undef TDQ_TS
  return hipGetLastError();
}

hipError_t launch_token_stats(const void* X, tdq_dtype dt, int M, int C, long long ld, float* r,
                              double* mean, double* m2, hipStream_t st) {
  if (dt == TDQ_F16)
    return token_stats_t<u16>(static_cast<const u16*>(X), M, C, ld, r, mean, m2, st);
  return token_stats_t<float>(static_cast<const float*>(X), M, C, ld, r, mean, m2, st);
}

// ---------------------------------------------------------------------------
// K_assign: one workgroup per image.
//   key_t = bits(r_t); hi = max key; lo = max(min key, hi - 24 octaves);
//   gid_t = key_t <= lo ? 0 : (key_t - lo) * G / (hi - lo + 1)      (64-bit integers)
// then per token set: token count, c_base = max r_t, and the tokens' moments merged about
// a pivot from inside the set (setacc_add) -> sigma = sqrt(S2/n - (S1/n)^2) + eps_std in
// binary64, rank k = ceil(zr n).
// Also clears this image's histogram slices and records whether the image holds
// a non-finite value (its largest range key is Inf/NaN).
// ---------------------------------------------------------------------------
constexpr int kAssignThreads = 1024;

__global__ __launch_bounds__(kAssignThreads) void k_assign(
    const float* __restrict__ r, const double* __restrict__ mean, const double* __restrict__ m2,
    int T, int C, int G, int* __restrict__ gid, SetAcc* __restrict__ part,
    u32* __restrict__ img_flag, u32* __restrict__ status) {
  extern __shared__ __attribute__((aligned(16))) unsigned char assign_lds[];
  __shared__ u32 s_min[kAssignThreads / 64], s_max[kAssignThreads / 64];
  __shared__ u32 s_lohi[2];
  SetAcc* wacc = reinterpret_cast<SetAcc*>(assign_lds);     // [NW][G]
  // S workgroups share an image: each finds the image's key range over all T tokens
  // (cheap) and then handles every S-th group of token batches
  const int b = blockIdx.y, sub = blockIdx.x, S = gridDim.x;
  const int tid = threadIdx.x;
  const int NW = blockDim.x >> 6;
  assign_tokens(r + (long long)b * T, mean + (long long)b * T, m2 + (long long)b * T, T, C, G,
                gid + (long long)b * T, wacc, s_min, s_max, s_lohi, sub, S);
  if (tid == 0 && sub == 0) {
    img_flag[b] = s_lohi[1] >= 0x7F800000u ? TDQ_DEV_NONFINITE : 0u;
    if (b == 0) {                         // counts of sets the single-sweep select misses
      status[1] = 0u;
      status[2] = 0u;
    }
  }
  for (int g = tid; g < G; g += blockDim.x) {      // merge the wavefronts in a fixed order
    SetAcc m;
    m.s1 = 0.0; m.s2 = 0.0; m.piv = 0.0; m.cnt = 0; m.kmax = 0;
    for (int w = 0; w < NW; ++w) setacc_add(m, wacc[w * G + g], (double)C);
    part[((long long)b * S + sub) * G + g] = m;
  }
}

// One workgroup per (image, token set): merges the partial records into the working
// record of this pass and clears the set's radix-level histograms.
__global__ __launch_bounds__(256) void k_finalize_groups(const SetAcc* __restrict__ part, int S, int G,
                                                         int C, Scalars sc, int pass, int keep_base,
                                                         GroupWork* __restrict__ grp,
                                                         u32* __restrict__ hist, LevelPlan lp) {
  const int idx = blockIdx.x;
  if (threadIdx.x == 0) {
    GroupWork w = merge_partials(part, idx / G, idx % G, S, G, C, sc, pass);
    if (keep_base) w.c_base = grp[idx].c_base;
    grp[idx] = w;
  }
  clear_level_hists(hist, lp, gridDim.x, idx, threadIdx.x, 256);
}

int assign_split(int T) {
  int s = T / 1024;                        // about 16 batches of 64 tokens per workgroup
  return s < 1 ? 1 : (s > kAssignSplitMax ? kAssignSplitMax : s);
}

hipError_t launch_assign(const float* r, const double* mean, const double* m2, int B, int T, int C,
                         int G, int* gid, void* part, unsigned* img_flag, unsigned* status,
                         hipStream_t st) {
  int nw = 1536 / G;                       // keep the per-wavefront accumulators under 48 KiB
  nw = nw > kAssignThreads / 64 ? kAssignThreads / 64 : (nw < 1 ? 1 : nw);
  const size_t lds = (size_t)nw * G * sizeof(SetAcc);
  hipLaunchKernelGGL(k_assign, dim3(assign_split(T), B), dim3(nw * 64), lds, st, r, mean, m2, T, C,
                     G, gid, static_cast<SetAcc*>(part), img_flag, status);
  return hipGetLastError();
}

hipError_t launch_finalize_groups(const void* part, int B, int T, int C, int G, const Scalars& sc,
                                  int pass, bool keep_base, GroupWork* grp, unsigned* hist,
                                  const LevelPlan& lp, hipStream_t st) {
  hipLaunchKernelGGL(k_finalize_groups, dim3(B * G), dim3(256), 0, st,
                     static_cast<const SetAcc*>(part), assign_split(T), G, C, sc, pass,
                     keep_base ? 1 : 0, grp, hist, lp);
  return hipGetLastError();
}

size_t assign_partial_bytes(int B, int G) {
  return (size_t)B * kAssignSplitMax * G * sizeof(SetAcc);
}

// ---------------------------------------------------------------------------
// K_hist: one radix level of the rank select.  Every element whose magnitude
// key matches its group's prefix above this level's digit adds one to the LDS
// histogram [G][1 << bits]; the workgroup then adds its non-zero bins to the
// global histogram of its image.
// ---------------------------------------------------------------------------
constexpr int kHistThreads = 1024;

template <typename T, int L, bool FIRST>
__global__ __launch_bounds__(kHistThreads) void k_hist(const T* __restrict__ X, long long ld, int T_,
                                                       int C, int G, int vec_ok,
                                                       const int* __restrict__ gid,
                                                       const GroupWork* __restrict__ grp,
                                                       u32* __restrict__ hist, int shift, int bits,
                                                       int rows_per_block) {
  extern __shared__ u32 lds[];
  constexpr int V = Elem<T>::V;
  // The top level walks X backwards: it runs right after the forward statistics sweep,
  // so the end of X is what the last-level cache still holds.
  const int b = FIRST ? (int)(gridDim.y - 1 - blockIdx.y) : (int)blockIdx.y;
  const int chunk = FIRST ? (int)(gridDim.x - 1 - blockIdx.x) : (int)blockIdx.x;
  const int tid = threadIdx.x;
  const int nwords = G << bits;
  for (int i = tid; i < nwords; i += kHistThreads) lds[i] = 0;
  __syncthreads();

  const int row0 = chunk * rows_per_block;
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
    const u32 prefix = FIRST ? 0u : grp[(long long)b * G + g].prefix;
    u32* h = lds + (g << bits);
    const T* xp = X + row * ld;
#pragma unroll 2
    for (int v = lr; v < nvec; v += L) {
      const uint4 q = *reinterpret_cast<const uint4*>(xp + (long long)v * V);
      if constexpr (FIRST && sizeof(T) == 2) {
        // top level of fp16: the digit is a bit field of the packed word (the sign
        // bit lies above it), one extract and one address add per element
        const u32 w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          atomicAdd(&h[__builtin_amdgcn_ubfe(w[j], (u32)shift, (u32)bits)], 1u);
          atomicAdd(&h[__builtin_amdgcn_ubfe(w[j], (u32)(16 + shift), (u32)bits)], 1u);
        }
      } else {
        T e[V];
        Elem<T>::unpack(q, e);
#pragma unroll
        for (int i = 0; i < V; ++i) {
          const u32 k = Elem<T>::key(e[i]);
          if (FIRST || (hs >= 32 ? 0u : (k >> hs)) == prefix) atomicAdd(&h[(k >> shift) & mask], 1u);
        }
      }
    }
    for (int c = nvec * V + lr; c < C; c += L) {
      const u32 k = Elem<T>::key(xp[c]);
      if (FIRST || (hs >= 32 ? 0u : (k >> hs)) == prefix) atomicAdd(&h[(k >> shift) & mask], 1u);
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
  const bool first = shift + bits >= (int)(sizeof(T) == 2 ? 15 : 31);   // the top level: no prefix yet
#define TDQ_HIST(LL)                                                                              \
  case LL:                                                                                     \
    if (first) {                                                                               \
      if (lds_bytes > 65536)                                                                   \
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_hist<T, LL, true>),         \
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes); \
      hipLaunchKernelGGL((k_hist<T, LL, true>), dim3(chunks, B), dim3(kHistThreads), lds_bytes, \
                         st, X, ld, T_, C, G, vec_ok, gid, grp, hist, shift, bits, (int)rpb);  \
    } else {                                                                                   \
      hipLaunchKernelGGL((k_hist<T, LL, false>), dim3(chunks, B), dim3(kHistThreads), lds_bytes, \
                         st, X, ld, T_, C, G, vec_ok, gid, grp, hist, shift, bits, (int)rpb);  \
    }                                                                                          \
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
                                               u32* __restrict__ status, int pass) {
  const int idx = blockIdx.x;
  const int lane = threadIdx.x;
  if (last && idx == 0 && pass == kPassZr) {   // fold the per-image flags into the status word
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
  if (pass == kPassBase) {       // the order statistic found is the set's base radius Q_p(|x|)
    if (w.tokens != 0) grp[idx].c_base = is_f16 ? h2f(prefix) : __uint_as_float(prefix);
    return;
  }
  project_store(idx, w, prefix, is_f16 != 0, sc, clip, scale, stats);
}

hipError_t launch_select(unsigned* hist_level, int B, int G, int, int bits, bool last, tdq_dtype dt,
                         const Scalars& sc, GroupWork* grp, float* clip, float* scale,
                         tdq_group_stats* stats, const unsigned* img_flag, unsigned* status,
                         int pass, hipStream_t st) {
  hipLaunchKernelGGL(k_select, dim3(B * G), dim3(64), 0, st, hist_level, bits, last ? 1 : 0,
                     dt == TDQ_F16 ? 1 : 0, sc, grp, clip, scale, stats, img_flag, B, status, pass);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// K_c: quantize + pack (the per-element arithmetic is in tdq_device.hpp).
// ---------------------------------------------------------------------------
// 16 bytes of X that nobody reads again after this sweep: a non-temporal load keeps
// them from displacing the packed codes, which the contraction reads next (measured on
// the 4096-channel layer of the largest configuration: this sweep 244 -> 205 us, and the
// contraction that follows 3 to 5 % faster).
template <typename T>
__device__ __forceinline__ uint4 load_last_use(const T* p) {
  typedef unsigned v4u __attribute__((ext_vector_type(4)));
  const v4u v = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(p));
  return make_uint4(v[0], v[1], v[2], v[3]);
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
  // rows are walked from the end of X (measured: no slower than forwards after either
  // form of the rank select)
  const long long gt = (long long)(gridDim.x - 1 - blockIdx.x) * 256 + threadIdx.x;
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
  if constexpr (sizeof(T) == 2) {
    const bool need_clamp = !(c <= 7.25f * d);
    if (__builtin_amdgcn_ballot_w64(need_clamp) == 0) {
#pragma unroll 4
      for (int u = lr; u < n8; u += L) {
        const uint4 q = load_last_use(xp + (long long)u * 8);
        *reinterpret_cast<u32*>(qp + (long long)u * 4) = quant8_f16<false>(q, c, d, rcp);
      }
    } else {
#pragma unroll 2
      for (int u = lr; u < n8; u += L) {
        const uint4 q = load_last_use(xp + (long long)u * 8);
        *reinterpret_cast<u32*>(qp + (long long)u * 4) = quant8_f16<true>(q, c, d, rcp);
      }
    }
  } else
#pragma unroll 2
  for (int u = lr; u < n8; u += L) {
    u32 word = 0;
#pragma unroll
    for (int j = 0; j < U; ++j) {
      const uint4 q = load_last_use(xp + (long long)u * 8 + j * V);
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
// K_c writing the operand format of the 6-bit contraction (tdq_w4a4_linear_f6): the same
// codes, each as the bf6 (e3m2) pattern of its integer value, in fragments of 32 rows x
// 64 codes laid out in the lane order of the matrix instruction.  One wavefront per
// fragment; lane l = row % 32 + 32 * ((k % 64) / 32) quantizes 32 consecutive elements of
// its row, rounds the quotients to integers (the same arithmetic as k_quantize) and
// packs them with one conversion instruction, which takes the even elements in its first
// and the odd ones in its second operand; a wavefront stores 1536 contiguous bytes.
// ---------------------------------------------------------------------------
typedef float v16f_t __attribute__((ext_vector_type(16)));
typedef int v6i_t __attribute__((ext_vector_type(6)));

template <typename T>
__global__ __launch_bounds__(256) void k_quantize_f6(const T* __restrict__ X, long long ld, int M, int C,
                                                     int T_, int G, int KB, int vec_ok,
                                                     const int* __restrict__ gid,
                                                     const float* __restrict__ clip,
                                                     const float* __restrict__ scale,
                                                     uint8_t* __restrict__ F, long long n_blocks) {
  constexpr int V = Elem<T>::V;
  constexpr int ROWB = 64 * (int)sizeof(T);                  // bytes of a fragment's row of X
  constexpr int PITCH = ROWB + 16;                           // LDS row pitch: 16-byte reads stay aligned
  constexpr int PPR = ROWB / 16;                             // 16-byte pieces per row: 8 or 16
  __shared__ __attribute__((aligned(16))) uint8_t stage[4][32 * PITCH];
  const int wave = threadIdx.x >> 6, l = threadIdx.x & 63;
  const long long blk_raw = (long long)blockIdx.x * 4 + wave;
  const bool live = blk_raw < n_blocks;                      // a wavefront without a fragment idles along
  const long long blk = live ? blk_raw : n_blocks - 1;
  const int kb = (int)(blk % KB);
  const long long row0 = (blk / KB) * 32;
  const long long row = row0 + (l & 31);
  const int k0 = kb * 64 + 32 * (l >> 5);
  // whole fragments of aligned rows go through LDS: the global loads then read every
  // 128-byte line exactly once, 8 (16) lanes to a row, and the lane that owns (row, half)
  // in the matrix instruction's order picks its 32 elements up from there
  const bool tile_ok = vec_ok && kb * 64 + 64 <= C && row0 + 32 <= M;      // uniform per wavefront
  if (tile_ok) {
#pragma unroll
    for (int j = 0; j < 32 * PPR / 64; ++j) {
      const int r = j * (64 / PPR) + l / PPR, pc = l % PPR;
      const uint4 w = load_last_use(reinterpret_cast<const T*>(
          reinterpret_cast<const uint8_t*>(X + (row0 + r) * ld + kb * 64) + pc * 16));
      *reinterpret_cast<uint4*>(&stage[wave][r * PITCH + pc * 16]) = w;
    }
  }
  __syncthreads();
  v16f_t ev, od;                                             // even / odd elements, as rounded quotients
#pragma unroll
  for (int i = 0; i < 16; ++i) { ev[i] = 0.f; od[i] = 0.f; }
  if (row < M && k0 < C) {
    const int b = (int)(row / T_);
    const int g = gid ? gid[row] : 0;
    const float c = clip[(long long)b * G + g], d = scale[(long long)b * G + g];
    const float rcp = 1.0f / d;
    const T* xp = X + row * ld + k0;
    auto q = [&](float x) {                                  // integer-valued float in [-8, 7]
      return __uint_as_float(quant_bits<true>(x, c, d, rcp)) - 12582912.0f;
    };
    if (tile_ok || (vec_ok && k0 + 32 <= C)) {
#pragma unroll
      for (int j = 0; j < 32 / V; ++j) {
        uint4 w;
        if (tile_ok)
          w = *reinterpret_cast<const uint4*>(&stage[wave][(l & 31) * PITCH + (l >> 5) * (ROWB / 2) + j * 16]);
        else
          w = *reinterpret_cast<const uint4*>(xp + j * V);   // plain: the line is shared with lane l ^ 32
        T e[V];
        Elem<T>::unpack(w, e);
#pragma unroll
        for (int i = 0; i < V; i += 2) {
          ev[(j * V + i) >> 1] = q(Elem<T>::val(e[i]));
          od[(j * V + i) >> 1] = q(Elem<T>::val(e[i + 1]));
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        if (k0 + 2 * i < C) ev[i] = q(Elem<T>::val(xp[2 * i]));
        if (k0 + 2 * i + 1 < C) od[i] = q(Elem<T>::val(xp[2 * i + 1]));
      }
    }
  }
  const v6i_t r = __builtin_amdgcn_cvt_scalef32_2xpk16_bf6_f32(ev, od, 1.0f);
  if (live) {
    uint2* dst = reinterpret_cast<uint2*>(F + (blk * 64 + l) * 24);
    dst[0] = make_uint2((u32)r[0], (u32)r[1]);
    dst[1] = make_uint2((u32)r[2], (u32)r[3]);
    dst[2] = make_uint2((u32)r[4], (u32)r[5]);
  }
}

hipError_t launch_quantize_f6(const void* X, tdq_dtype dt, int B, int T, int C, long long ld, int G,
                              const int* gid, const float* clip, const float* scale, uint8_t* F,
                              hipStream_t st) {
  const long long M = (long long)B * T;
  const int KB = 2 * ((C + 127) / 128);
  const long long n_blocks = ((M + 31) / 32) * KB;
  const unsigned grid = (unsigned)((n_blocks + 3) / 4);
  if (dt == TDQ_F16) {
    const int vec_ok = ((reinterpret_cast<uintptr_t>(X) & 15) == 0 && ld % 8 == 0) ? 1 : 0;
    hipLaunchKernelGGL((k_quantize_f6<u16>), dim3(grid), dim3(256), 0, st, static_cast<const u16*>(X),
                       ld, (int)M, C, T, G, KB, vec_ok, gid, clip, scale, F, n_blocks);
  } else {
    const int vec_ok = ((reinterpret_cast<uintptr_t>(X) & 15) == 0 && ld % 4 == 0) ? 1 : 0;
    hipLaunchKernelGGL((k_quantize_f6<float>), dim3(grid), dim3(256), 0, st,
                       static_cast<const float*>(X), ld, (int)M, C, T, G, KB, vec_ok, gid, clip, scale,
                       F, n_blocks);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Diagnostics of Sec. 3.2 per (image, token set), as exact counts: elements whose code
// is 0 (zero-bin mass rho_0 = count / n, Eq. rho0_def) and elements clipped by the
// radius (|x| > c).  The code is computed exactly as K_c computes it.  One sweep of X.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_group_diag(const T* __restrict__ X, long long ld, int T_, int C,
                                                    int G, const int* __restrict__ gid,
                                                    const float* __restrict__ clip,
                                                    const float* __restrict__ scale,
                                                    unsigned long long* __restrict__ zero_count,
                                                    unsigned long long* __restrict__ clipped_count,
                                                    int rows_per_block) {
  extern __shared__ u32 diag_lds[];              // [G] zero codes, [G] clipped
  const int b = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < 2 * G; i += 256) diag_lds[i] = 0;
  __syncthreads();
  const int row0 = blockIdx.x * rows_per_block;
  int nrows = T_ - row0;
  nrows = nrows < rows_per_block ? nrows : rows_per_block;
  for (int rr = wave; rr < nrows; rr += 4) {     // one wavefront per row
    const long long row = (long long)b * T_ + row0 + rr;
    const int g = gid ? gid[row] : 0;
    const float c = clip[(long long)b * G + g];
    const float d = scale[(long long)b * G + g];
    const float rcp = 1.0f / d;
    const T* xp = X + row * ld;
    u32 nz = 0, nc = 0;
    for (int ch = lane; ch < C; ch += 64) {
      const float x = Elem<T>::val(xp[ch]);
      nz += quant_nibble(x, c, d, rcp) == 0u ? 1u : 0u;
      nc += fabsf(x) > c ? 1u : 0u;
    }
    nz = group_sum_u32<64>(nz);
    nc = group_sum_u32<64>(nc);
    if (lane == 63) {
      atomicAdd(&diag_lds[g], nz);
      atomicAdd(&diag_lds[G + g], nc);
    }
  }
  __syncthreads();
  for (int g = tid; g < G; g += 256) {
    if (diag_lds[g]) atomicAdd(&zero_count[(long long)b * G + g], (unsigned long long)diag_lds[g]);
    if (diag_lds[G + g])
      atomicAdd(&clipped_count[(long long)b * G + g], (unsigned long long)diag_lds[G + g]);
  }
}

__global__ __launch_bounds__(256) void k_zero_u64(unsigned long long* __restrict__ a,
                                                  unsigned long long* __restrict__ b2, long long n) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i < n) {
    a[i] = 0;
    b2[i] = 0;
  }
}

hipError_t launch_group_diag(const void* X, tdq_dtype dt, int B, int T, int C, long long ld, int G,
                             const int* gid, const float* clip, const float* scale,
                             unsigned long long* zero_count, unsigned long long* clipped_count,
                             hipStream_t st) {
  const long long total = (long long)B * G;
  hipLaunchKernelGGL(k_zero_u64, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, zero_count,
                     clipped_count, total);
  // a workgroup's counters are 32-bit: at most 2^31 elements per workgroup
  long long rpb = (1ll << 20) / (C > 0 ? C : 1);
  rpb = rpb < 4 ? 4 : rpb;
  if (rpb * C >= (1ll << 31)) rpb = ((1ll << 31) - 1) / C;
  if (rpb < 1) rpb = 1;
  if (rpb > T) rpb = T;
  const unsigned chunks = (unsigned)((T + rpb - 1) / rpb);
  const size_t lds = (size_t)2 * G * sizeof(u32);
  if (dt == TDQ_F16)
    hipLaunchKernelGGL((k_group_diag<u16>), dim3(chunks, B), dim3(256), lds, st,
                       static_cast<const u16*>(X), ld, T, C, G, gid, clip, scale, zero_count,
                       clipped_count, (int)rpb);
  else
    hipLaunchKernelGGL((k_group_diag<float>), dim3(chunks, B), dim3(256), lds, st,
                       static_cast<const float*>(X), ld, T, C, G, gid, clip, scale, zero_count,
                       clipped_count, (int)rpb);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Range disparity D(X) = max |x| / median_t median_c |x| (Eq. range_disparity), per
// image.  Medians are lower medians, the ceil(n/2)-th smallest (the rank rule
// k = ceil(p n) at p = 1/2), found exactly by a radix select on the magnitude bit
// patterns: k_row_median, a wavefront per token over its C channels; k_image_disparity,
// a workgroup per image over its T token medians.
// ---------------------------------------------------------------------------
// One step of a radix select by the lanes of ONE wavefront on a 256-bin LDS histogram
// (already filled): finds the digit where the running count first reaches k_rem,
// returns it in every lane and lowers k_rem by the count below it.
__device__ __forceinline__ u32 wave_pick_digit(const u32* h, long long& k_rem) {
  const int lane = threadIdx.x & 63;
  const uint4 hb = *reinterpret_cast<const uint4*>(&h[4 * lane]);
  const u32 c4[4] = {hb.x, hb.y, hb.z, hb.w};
  const long long mine = (long long)c4[0] + c4[1] + c4[2] + c4[3];
  long long incl = mine;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const long long o = __shfl_up(incl, d, 64);
    if (lane >= d) incl += o;
  }
  const unsigned long long reached = __ballot(incl >= k_rem);
  const int first = reached ? __ffsll((long long)reached) - 1 : 63;
  long long below = incl - mine;
  int j = 0;
  for (; j < 3; ++j) {
    if (below + (long long)c4[j] >= k_rem) break;
    below += (long long)c4[j];
  }
  const u32 digit = (u32)__shfl((int)(4 * lane + j), first, 64);
  below = __shfl(below, first, 64);
  k_rem -= below;
  return digit;
}

template <typename T>
__global__ __launch_bounds__(256) void k_row_median(const T* __restrict__ X, long long ld, int M, int C,
                                                    float* __restrict__ med, float* __restrict__ rmax) {
  constexpr bool F16 = sizeof(T) == 2;
  constexpr int kLevels = F16 ? 2 : 4;
  constexpr int kBits = F16 ? 15 : 31;
  __shared__ __attribute__((aligned(16))) u32 hist[4][256];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const long long row_raw = (long long)blockIdx.x * 4 + wave;
  const bool valid = row_raw < M;                  // a wavefront without a row works on the last one
  const T* xp = X + (valid ? row_raw : (long long)(M - 1)) * ld;
  u32* h = hist[wave];
  long long k_rem = ((long long)C + 1) / 2;
  u32 prefix = 0, kmax = 0;
#pragma unroll 1
  for (int lev = 0; lev < kLevels; ++lev) {
    const int done = 8 * lev;
    const int bits = (lev == kLevels - 1) ? 7 : 8;
    const int shift = kBits - done - bits;
#pragma unroll
    for (int i = 0; i < 4; ++i) h[lane + 64 * i] = 0;
    __syncthreads();
    for (int c = lane; c < C; c += 64) {
      const u32 key = Elem<T>::key(xp[c]);
      if (lev == 0) kmax = key > kmax ? key : kmax;
      if (done == 0 || (key >> (kBits - done)) == prefix)
        atomicAdd(&h[(key >> shift) & ((1u << bits) - 1u)], 1u);
    }
    __syncthreads();
    const u32 digit = wave_pick_digit(h, k_rem);
    prefix = (prefix << bits) | digit;
    __syncthreads();
  }
  kmax = xor_reduce_max<64>(kmax);
  if (lane == 0 && valid) {
    med[row_raw] = Elem<T>::key_to_float(prefix);
    rmax[row_raw] = Elem<T>::key_to_float(kmax);
  }
}

// med, rmax [B*T] hold non-negative floats: their bit patterns order like the values.
__global__ __launch_bounds__(256) void k_image_disparity(const float* __restrict__ med,
                                                         const float* __restrict__ rmax, int T,
                                                         float* __restrict__ disparity,
                                                         float* __restrict__ max_abs) {
  __shared__ __attribute__((aligned(16))) u32 hist[256];
  __shared__ u32 s_max[4], s_digit;
  __shared__ long long s_krem;
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* mb = med + (long long)b * T;
  const float* rb = rmax + (long long)b * T;
  u32 kmax = 0;
  for (int t = tid; t < T; t += 256) {
    const u32 k = __float_as_uint(rb[t]);
    kmax = k > kmax ? k : kmax;
  }
  kmax = xor_reduce_max<64>(kmax);
  if (lane == 0) s_max[wave] = kmax;
  if (tid == 0) s_krem = ((long long)T + 1) / 2;
  u32 prefix = 0;
#pragma unroll 1
  for (int lev = 0; lev < 4; ++lev) {
    const int done = 8 * lev;
    const int bits = lev == 3 ? 7 : 8;
    const int shift = 31 - done - bits;
    hist[tid] = 0;
    __syncthreads();
    for (int t = tid; t < T; t += 256) {
      const u32 key = __float_as_uint(mb[t]) & 0x7FFFFFFFu;
      if (done == 0 || (key >> (31 - done)) == prefix)
        atomicAdd(&hist[(key >> shift) & ((1u << bits) - 1u)], 1u);
    }
    __syncthreads();
    if (wave == 0) {
      long long k_rem = s_krem;
      const u32 digit = wave_pick_digit(hist, k_rem);
      if (lane == 0) { s_digit = digit; s_krem = k_rem; }
    }
    __syncthreads();
    prefix = (prefix << bits) | s_digit;
    __syncthreads();
  }
  if (tid == 0) {
    u32 k = s_max[0];
    for (int w = 1; w < 4; ++w) k = s_max[w] > k ? s_max[w] : k;
    const float mx = __uint_as_float(k), den = __uint_as_float(prefix);
    max_abs[b] = mx;
    disparity[b] = den > 0.f ? mx / den : __uint_as_float(0x7F800000u);
  }
}

hipError_t launch_range_disparity(const void* X, tdq_dtype dt, int B, int T, int C, long long ld,
                                  float* token_median, float* token_max, float* disparity,
                                  float* max_abs, hipStream_t st) {
  const long long M = (long long)B * T;
  const unsigned grid = (unsigned)((M + 3) / 4);
  if (dt == TDQ_F16)
    hipLaunchKernelGGL((k_row_median<u16>), dim3(grid), dim3(256), 0, st, static_cast<const u16*>(X),
                       ld, (int)M, C, token_median, token_max);
  else
    hipLaunchKernelGGL((k_row_median<float>), dim3(grid), dim3(256), 0, st,
                       static_cast<const float*>(X), ld, (int)M, C, token_median, token_max);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_image_disparity, dim3(B), dim3(256), 0, st, token_median, token_max, T,
                     disparity, max_abs);
  return hipGetLastError();
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
