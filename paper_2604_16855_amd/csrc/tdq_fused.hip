// Single-launch form of the activation path for shapes where launch latency, not
// bandwidth, sets the time (a few hundred kilobytes per image): what tdq_calibrate_groups
// followed by tdq_quantize_act compute, in ONE kernel, one workgroup of 1024 threads per
// image, the steps separated by workgroup barriers instead of kernel boundaries:
//   A  per-token range, mean and centred second moment  (Sec. 4.2)
//   B  token -> token set, per-set sums                 (assign_tokens)
//   C  per set: n, sigma, rank k                        (merge_partials)
//   D  k-th smallest |x| of every set: radix select on the magnitude bit pattern, 8 bits
//      per level, LDS histogram [G][256]                (Eq. zr_constraint, exact)
//   E  projection                                       (Eq. dcrp)
//   F  quantize + pack                                  (Eqs. clipx, dequant)
// X is read once per step that needs it (A, every level of D, F) and comes from the
// cache after the first.  Same arithmetic as the multi-kernel path wherever a result is
// rounded: group ids, thresholds and codes are integer work, sigma is binary64.
#include "tdq_device.hpp"

namespace tdq {

constexpr int kFusedThreads = 1024;
constexpr int kFusedMaxG = TDQ_FUSED_MAX_GROUPS;

template <typename T>
__global__ __launch_bounds__(kFusedThreads) void k_fused_small(
    const T* __restrict__ X, long long ld, int T_, int C, int G, int L, int vec_ok, int q_vec_ok,
    Scalars sc, int with_base, float* __restrict__ r, double* __restrict__ mean,
    double* __restrict__ m2, int* __restrict__ gid, float* __restrict__ clip,
    float* __restrict__ scale, tdq_group_stats* __restrict__ stats, u32* __restrict__ image_flags,
    uint8_t* __restrict__ Q, long long ld_q) {
  constexpr int V = Elem<T>::V;
  constexpr bool F16 = sizeof(T) == 2;
  constexpr int NW = kFusedThreads / 64;
  constexpr int kLevels = F16 ? 2 : 4;
  __shared__ SetAcc wacc[NW * kFusedMaxG];
  __shared__ u32 hist[kFusedMaxG * 256];
  __shared__ GroupWork grp[kFusedMaxG];
  __shared__ u32 s_min[NW], s_max[NW], s_lohi[2];

  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  const int lr = tid & (L - 1);                  // lane of the row group (L a power of two)
  const int rsub = tid / L, rpp = kFusedThreads / L;
  const T* Xb = X + (long long)b * T_ * ld;
  float* rb = r + (long long)b * T_;
  double* meanb = mean + (long long)b * T_;
  double* m2b = m2 + (long long)b * T_;
  int* gb = gid + (long long)b * T_;
  const int nvec = vec_ok ? C / V : 0;

  // ---- A: rows are shared out to groups of L lanes; every lane runs every pass (the
  // reductions are lane exchanges), rows past the end are clamped and not stored
  for (int row0 = 0; row0 < T_; row0 += rpp) {
    const int row = row0 + rsub;
    const bool valid = row < T_;
    const T* xp = Xb + (long long)(valid ? row : T_ - 1) * ld;
    u32 kmax = 0;
    double a1 = 0.0, a2 = 0.0;
    // binary64 sums about the row's first value (any value of the row is a good enough
    // pivot in binary64; see "Moments" in tdq_device.hpp)
    const double P = (double)Elem<T>::val(xp[0]);
    for (int v = lr; v < nvec; v += L) {
      const uint4 q = *reinterpret_cast<const uint4*>(xp + (long long)v * V);
      T e[V];
      Elem<T>::unpack(q, e);
#pragma unroll
      for (int i = 0; i < V; ++i) {
        const double d = (double)Elem<T>::val(e[i]) - P;
        const u32 k = Elem<T>::key(e[i]);
        kmax = k > kmax ? k : kmax;
        a1 += d;
        a2 = fma(d, d, a2);
      }
    }
    for (int c = nvec * V + lr; c < C; c += L) {
      const T x = xp[c];
      const double d = (double)Elem<T>::val(x) - P;
      const u32 k = Elem<T>::key(x);
      kmax = k > kmax ? k : kmax;
      a1 += d;
      a2 = fma(d, d, a2);
    }
    for (int m = L >> 1; m > 0; m >>= 1) {       // butterfly: all L lanes end with the same bits
      const u32 ok = (u32)__shfl_xor((int)kmax, m, 64);
      kmax = ok > kmax ? ok : kmax;
      a1 += __shfl_xor(a1, m, 64);
      a2 += __shfl_xor(a2, m, 64);
    }
    if (lr == 0 && valid) {
      double mu, q;
      pivot_to_central(P, a1, a2, 1.0 / (double)C, mu, q);
      rb[row] = Elem<T>::key_to_float(kmax);
      meanb[row] = mu;
      m2b[row] = q;
    }
  }
  __syncthreads();                               // the workgroup's global writes are visible to it

  // ---- B
  assign_tokens(rb, meanb, m2b, T_, C, G, gb, wacc, s_min, s_max, s_lohi, 0, 1);
  if (tid == 0 && image_flags) image_flags[b] = s_lohi[1] >= 0x7F800000u ? TDQ_DEV_NONFINITE : 0u;

  // one rank select per rank wanted: the percentile base radius first (if asked for)
  for (int pass = with_base ? kPassBase : kPassZr; pass >= kPassZr; --pass) {
    // ---- C
    if (tid < G) {
      GroupWork w = merge_partials(wacc, 0, tid, NW, G, C, sc, pass);
      if (pass == kPassZr && with_base) w.c_base = grp[tid].c_base;
      grp[tid] = w;
    }
    // ---- D
#pragma unroll 1
    for (int lev = 0; lev < kLevels; ++lev) {
      const int bits = (F16 && lev == 1) ? 7 : ((!F16 && lev == 3) ? 7 : 8);
      const int done = 8 * lev;                                  // key bits fixed so far
      const int total_bits = F16 ? 15 : 31;
      const int shift = total_bits - done - bits;                // bits below this level's digit
      for (int i = tid; i < G * 256; i += kFusedThreads) hist[i] = 0;
      __syncthreads();
      for (int row = rsub; row < T_; row += rpp) {
        const T* xp = Xb + (long long)row * ld;
        const int g = gb[row];
        const u32 want = grp[g].prefix;                          // the `done` high bits
        u32* h = hist + g * 256;
        auto count = [&](u32 key) {
          if (done == 0 || (key >> (total_bits - done)) == want)
            atomicAdd(&h[(key >> shift) & ((1u << bits) - 1u)], 1u);
        };
        for (int v = lr; v < nvec; v += L) {
          const uint4 q = *reinterpret_cast<const uint4*>(xp + (long long)v * V);
          T e[V];
          Elem<T>::unpack(q, e);
#pragma unroll
          for (int i = 0; i < V; ++i) count(Elem<T>::key(e[i]));
        }
        for (int c = nvec * V + lr; c < C; c += L) count(Elem<T>::key(xp[c]));
      }
      __syncthreads();
      // a wavefront per set: every lane takes 4 consecutive bins, the running count
      // over the lanes finds the lane, then the bin, where it first reaches the rank
      for (int g = tid >> 6; g < G; g += NW) {
        const GroupWork w = grp[g];
        if (w.tokens == 0) continue;                               // uniform over the wavefront
        const int lane = tid & 63;
        const uint4 hb = *reinterpret_cast<const uint4*>(&hist[g * 256 + 4 * lane]);
        const u32 c4[4] = {hb.x, hb.y, hb.z, hb.w};
        const bool in_range = 4 * lane < (1 << bits);
        long long mine = in_range ? (long long)c4[0] + c4[1] + c4[2] + c4[3] : 0;
        long long incl = mine;                                     // inclusive scan over the lanes
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
          const long long o = __shfl_up(incl, d, 64);
          if (lane >= d) incl += o;
        }
        const unsigned long long reached = __ballot(incl >= w.k_rem);
        // the ranks never exceed the count of the set's elements under the prefix
        const int first = reached ? __ffsll((long long)reached) - 1 : 63;
        if (lane == first) {
          long long below = incl - mine;
          int j = 0;
          for (; j < 3; ++j) {
            if (below + (long long)c4[j] >= w.k_rem) break;
            below += (long long)c4[j];
          }
          GroupWork nw = w;
          nw.k_rem = w.k_rem - below;
          nw.prefix = (w.prefix << bits) | (u32)(4 * lane + j);
          grp[g] = nw;
        }
      }
      __syncthreads();
    }
    // ---- E
    if (tid < G) {
      const GroupWork w = grp[tid];
      if (pass == kPassBase) {
        if (w.tokens != 0) grp[tid].c_base = Elem<T>::key_to_float(w.prefix);
      } else {
        project_store(b * G + tid, w, w.prefix, F16, sc, clip, scale, stats);
      }
    }
    __syncthreads();
  }

  // ---- F
  const int n8 = (vec_ok && q_vec_ok) ? C / 8 : 0;               // units of 8 elements -> 4 bytes
  const int nbytes = (C + 1) / 2;
  for (int row = rsub; row < T_; row += rpp) {
    const T* xp = Xb + (long long)row * ld;
    uint8_t* qp = Q + ((long long)b * T_ + row) * ld_q;
    const int g = gb[row];
    const float c = clip[b * G + g], d = scale[b * G + g];
    const float rcp = 1.0f / d;
    for (int u = lr; u < n8; u += L) {
      u32 word = 0;
#pragma unroll
      for (int j = 0; j < 8 / V; ++j) {
        const uint4 q = *reinterpret_cast<const uint4*>(xp + (long long)u * 8 + j * V);
        T e[V];
        Elem<T>::unpack(q, e);
#pragma unroll
        for (int i = 0; i < V; ++i)
          word |= quant_nibble(Elem<T>::val(e[i]), c, d, rcp) << (4 * (j * V + i));
      }
      *reinterpret_cast<u32*>(qp + (long long)u * 4) = word;
    }
    for (int by = n8 * 4 + lr; by < nbytes; by += L) {
      const int c0 = 2 * by;
      u32 v = quant_nibble(Elem<T>::val(xp[c0]), c, d, rcp);
      if (c0 + 1 < C) v |= quant_nibble(Elem<T>::val(xp[c0 + 1]), c, d, rcp) << 4;
      qp[by] = (uint8_t)v;
    }
  }
}

template <typename T>
static hipError_t fused_t(const T* X, int B, int T_, int C, long long ld, int G, const Scalars& sc,
                          float* r, double* mean, double* m2, int* gid, float* clip, float* scale,
                          tdq_group_stats* stats, unsigned* image_flags, uint8_t* Q, long long ld_q,
                          hipStream_t st) {
  constexpr int V = Elem<T>::V;
  const int vec_ok = ((reinterpret_cast<uintptr_t>(X) & 15) == 0 && ld % V == 0) ? 1 : 0;
  const int q_vec_ok = ((reinterpret_cast<uintptr_t>(Q) & 3) == 0 && ld_q % 4 == 0) ? 1 : 0;
  const int L = lanes_per_row(C, 8);
  const int with_base = sc.base_pct > 0.0 ? 1 : 0;
  hipLaunchKernelGGL((k_fused_small<T>), dim3(B), dim3(kFusedThreads), 0, st, X, ld, T_, C, G, L,
                     vec_ok, q_vec_ok, sc, with_base, r, mean, m2, gid, clip, scale, stats, image_flags,
                     Q, ld_q);
  return hipGetLastError();
}

hipError_t launch_fused_small(const void* X, tdq_dtype dt, int B, int T, int C, long long ld, int G,
                              const Scalars& sc, float* r, double* mean, double* m2, int* gid,
                              float* clip, float* scale, tdq_group_stats* stats,
                              unsigned* image_flags, uint8_t* Q, long long ld_q, hipStream_t st) {
  if (dt == TDQ_F16)
    return fused_t<u16>(static_cast<const u16*>(X), B, T, C, ld, G, sc, r, mean, m2, gid, clip, scale,
                        stats, image_flags, Q, ld_q, st);
  return fused_t<float>(static_cast<const float*>(X), B, T, C, ld, G, sc, r, mean, m2, gid, clip, scale,
                        stats, image_flags, Q, ld_q, st);
}

}  // namespace tdq
