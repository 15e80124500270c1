// Convolutional feature maps as tokens (Supp. "Implementation details": the dynamic
// activation path maps X[B, C, H, W] to X'[B, HW, C] and applies DSTG + DCRP along the
// channel dimension): an exact re-layout X[b, c, t] -> Xt[b * T + t, c], t = h * W + w,
// after which every token-major entry point applies.
//
// One workgroup moves a tile of 64 channels x TT tokens (TT = 128 for binary16, 64 for
// binary32) through LDS: 16-byte loads along the token axis (the contiguous one of the
// input), 16-byte stores along the channel axis (the contiguous one of the output), so
// both sides move whole 128-byte lines per 8 lanes.  The transposition is on the LDS
// read side: 8 (4) two- (four-) byte reads per 16-byte store; rows of the LDS tile are 8
// bytes longer than the data, which leaves those reads with two-way bank conflicts at
// most.
#include <type_traits>

#include "tdq_device.hpp"

namespace tdq {

template <typename T>
__global__ __launch_bounds__(256) void k_tokenize_chw(const T* __restrict__ X, long long ld_c,
                                                      long long ld_b, int C, int T_,
                                                      T* __restrict__ Xt, long long ld_xt, int vin_ok,
                                                      int vout_ok) {
  constexpr int E = 16 / (int)sizeof(T);     // elements per 16 bytes
  constexpr int TC = 64;                     // channels per tile
  constexpr int TT = 16 * E;                 // tokens per tile
  constexpr int PITCH = TT + 8 / (int)sizeof(T);
  constexpr int PQ = TC / E;                 // 16-byte pieces per token row of the tile
  __shared__ __attribute__((aligned(16))) T tile[TC][PITCH];

  const int t0 = blockIdx.x * TT, c0 = blockIdx.y * TC, b = blockIdx.z;
  const int tid = threadIdx.x;
  const T* xb = X + (long long)b * ld_b;

  // in: thread t owns the piece t % 16 (E tokens) of channels t / 16 + 16 i
  {
    const int p = tid & 15;
    const int tok = t0 + p * E;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int ch = (tid >> 4) + 16 * i;
      const int c = c0 + ch;
      __attribute__((aligned(16))) T v[E];
      if (c < C && vin_ok && tok + E <= T_) {
        const uint4 q = *reinterpret_cast<const uint4*>(xb + (long long)c * ld_c + tok);
        *reinterpret_cast<uint4*>(v) = q;
      } else {
#pragma unroll
        for (int k = 0; k < E; ++k)
          v[k] = (c < C && tok + k < T_) ? xb[(long long)c * ld_c + tok + k] : (T)0;
      }
      // rows are 8 bytes apart from a multiple of 16: two 8-byte writes
      uint2* d = reinterpret_cast<uint2*>(&tile[ch][p * E]);
      const uint2* s = reinterpret_cast<const uint2*>(v);
      d[0] = s[0];
      d[1] = s[1];
    }
  }
  __syncthreads();
  // out: thread t owns the piece t % PQ (E channels) of tokens t / PQ + (256 / PQ) i
  {
    const int q = tid % PQ;
    const int c = c0 + q * E;
    constexpr int TPP = 256 / PQ;            // tokens per pass
#pragma unroll
    for (int i = 0; i < TT / TPP; ++i) {
      const int tl = tid / PQ + TPP * i;
      const int tok = t0 + tl;
      if (tok >= T_) continue;
      __attribute__((aligned(16))) T v[E];
#pragma unroll
      for (int k = 0; k < E; ++k) v[k] = tile[q * E + k][tl];
      T* dst = Xt + ((long long)b * T_ + tok) * ld_xt + c;
      if (vout_ok && c + E <= C) {
        *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(v);
      } else {
#pragma unroll
        for (int k = 0; k < E; ++k)
          if (c + k < C) dst[k] = v[k];
      }
    }
  }
}

template <typename T>
static hipError_t tokenize_t(const T* X, int B, int C, int T_, long long ld_c, long long ld_b, T* Xt,
                             long long ld_xt, hipStream_t st) {
  constexpr int E = 16 / (int)sizeof(T);
  const int vin_ok =
      ((reinterpret_cast<uintptr_t>(X) & 15) == 0 && ld_c % E == 0 && ld_b % E == 0) ? 1 : 0;
  const int vout_ok = ((reinterpret_cast<uintptr_t>(Xt) & 15) == 0 && ld_xt % E == 0) ? 1 : 0;
  const dim3 grid((unsigned)((T_ + 16 * E - 1) / (16 * E)), (unsigned)((C + 63) / 64), (unsigned)B);
  hipLaunchKernelGGL((k_tokenize_chw<T>), grid, dim3(256), 0, st, X, ld_c, ld_b, C, T_, Xt, ld_xt,
                     vin_ok, vout_ok);
  return hipGetLastError();
}

hipError_t launch_tokenize_chw(const void* X, tdq_dtype dt, int B, int C, int T, long long ld_c,
                               long long ld_b, void* Xt, long long ld_xt, hipStream_t st) {
  if (dt == TDQ_F16)
    return tokenize_t<u16>(static_cast<const u16*>(X), B, C, T, ld_c, ld_b, static_cast<u16*>(Xt),
                           ld_xt, st);
  return tokenize_t<float>(static_cast<const float*>(X), B, C, T, ld_c, ld_b,
                           static_cast<float*>(Xt), ld_xt, st);
}

// ---------------------------------------------------------------------------
// The re-layout fused with the statistics sweep of the token-set path: one read of the
// feature map yields the token-major copy Xt AND every token's range and moments
// (r_t = max_c |x|, mean_t, M2_t = sum_c (x - mean_t)^2; Sec. 4.2), so a convolutional input costs
// the token-set path one extra write of X, not an extra read and write.  A workgroup
// owns TT consecutive tokens of one image and walks the channel axis in tiles of 64:
// every thread keeps the partial statistics of its 4 tokens across the tiles; at the end
// the lanes that share a token (adjacent ones) are reduced with DPP.  The sums are taken
// about a per-token pivot taken from the first tile, see "Moments" in tdq_device.hpp:
// binary32 input, the token's first channel; binary16 input, the mean of its first
// min(C, 64) channels.  The map is read once, so a token cannot be summed again about a
// better pivot as in the token-major sweep; the mean of 64 of its values lies within
// sigma_t sqrt(C / 64) of the token's mean (Cauchy-Schwarz), which bounds what the
// binary32 partial sums can cost its M2 at (1 + C / 64) * 3 * 2^-24 per partial.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_tokenize_stats_chw(
    const T* __restrict__ X, long long ld_c, long long ld_b, int C, int T_, T* __restrict__ Xt,
    long long ld_xt, int vin_ok, int vout_ok, float* __restrict__ r, double* __restrict__ mean,
    double* __restrict__ m2) {
  constexpr int E = 16 / (int)sizeof(T);
  constexpr int TC = 64;
  constexpr int TT = 16 * E;
  constexpr int PITCH = TT + 8 / (int)sizeof(T);
  constexpr int PQ = TC / E;                 // lanes per token
  constexpr int TPP = 256 / PQ;              // tokens per pass
  constexpr int NP = TT / TPP;               // passes = tokens per thread (4)
  __shared__ __attribute__((aligned(16))) T tile[TC][PITCH];

  const int t0 = blockIdx.x * TT, b = blockIdx.y;
  const int tid = threadIdx.x;
  const T* xb = X + (long long)b * ld_b;
  const int q = tid % PQ;
  u32 kmax[NP];
  double a1[NP], a2[NP];
  typedef typename std::conditional<sizeof(T) == 2, float, double>::type PT;
  PT P[NP];
#pragma unroll
  for (int i = 0; i < NP; ++i) { kmax[i] = 0; a1[i] = 0.0; a2[i] = 0.0; P[i] = 0; }

  // the next tile's global loads are in flight while the current one is processed
  const int lp = tid & 15, ltok = t0 + (tid & 15) * E;
  uint4 stage[4];
  auto load_tile = [&](int c0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = c0 + (tid >> 4) + 16 * i;
      if (c < C && vin_ok && ltok + E <= T_) {
        stage[i] = *reinterpret_cast<const uint4*>(xb + (long long)c * ld_c + ltok);
      } else {
        __attribute__((aligned(16))) T v[E];
#pragma unroll
        for (int k = 0; k < E; ++k)
          v[k] = (c < C && ltok + k < T_) ? xb[(long long)c * ld_c + ltok + k] : (T)0;
        stage[i] = *reinterpret_cast<const uint4*>(v);
      }
    }
  };
  load_tile(0);
  for (int c0 = 0; c0 < C; c0 += TC) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint2* d = reinterpret_cast<uint2*>(&tile[(tid >> 4) + 16 * i][lp * E]);
      d[0] = make_uint2(stage[i].x, stage[i].y);
      d[1] = make_uint2(stage[i].z, stage[i].w);
    }
    __syncthreads();
    if (c0 + TC < C) load_tile(c0 + TC);
    const int c = c0 + q * E;
    if (c0 == 0) {                               // the tokens' pivots, from the first tile
#pragma unroll
      for (int i = 0; i < NP; ++i) {
        const int tl = tid / PQ + TPP * i;
        if constexpr (sizeof(T) == 2) {
          float sum = 0.f;                       // channels past C are zeros in the tile
#pragma unroll
          for (int k = 0; k < E; ++k) sum += Elem<T>::val(tile[q * E + k][tl]);
          sum = xor_reduce_sum<PQ, float>(sum);  // the same bits in all lanes of the token
          P[i] = sum / (float)(C < TC ? C : TC);
        } else {
          P[i] = (double)Elem<T>::val(tile[0][tl]);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int tl = tid / PQ + TPP * i;
      const int tok = t0 + tl;
      __attribute__((aligned(16))) T v[E];
#pragma unroll
      for (int k = 0; k < E; ++k) v[k] = tile[q * E + k][tl];
      // channels beyond C are zeros in the tile: they do not change the maximum, and are
      // kept out of the sums
      if constexpr (sizeof(T) == 2) {
        // as in the token-major statistics sweep: the 8 differences and their squares are
        // first summed in binary32, then accumulated in binary64
        float p1 = 0.f, p2 = 0.f;
#pragma unroll
        for (int k = 0; k < E; ++k) {
          const float f = Elem<T>::val(v[k]);
          const u32 key = Elem<T>::key(v[k]);
          kmax[i] = key > kmax[i] ? key : kmax[i];
          const float d = c + k < C ? f - P[i] : 0.f;
          p1 += d;
          p2 = __builtin_fmaf(d, d, p2);
        }
        a1[i] += (double)p1;
        a2[i] += (double)p2;
      } else {
#pragma unroll
        for (int k = 0; k < E; ++k) {
          const double f = (double)Elem<T>::val(v[k]);
          const u32 key = Elem<T>::key(v[k]);
          kmax[i] = key > kmax[i] ? key : kmax[i];
          const double d = c + k < C ? f - P[i] : 0.0;
          a1[i] += d;
          a2[i] = fma(d, d, a2[i]);
        }
      }
      if (tok < T_) {
        T* dst = Xt + ((long long)b * T_ + tok) * ld_xt + c;
        if (vout_ok && c + E <= C) {
          *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(v);
        } else {
#pragma unroll
          for (int k = 0; k < E; ++k)
            if (c + k < C) dst[k] = v[k];
        }
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < NP; ++i) {
    const u32 km = group_max_u32<PQ>(kmax[i]);
    const double t1 = group_sum_f64<PQ>(a1[i]);
    const double t2 = group_sum_f64<PQ>(a2[i]);
    const int tok = t0 + tid / PQ + TPP * i;
    if (q == PQ - 1 && tok < T_) {               // the group's last lane holds the totals
      const long long row = (long long)b * T_ + tok;
      double mu, qq;
      pivot_to_central((double)P[i], t1, t2, 1.0 / (double)C, mu, qq);
      r[row] = Elem<T>::key_to_float(km);
      mean[row] = mu;
      m2[row] = qq;
    }
  }
}

template <typename T>
static hipError_t tokenize_stats_t(const T* X, int B, int C, int T_, long long ld_c, long long ld_b,
                                   T* Xt, long long ld_xt, float* r, double* mean, double* m2,
                                   hipStream_t st) {
  constexpr int E = 16 / (int)sizeof(T);
  const int vin_ok =
      ((reinterpret_cast<uintptr_t>(X) & 15) == 0 && ld_c % E == 0 && ld_b % E == 0) ? 1 : 0;
  const int vout_ok = ((reinterpret_cast<uintptr_t>(Xt) & 15) == 0 && ld_xt % E == 0) ? 1 : 0;
  const dim3 grid((unsigned)((T_ + 16 * E - 1) / (16 * E)), (unsigned)B);
  hipLaunchKernelGGL((k_tokenize_stats_chw<T>), grid, dim3(256), 0, st, X, ld_c, ld_b, C, T_, Xt,
                     ld_xt, vin_ok, vout_ok, r, mean, m2);
  return hipGetLastError();
}

hipError_t launch_tokenize_stats_chw(const void* X, tdq_dtype dt, int B, int C, int T, long long ld_c,
                                     long long ld_b, void* Xt, long long ld_xt, float* r, double* mean,
                                     double* m2, hipStream_t st) {
  if (dt == TDQ_F16)
    return tokenize_stats_t<u16>(static_cast<const u16*>(X), B, C, T, ld_c, ld_b,
                                 static_cast<u16*>(Xt), ld_xt, r, mean, m2, st);
  return tokenize_stats_t<float>(static_cast<const float*>(X), B, C, T, ld_c, ld_b,
                                 static_cast<float*>(Xt), ld_xt, r, mean, m2, st);
}

}  // namespace tdq
