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

}  // namespace tdq
