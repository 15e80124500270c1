// W4A4 contraction on the int8 matrix cores of gfx950 with the dequantizing
// epilogue (Supp. Algorithm 1, step 10, written on the integer codes):
//   acc[m, n] = sum_i Qx[m, i] * Qw[n, i]            (int32, exact)
//   Y[m, n]   = (float(acc) * Delta[row m]) * s_w[n] (+ bias[n])
//
// Both operands arrive as packed two's-complement nibbles, K-contiguous.  The
// packed bytes are staged through LDS as they are (half the LDS traffic of int8)
// and expanded in registers: for a 32-bit word w of eight nibbles,
//   (w << 4) & 0xF0F0F0F0  holds the even elements and  w & 0xF0F0F0F0  the odd
// ones, each as an int8 equal to 16 * code (the sign lands in the byte's top bit
// for free).  Both operands carry the factor 16, so the int32 accumulator is
// 256 * acc and an arithmetic shift by 8 recovers acc exactly.  The order in
// which the K elements meet inside the matrix instruction is irrelevant as long
// as both operands use the same one, which they do by construction.
#include "tdq_internal.hpp"

namespace tdq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned int u32;

constexpr int BM = 128;          // rows of Y per workgroup
constexpr int BN = 128;          // columns of Y per workgroup
constexpr int BKB = 64;          // packed bytes of K per stage (128 codes)
constexpr int LDS_STRIDE = BKB + 16;   // +16 B pad: 16-byte reads of 8 rows hit 8 different bank groups
constexpr int GEMM_THREADS = 256;      // 4 wavefronts, 2 x 2, each 64 x 64 of Y
constexpr int XCDS = 8;

// Two packed words (16 codes) -> the four operand registers of one matrix instruction.
__device__ __forceinline__ v4i expand(u32 w0, u32 w1) {
  v4i r;
  r[0] = (int)((w0 << 4) & 0xF0F0F0F0u);   // even codes of w0, times 16
  r[1] = (int)(w0 & 0xF0F0F0F0u);          // odd codes of w0, times 16
  r[2] = (int)((w1 << 4) & 0xF0F0F0F0u);
  r[3] = (int)(w1 & 0xF0F0F0F0u);
  return r;
}

// Keeps the first `keep` (1..15) bytes of a 16-byte piece and zeroes the rest.
__device__ __forceinline__ u32 tail_mask(int keep, int lo) {
  return keep >= lo + 4 ? 0xFFFFFFFFu : keep <= lo ? 0u : (0xFFFFFFFFu >> (8 * (lo + 4 - keep)));
}
__device__ __forceinline__ void mask_piece(uint4& q, int keep) {
  q.x &= tail_mask(keep, 0);
  q.y &= tail_mask(keep, 4);
  q.z &= tail_mask(keep, 8);
  q.w &= tail_mask(keep, 12);
}

template <typename OUT>
__device__ __forceinline__ void store_out(OUT* p, float v);
template <>
__device__ __forceinline__ void store_out<float>(float* p, float v) { *p = v; }
template <>
__device__ __forceinline__ void store_out<_Float16>(_Float16* p, float v) { *p = (_Float16)v; }

template <typename OUT>
__global__ __launch_bounds__(GEMM_THREADS) void k_w4a4_gemm(
    const uint8_t* __restrict__ Qx, long long ld_q, const int* __restrict__ gid,
    const float* __restrict__ scale, int M, int T, int K, int N, int G,
    const uint8_t* __restrict__ Qw, long long ld_w, const float* __restrict__ w_scale,
    const float* __restrict__ bias, OUT* __restrict__ Y, long long ld_y, int* __restrict__ acc_dump,
    int m_tiles, int n_tiles) {
  __shared__ __attribute__((aligned(16))) uint8_t sA[2][BM * LDS_STRIDE];
  __shared__ __attribute__((aligned(16))) uint8_t sB[2][BN * LDS_STRIDE];
  __shared__ float sRow[BM], sCol[BN], sBias[BN];

  // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2: give
  // every XCD whole rows of tiles so the activation tile it streams is reused by
  // consecutive workgroups of the same XCD.
  const int bid = blockIdx.x;
  const int xcd = bid % XCDS, idx = bid / XCDS;
  const int m_tile = (idx / n_tiles) * XCDS + xcd;
  const int n_tile = idx % n_tiles;
  if (m_tile >= m_tiles) return;
  const int m0 = m_tile * BM, n0 = n_tile * BN;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int kbytes = (K + 1) / 2;
  const int k_tiles = (kbytes + BKB - 1) / BKB;

  if (tid < BM) {
    const int m = m0 + tid;
    float rs = 0.f;
    if (m < M) {
      const int b = m / T;
      const int g = gid ? gid[m] : 0;
      rs = scale[(long long)b * G + g];
    }
    sRow[tid] = rs;
  } else {
    const int j = tid - BM;   // BM == BN == GEMM_THREADS / 2
    const int n = n0 + j;
    sCol[j] = n < N ? w_scale[n] : 0.f;
    sBias[j] = (bias && n < N) ? bias[n] : 0.f;
  }

  // global -> register staging: each stage is 128 rows x 64 B per operand =
  // 512 pieces of 16 B; a thread moves pieces tid and tid + 256 of A and of B.
  const int pr0 = tid >> 2, pc = (tid & 3) * 16;     // rows pr0 and pr0 + 64
  int ra0 = m0 + pr0, ra1 = m0 + pr0 + 64;
  ra0 = ra0 < M ? ra0 : M - 1;
  ra1 = ra1 < M ? ra1 : M - 1;
  int rb0 = n0 + pr0, rb1 = n0 + pr0 + 64;
  rb0 = rb0 < N ? rb0 : N - 1;
  rb1 = rb1 < N ? rb1 : N - 1;
  const uint8_t* pa0 = Qx + (long long)ra0 * ld_q + pc;
  const uint8_t* pa1 = Qx + (long long)ra1 * ld_q + pc;
  const uint8_t* pb0 = Qw + (long long)rb0 * ld_w + pc;
  const uint8_t* pb1 = Qw + (long long)rb1 * ld_w + pc;

  uint4 ga0, ga1, gb0, gb1;
  auto load_stage = [&](int kt) {
    const int kb = kt * BKB + pc;          // first packed byte of this piece
    const uint4 z = make_uint4(0, 0, 0, 0);
    if (kb < kbytes) {
      ga0 = *reinterpret_cast<const uint4*>(pa0 + (long long)kt * BKB);
      ga1 = *reinterpret_cast<const uint4*>(pa1 + (long long)kt * BKB);
      gb0 = *reinterpret_cast<const uint4*>(pb0 + (long long)kt * BKB);
      gb1 = *reinterpret_cast<const uint4*>(pb1 + (long long)kt * BKB);
      if (kb + 16 > kbytes) {              // piece straddles the end of the row: zero the rest
        const int keep = kbytes - kb;      // 1..15 bytes are real
        mask_piece(ga0, keep);
        mask_piece(ga1, keep);
        mask_piece(gb0, keep);
        mask_piece(gb1, keep);
      }
    } else {
      ga0 = ga1 = gb0 = gb1 = z;
    }
  };
  auto store_stage = [&](int buf) {
    *reinterpret_cast<uint4*>(&sA[buf][pr0 * LDS_STRIDE + pc]) = ga0;
    *reinterpret_cast<uint4*>(&sA[buf][(pr0 + 64) * LDS_STRIDE + pc]) = ga1;
    *reinterpret_cast<uint4*>(&sB[buf][pr0 * LDS_STRIDE + pc]) = gb0;
    *reinterpret_cast<uint4*>(&sB[buf][(pr0 + 64) * LDS_STRIDE + pc]) = gb1;
  };

  v16i acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  load_stage(0);
  store_stage(0);
  __syncthreads();

  // Lane l of a wavefront feeds row (l & 31) of a 32-row fragment and, of each
  // 32-byte slab (64 codes) of K, the 16 bytes at offset 16 * (l >> 5).
  const int frow = lane & 31, fhalf = (lane >> 5) * 16;
  for (int kt = 0; kt < k_tiles; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < k_tiles) load_stage(kt + 1);
#pragma unroll
    for (int ks = 0; ks < BKB / 32; ++ks) {
      uint4 fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i)
        fa[i] = *reinterpret_cast<const uint4*>(
            &sA[cur][(wm * 64 + i * 32 + frow) * LDS_STRIDE + ks * 32 + fhalf]);
#pragma unroll
      for (int j = 0; j < 2; ++j)
        fb[j] = *reinterpret_cast<const uint4*>(
            &sB[cur][(wn * 64 + j * 32 + frow) * LDS_STRIDE + ks * 32 + fhalf]);
      v4i a0[2], a1[2], b0[2], b1[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        a0[i] = expand(fa[i].x, fa[i].y);
        a1[i] = expand(fa[i].z, fa[i].w);
        b0[i] = expand(fb[i].x, fb[i].y);
        b1[i] = expand(fb[i].z, fb[i].w);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0[i], b0[j], acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1[i], b1[j], acc[i][j], 0, 0, 0);
        }
    }
    if (kt + 1 < k_tiles) store_stage(cur ^ 1);
    __syncthreads();
  }

  // Epilogue.  Register r of a 32x32 accumulator fragment held by lane l is
  // element (row 8*(r/4) + 4*(l/32) + r%4, column l%32).
  const int ccol = lane & 31, rquad = (lane >> 5) * 4;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int cl = wn * 64 + j * 32 + ccol;
      const int n = n0 + cl;
      const float ws = sCol[cl], bs = sBias[cl];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int rl = wm * 64 + i * 32 + (r >> 2) * 8 + rquad + (r & 3);
        const int m = m0 + rl;
        if (m < M && n < N) {
          const int a = acc[i][j][r] >> 8;            // exact: accumulator is 256 * acc
          if (acc_dump) acc_dump[(long long)m * N + n] = a;
          float y = ((float)a * sRow[rl]) * ws;
          if (bias) y = y + bs;
          store_out<OUT>(Y + (long long)m * ld_y + n, y);
        }
      }
    }
}

hipError_t launch_w4a4_gemm(const uint8_t* Qx, long long ld_q, const int* gid, const float* scale,
                            int M, int T, int K, int N, int G, const uint8_t* Qw, long long ld_w,
                            const float* w_scale, const float* bias, void* Y, tdq_dtype y_dt,
                            long long ld_y, int* acc_dump, hipStream_t st) {
  const int m_tiles = (M + BM - 1) / BM, n_tiles = (N + BN - 1) / BN;
  const long long m_groups = (m_tiles + XCDS - 1) / XCDS;
  const unsigned grid = (unsigned)(m_groups * XCDS * n_tiles);
  if (y_dt == TDQ_F32)
    hipLaunchKernelGGL((k_w4a4_gemm<float>), dim3(grid), dim3(GEMM_THREADS), 0, st, Qx, ld_q, gid,
                       scale, M, T, K, N, G, Qw, ld_w, w_scale, bias, static_cast<float*>(Y), ld_y,
                       acc_dump, m_tiles, n_tiles);
  else
    hipLaunchKernelGGL((k_w4a4_gemm<_Float16>), dim3(grid), dim3(GEMM_THREADS), 0, st, Qx, ld_q,
                       gid, scale, M, T, K, N, G, Qw, ld_w, w_scale, bias,
                       static_cast<_Float16*>(Y), ld_y, acc_dump, m_tiles, n_tiles);
  return hipGetLastError();
}

}  // namespace tdq
