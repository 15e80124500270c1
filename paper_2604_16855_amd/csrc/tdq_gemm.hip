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
#include <stdlib.h>

#include <type_traits>

#include "tdq_internal.hpp"

namespace tdq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned int u32;

constexpr int BKB = 64;          // packed bytes of K per stage (128 codes)
constexpr int LDS_STRIDE = BKB + 16;   // +16 B pad: 16-byte reads of 8 rows hit 8 different bank groups
constexpr int GEMM_THREADS = 256;      // 4 wavefronts, 2 x 2
constexpr int XCDS = 8;

// Two packed words (16 codes) -> the four operand registers of one matrix instruction.
// `hi` is 0xF0F0F0F0; the pipelined kernel passes it in a scalar register so that the
// four ANDs are 4-byte instructions instead of 8-byte ones carrying a literal.
__device__ __forceinline__ v4i expand(u32 w0, u32 w1, u32 hi = 0xF0F0F0F0u) {
  v4i r;
  r[0] = (int)((w0 << 4) & hi);   // even codes of w0, times 16
  r[1] = (int)(w0 & hi);          // odd codes of w0, times 16
  r[2] = (int)((w1 << 4) & hi);
  r[3] = (int)(w1 & hi);
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
// Y is written once and not read again by this kernel: non-temporal stores keep the
// output stream from evicting the packed operands (above all the weights, which every
// tile re-reads) out of the L2.  Measured on the 131072 x 1024 x 4096 shape: plain
// stores cost 12 % (binary16 out) to 23 % (binary32 out) more time.  A non-temporal
// store that leaves part of a 128-byte line unwritten is expensive on the memory side,
// so the callers order their stores to complete lines within a few instructions.
template <>
__device__ __forceinline__ void store_out<float>(float* p, float v) {
  __builtin_nontemporal_store(v, p);
}
template <>
__device__ __forceinline__ void store_out<_Float16>(_Float16* p, float v) {
  // v is the binary32 result; it is rounded to binary16 in a second, separate step.
  // The empty asm keeps the compiler from merging the last binary32 operation with the
  // conversion into one mixed-precision instruction, which would round only once.
  asm volatile("" : "+v"(v));
  __builtin_nontemporal_store((_Float16)v, p);
}

typedef _Float16 h2v __attribute__((ext_vector_type(2)));
typedef float f2v __attribute__((ext_vector_type(2)));
// Two binary32 results -> two binary16 values with one packed conversion (round to
// nearest even, as the scalar one).  As in store_out, the empty asm keeps the last
// binary32 operations from being merged with the conversion into mixed-precision
// instructions that would round only once.
__device__ __forceinline__ h2v round_pair_to_half(float a, float b) {
  asm volatile("" : "+v"(a), "+v"(b));
  const f2v v = {a, b};
  return __builtin_convertvector(v, h2v);
}

// 16 bytes of consecutive outputs with one store (p aligned to 16 bytes).
template <typename OUT>
struct OutVec;
template <>
struct OutVec<float> { static constexpr int W = 4; };
template <>
struct OutVec<_Float16> { static constexpr int W = 8; };
template <typename OUT>
__device__ __forceinline__ void store_out_vec(OUT* p, const float (&y)[OutVec<OUT>::W]);
template <>
__device__ __forceinline__ void store_out_vec<float>(float* p, const float (&y)[4]) {
  typedef float f4v __attribute__((ext_vector_type(4)));
  const f4v v = {y[0], y[1], y[2], y[3]};
  __builtin_nontemporal_store(v, reinterpret_cast<f4v*>(p));
}
template <>
__device__ __forceinline__ void store_out_vec<_Float16>(_Float16* p, const float (&y)[8]) {
  typedef _Float16 h8v __attribute__((ext_vector_type(8)));
  const h2v a = round_pair_to_half(y[0], y[1]), b = round_pair_to_half(y[2], y[3]);
  const h2v c = round_pair_to_half(y[4], y[5]), d = round_pair_to_half(y[6], y[7]);
  const h8v v = {a[0], a[1], b[0], b[1], c[0], c[1], d[0], d[1]};
  __builtin_nontemporal_store(v, reinterpret_cast<h8v*>(p));
}

// Wavefront tile = (32 MT) x (32 NT) of Y, workgroup = 2 x 2 wavefronts.
//   MT = NT = 4: 256 x 256 per workgroup, 256 accumulator registers per lane, one
//                wavefront per SIMD; 3 expand operations per matrix instruction.
//   MT = NT = 2: 128 x 128, for shapes too small to fill the chip with big tiles.
template <typename OUT, int MT, int NT>
__global__ __launch_bounds__(GEMM_THREADS, (MT * NT >= 16 ? 1 : MT * NT >= 8 ? 2 : 3)) void k_w4a4_gemm(
    const uint8_t* __restrict__ Qx, long long ld_q, const int* __restrict__ gid,
    const float* __restrict__ scale, int M, int T, int K, int N, int G,
    const uint8_t* __restrict__ Qw, long long ld_w, const float* __restrict__ w_scale,
    const float* __restrict__ bias, OUT* __restrict__ Y, long long ld_y, int* __restrict__ acc_dump,
    int m_tiles, int n_tiles) {
  constexpr int BM = 64 * MT, BN = 64 * NT;
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

  for (int i = tid; i < BM; i += GEMM_THREADS) {
    const int m = m0 + i;
    float rs = 0.f;
    if (m < M) {
      const int b = m / T;
      const int g = gid ? gid[m] : 0;
      rs = scale[(long long)b * G + g];
    }
    sRow[i] = rs;
  }
  for (int j = tid; j < BN; j += GEMM_THREADS) {
    const int n = n0 + j;
    sCol[j] = n < N ? w_scale[n] : 0.f;
    sBias[j] = (bias && n < N) ? bias[n] : 0.f;
  }

  // global -> register staging: a stage is BM (BN) rows x 64 B per operand, moved
  // as 16-byte pieces; thread t owns column piece (t & 3) of rows (t >> 2) + 64 i.
  const int pr0 = tid >> 2, pc = (tid & 3) * 16;
  const uint8_t* pa[MT];
  const uint8_t* pb[NT];
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    int r = m0 + pr0 + 64 * i;
    r = r < M ? r : M - 1;
    pa[i] = Qx + (long long)r * ld_q + pc;
  }
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    int r = n0 + pr0 + 64 * j;
    r = r < N ? r : N - 1;
    pb[j] = Qw + (long long)r * ld_w + pc;
  }
  uint4 ga[MT], gb[NT];
  auto load_stage = [&](int kt) {
    const int kb = kt * BKB + pc;          // first packed byte of this piece
    if (kb < kbytes) {
#pragma unroll
      for (int i = 0; i < MT; ++i)
        ga[i] = *reinterpret_cast<const uint4*>(pa[i] + (long long)kt * BKB);
#pragma unroll
      for (int j = 0; j < NT; ++j)
        gb[j] = *reinterpret_cast<const uint4*>(pb[j] + (long long)kt * BKB);
      if (kb + 16 > kbytes) {              // piece straddles the end of the row: zero the rest
        const int keep = kbytes - kb;      // 1..15 bytes are real
#pragma unroll
        for (int i = 0; i < MT; ++i) mask_piece(ga[i], keep);
#pragma unroll
        for (int j = 0; j < NT; ++j) mask_piece(gb[j], keep);
      }
    } else {
#pragma unroll
      for (int i = 0; i < MT; ++i) ga[i] = make_uint4(0, 0, 0, 0);
#pragma unroll
      for (int j = 0; j < NT; ++j) gb[j] = make_uint4(0, 0, 0, 0);
    }
  };
  auto store_stage = [&](int buf) {
#pragma unroll
    for (int i = 0; i < MT; ++i)
      *reinterpret_cast<uint4*>(&sA[buf][(pr0 + 64 * i) * LDS_STRIDE + pc]) = ga[i];
#pragma unroll
    for (int j = 0; j < NT; ++j)
      *reinterpret_cast<uint4*>(&sB[buf][(pr0 + 64 * j) * LDS_STRIDE + pc]) = gb[j];
  };

  v16i acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  load_stage(0);
  store_stage(0);
  __syncthreads();

  // Lane l of a wavefront feeds row (l & 31) of a 32-row fragment and, of each
  // 32-byte slab (64 codes) of K, the 16 bytes at offset 16 * (l >> 5).
  const int frow = lane & 31, fhalf = (lane >> 5) * 16;
  const int a_off = (wm * 32 * MT + frow) * LDS_STRIDE + fhalf;
  const int b_off = (wn * 32 * NT + frow) * LDS_STRIDE + fhalf;
  for (int kt = 0; kt < k_tiles; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < k_tiles) load_stage(kt + 1);
#pragma unroll
    for (int ks = 0; ks < BKB / 32; ++ks) {
      uint4 fa[MT], fb[NT];
#pragma unroll
      for (int i = 0; i < MT; ++i)
        fa[i] = *reinterpret_cast<const uint4*>(&sA[cur][a_off + i * 32 * LDS_STRIDE + ks * 32]);
#pragma unroll
      for (int j = 0; j < NT; ++j)
        fb[j] = *reinterpret_cast<const uint4*>(&sB[cur][b_off + j * 32 * LDS_STRIDE + ks * 32]);
      v4i a0[MT], a1[MT], b0[NT], b1[NT];
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        a0[i] = expand(fa[i].x, fa[i].y);
        a1[i] = expand(fa[i].z, fa[i].w);
      }
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        b0[j] = expand(fb[j].x, fb[j].y);
        b1[j] = expand(fb[j].z, fb[j].w);
      }
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0[i], b0[j], acc[i][j], 0, 0, 0);
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1[i], b1[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < k_tiles) store_stage(cur ^ 1);
    __syncthreads();
  }

  // Epilogue.  Register r of a 32x32 accumulator fragment held by lane l is
  // element (row 8*(r/4) + 4*(l/32) + r%4, column l%32).
  const int ccol = lane & 31, rquad = (lane >> 5) * 4;
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int cl = wn * 32 * NT + j * 32 + ccol;
      const int n = n0 + cl;
      const float ws = sCol[cl], bs = sBias[cl];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int rl = wm * 32 * MT + i * 32 + (r >> 2) * 8 + rquad + (r & 3);
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

// ---------------------------------------------------------------------------
// Software-pipelined kernel for large shapes (K a multiple of 128 codes).
//
// A wavefront owns (32 MT) x (32 NT) of Y; a workgroup is 2 x 2 wavefronts.
//   MT = NT = 4: 256 x 256 tile, 256 accumulator registers, one wavefront per SIMD:
//                nothing but the wavefront's own instruction stream hides latency.
//   (The template also builds 256 x 128 and 128 x 256 tiles with two workgroups per
//   CU; on the 131072-row shapes of the largest configuration they measured within
//   3 % of the square tile, slower on K = 4096, so the dispatcher does not use them.)
// The stream is laid out by hand in bundles of one or two matrix instructions, the
// six expand operations of ONE operand fragment of the NEXT operand set (3 vector
// ops per matrix op at MT = NT = 4, which the vector unit absorbs while the matrix
// unit is busy) and at most one LDS read or one global load.  Per stage of 128
// codes (4 half-slabs of MT + NT bundles):
//   X0: set 0 of slab 0 | expand set 1 of slab 0 | LDS reads of slab 1
//   Y0: set 1 of slab 0 | expand set 0 of slab 1 | direct-to-LDS loads of stage + 2
//   wait for stage + 1, barrier
//   X1: set 0 of slab 1 | expand set 1 of slab 1 | LDS reads of slab 0 of stage + 1
//   Y1: set 1 of slab 1 | expand set 0 of that slab
//
// The activations are the row operand of the matrix instruction, so the 32 lanes of
// a half-wavefront hold 32 consecutive columns of one row of Y and every store
// instruction writes whole 128-byte (fp32) / 64-byte (fp16) row segments.  (With
// the operands swapped a lane would own 4 consecutive columns and could store 16
// bytes at once, but into 64 different rows per instruction: measured 40 % slower.)
//
// Stages arrive by direct-to-LDS loads (global_load_lds_dwordx4): no staging
// registers and no LDS write instructions in the wavefront's stream (an LDS write of
// 16 bytes per lane costs more than twice an LDS read of the same size on this
// chip), into a ring of three LDS slots so the loads run two stages ahead.
//
// LDS layout of a slot: rows of 64 bytes (4 pieces of 16), piece c of row r stored
// at position c ^ ((r >> 2) & 3): the 16-byte reads of 16 consecutive rows then
// fall on 16 different bank groups of the 64-bank LDS.  A direct load writes 64
// lanes x 16 bytes contiguously from the address in M0, so lane l of load i of
// wavefront w fills position l & 3 of row 64 i + 16 w + (l >> 2) and fetches the
// global piece that belongs there.
//
// These loads are issued from inline assembly, so the compiler neither sees that
// they write LDS nor counts them in vmcnt; the kernel waits for them itself: every
// stage issues exactly MT + NT per thread, hence "vmcnt(MT + NT)" = everything but
// the newest stage has landed.
// ---------------------------------------------------------------------------
template <int MT, int NT>
struct Frags {
  uint4 a[MT], b[NT];     // packed 16-byte pieces: .x .y feed operand set 0, .z .w set 1
};
template <int MT, int NT>
struct Operands {
  v4i a[MT], b[NT];
};

template <int SET, int MT, int NT>
__device__ __forceinline__ void expand_one(Operands<MT, NT>& dst, const Frags<MT, NT>& f, int e,
                                           u32 hi) {
  // e is a compile-time constant after unrolling
  if (e < MT) {
    dst.a[e] = SET == 0 ? expand(f.a[e].x, f.a[e].y, hi) : expand(f.a[e].z, f.a[e].w, hi);
  } else {
    dst.b[e - MT] = SET == 0 ? expand(f.b[e - MT].x, f.b[e - MT].y, hi)
                             : expand(f.b[e - MT].z, f.b[e - MT].w, hi);
  }
}

// MT * NT matrix instructions on `cur`, spread over MT + NT bundles, each with the
// expansion of one fragment of operand set EXP_SET from `f` into `nxt` and with
// mem(b), at most one memory instruction.
// One half (HALF = 0: words x / z -> elements 0, 1; HALF = 1: words y / w -> elements
// 2, 3) of the expansion of fragment e: three vector operations.
template <int SET, int HALF, int MT, int NT>
__device__ __forceinline__ void expand_half(Operands<MT, NT>& dst, const Frags<MT, NT>& f, int e,
                                            u32 hi) {
  const uint4& q = e < MT ? f.a[e] : f.b[e - MT];
  const u32 w = SET == 0 ? (HALF == 0 ? q.x : q.y) : (HALF == 0 ? q.z : q.w);
  v4i& d = e < MT ? dst.a[e] : dst.b[e - MT];
  d[2 * HALF] = (int)((w << 4) & hi);      // even codes of w, times 16
  d[2 * HALF + 1] = (int)(w & hi);         // odd codes of w, times 16
}

// MT * NT matrix instructions on `cur`, spread over MT + NT bundles, each with the
// expansion of one fragment of operand set EXP_SET from `f` into `nxt` and with
// mem(b), at most one memory instruction.  A wavefront issues in order, and a matrix
// instruction cannot start before the previous one has left the matrix pipe, so the
// vector work of a bundle is split between the shadows of its matrix instructions
// (matrix, three vector, matrix, three vector + memory) rather than queued behind both.
// ZERO: the matrix instructions start a fresh accumulation (C operand 0) instead of adding
// to acc: the first half-slab of a tile in a kernel that keeps its accumulators across tiles.
template <int EXP_SET, int MT, int NT, bool ZERO = false, typename MEM>
__device__ __forceinline__ void half_slab(v16i (&acc)[MT][NT], const Operands<MT, NT>& cur,
                                          Operands<MT, NT>& nxt, const Frags<MT, NT>& f, u32 hi,
                                          MEM mem) {
  constexpr int NB = MT + NT, NM = MT * NT;
  const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    const int lo = (b * NM) / NB, up = ((b + 1) * NM) / NB, mid = lo + (up - lo + 1) / 2;
#pragma unroll
    for (int m = lo; m < mid; ++m) {
      const int i = m / NT, j = m % NT;
      acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(cur.a[i], cur.b[j], ZERO ? zero : acc[i][j],
                                                        0, 0, 0);
    }
    expand_half<EXP_SET, 0>(nxt, f, b, hi);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int m = mid; m < up; ++m) {
      const int i = m / NT, j = m % NT;
      acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(cur.a[i], cur.b[j], ZERO ? zero : acc[i][j],
                                                        0, 0, 0);
    }
    expand_half<EXP_SET, 1>(nxt, f, b, hi);
    mem(b);
    __builtin_amdgcn_sched_barrier(0);
  }
}

__device__ __forceinline__ void dma16(const uint8_t* gptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :
               : "v"(gptr), "s"(lds_base)
               : "memory");
}

// The same with a wavefront-uniform 64-bit base and a 32-bit per-lane byte offset.
__device__ __forceinline__ void dma16s(const uint8_t* base, unsigned off, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(off), "s"(base), "s"(lds_base)
               : "memory");
}

// 64 floats from 64 addresses -> 64 consecutive floats of LDS
__device__ __forceinline__ void dma4s(const float* sbase, unsigned voff, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
               :
               : "v"(voff), "s"(sbase), "s"(lds_base)
               : "memory");
}

// Output of a wavefront's (32 MT) x (32 NT) part of a tile that lies wholly inside Y:
// y = (float(acc) * row scale) * column scale (+ bias), each product rounded to binary32.
// Register r of a 32x32 accumulator fragment held by lane l is element
// (row 8*(r/4) + 4*(l/32) + r%4, column l%32).  Every address is a wavefront-uniform row
// pointer plus one per-lane 32-bit offset.  wtile = &Y[first row][first column] of the
// wavefront's part.
template <typename OUT, int MT, int NT, typename ACC, bool BIAS>
__device__ __forceinline__ void tile_store_fast(ACC (&acc)[MT][NT], const float* sRow,
                                                const float* sCol, const float* sBias, int lane,
                                                int wm, int wn, OUT* __restrict__ wtile,
                                                long long ld_y) {
  const int ccol = lane & 31, rquad = (lane >> 5) * 4;
  const unsigned lane_offu = (unsigned)(rquad * (int)ld_y + ccol);
  float ws[NT], bs[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    ws[j] = sCol[wn * 32 * NT + j * 32 + ccol];
    bs[j] = sBias[wn * 32 * NT + j * 32 + ccol];
  }
#pragma unroll
  for (int i = 0; i < MT; ++i) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float4 rs4 =
          *reinterpret_cast<const float4*>(&sRow[wm * 32 * MT + i * 32 + q * 8 + rquad]);
      const float rsv[4] = {rs4.x, rs4.y, rs4.z, rs4.w};
      // Two rows at a time.  The NT column blocks of one row are stored back to back:
      // together they cover whole cache lines of Y, written within a few instructions of
      // each other.
#pragma unroll
      for (int t = 0; t < 4; t += 2) {
        OUT* row0 = wtile + (long long)(i * 32 + q * 8 + t) * ld_y + lane_offu;   // uniform + lane
        OUT* row1 = row0 + ld_y;
        float y0[NT], y1[NT];
#pragma unroll
        for (int j = 0; j < NT; ++j) {
          const auto a0 = acc[i][j][4 * q + t], a1 = acc[i][j][4 * q + t + 1];
          y0[j] = ((float)a0 * rsv[t]) * ws[j];
          y1[j] = ((float)a1 * rsv[t + 1]) * ws[j];
          if (BIAS) {
            y0[j] = y0[j] + bs[j];
            y1[j] = y1[j] + bs[j];
          }
        }
        if constexpr (sizeof(OUT) == 2) {
          // one packed conversion rounds the two rows' binary32 results to binary16
          h2v p[NT];
#pragma unroll
          for (int j = 0; j < NT; ++j) p[j] = round_pair_to_half(y0[j], y1[j]);
#pragma unroll
          for (int j = 0; j < NT; ++j) __builtin_nontemporal_store(p[j][0], row0 + j * 32);
#pragma unroll
          for (int j = 0; j < NT; ++j) __builtin_nontemporal_store(p[j][1], row1 + j * 32);
        } else {
#pragma unroll
          for (int j = 0; j < NT; ++j) store_out<OUT>(row0 + j * 32, y0[j]);
#pragma unroll
          for (int j = 0; j < NT; ++j) store_out<OUT>(row1 + j * 32, y1[j]);
        }
      }
    }
  }
}

// Output phase of the persistent kernel.  Its weight rows are dealt to the column blocks so
// that column block j of a wavefront holds output columns 4 c + j (c = lane % 32): the four
// accumulators acc[i][0..3][r] of a lane are then four ADJACENT outputs of one row, and a lane
// stores them with one instruction (8 bytes of binary16, 16 of binary32) -- 64 stores per
// wavefront and tile instead of 256, each completing 256 or 512 contiguous bytes of two rows.
// y = (float(acc) * row scale) * (column scale * 2^-8) (+ bias): the 2^-8 that takes the 256
// out of the int8 accumulators rides on the column scale (a power of two: the same bits).
// The accumulators are read where they are used and the scheduler may not move code across
// rows, which keeps the registers this needs at any one time to a few dozen.  The stores are
// the compiler's own (non-temporal, see store_out): a 16-byte store reads its data registers
// over several cycles and the compiler, not inline assembly, knows how long to keep them.
typedef float f4v __attribute__((ext_vector_type(4)));
typedef unsigned u2v __attribute__((ext_vector_type(2)));
template <typename OUT, bool BIAS>
__device__ __forceinline__ void tile_store_cols4(v16i (&acc)[4][4], const float* sRow, const float* sCol,
                                                 const float* sBias, int lane, int wm, int wn,
                                                 const OUT* __restrict__ wtile, long long ld_y) {
  const int ccol = lane & 31, rquad = (lane >> 5) * 4;
  // byte offset of the lane inside the wavefront's 128 rows; 132 rows of ld_y elements fit 32 bits (host)
  const unsigned lane_off = (unsigned)(rquad * (int)ld_y + 4 * ccol) * (unsigned)sizeof(OUT);
  const float4 w4 = *reinterpret_cast<const float4*>(&sCol[wn * 128 + 4 * ccol]);
  const float4 b4 = *reinterpret_cast<const float4*>(&sBias[wn * 128 + 4 * ccol]);
  const float ws[4] = {w4.x * 0.00390625f, w4.y * 0.00390625f, w4.z * 0.00390625f, w4.w * 0.00390625f};
  const float bs[4] = {b4.x, b4.y, b4.z, b4.w};
  // Every instruction of a lone wavefront costs an issue slot here (nothing else runs on the
  // SIMD during the output phase), so the store address costs one vector add per row: scalar
  // base of the wavefront's part of the tile + a 32-bit lane offset that walks down the rows
  // (rows 0-3, 8-11, ... of every 32: steps of one row and of five).
  typedef __attribute__((address_space(1))) char gchar;
  gchar* const base = reinterpret_cast<gchar*>(reinterpret_cast<unsigned long long>(wtile));
  unsigned voff = lane_off;
  const unsigned step1 = (unsigned)ld_y * (unsigned)sizeof(OUT), step5 = 5u * step1;
  // The four row scales of a group of four rows are read from LDS one group ahead: a lone
  // wavefront has nothing else to run while it waits for an LDS read.  The accumulators of a
  // row are copied out of the accumulation registers one row ahead, between the previous
  // row's last binary32 operation and its conversion / store: the instruction after an asm
  // statement then never reads what the statement wrote, and no wait state is inserted.
  const float* rs_src = sRow + wm * 128 + rquad;
  float4 rs_next = *reinterpret_cast<const float4*>(rs_src);
  int a_cur[4], a_nxt[4] = {0, 0, 0, 0};
#pragma unroll
  for (int j = 0; j < 4; ++j) asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(a_cur[j]) : "a"(acc[0][j][0]));
#pragma unroll
  for (int g = 0; g < 16; ++g) {                   // row group g: rows 8 g .. 8 g + 3 (+ 4 for the upper lanes)
    const float rsv[4] = {rs_next.x, rs_next.y, rs_next.z, rs_next.w};
    if (g + 1 < 16) rs_next = *reinterpret_cast<const float4*>(rs_src + (g + 1) * 8);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      float y[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        y[j] = ((float)a_cur[j] * rsv[t]) * ws[j];
        if (BIAS) y[j] = y[j] + bs[j];
      }
      __builtin_amdgcn_sched_barrier(0);
      const int r2 = 4 * g + t + 1;                // the next row's accumulators
      const int i2 = (r2 >> 4) & 3, q2 = (r2 >> 2) & 3, t2 = r2 & 3;
      if constexpr (sizeof(OUT) == 2) {
        // One asm statement copies the next row's accumulators out and rounds this row's pairs
        // of binary32 results to binary16 (packed conversion, to nearest even): the conversion
        // cannot be merged with the multiplication before it into a mixed-precision
        // instruction that would round only once, and the instruction after the statement --
        // the next row's address -- reads nothing the statement wrote.
        u2v v;
        if (r2 < 64)
          asm volatile(
              "v_accvgpr_read_b32 %2, %10\n\tv_accvgpr_read_b32 %3, %11\n\t"
              "v_accvgpr_read_b32 %4, %12\n\tv_accvgpr_read_b32 %5, %13\n\t"
              "v_cvt_pk_f16_f32 %0, %6, %7\n\tv_cvt_pk_f16_f32 %1, %8, %9"
              : "=&v"(v.x), "=&v"(v.y), "=&v"(a_nxt[0]), "=&v"(a_nxt[1]), "=&v"(a_nxt[2]), "=&v"(a_nxt[3])
              : "v"(y[0]), "v"(y[1]), "v"(y[2]), "v"(y[3]), "a"(acc[i2][0][4 * q2 + t2]),
                "a"(acc[i2][1][4 * q2 + t2]), "a"(acc[i2][2][4 * q2 + t2]), "a"(acc[i2][3][4 * q2 + t2]));
        else
          asm volatile("v_cvt_pk_f16_f32 %0, %2, %3\n\tv_cvt_pk_f16_f32 %1, %4, %5"
                       : "=&v"(v.x), "=&v"(v.y)
                       : "v"(y[0]), "v"(y[1]), "v"(y[2]), "v"(y[3]));
        __builtin_amdgcn_sched_barrier(0);
        const unsigned voff_next = voff + (t == 3 ? step5 : step1);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_nontemporal_store(v, reinterpret_cast<__attribute__((address_space(1))) u2v*>(base + voff));
        voff = voff_next;
      } else {
        if (r2 < 64) {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(a_nxt[j]) : "a"(acc[i2][j][4 * q2 + t2]));
        }
        __builtin_amdgcn_sched_barrier(0);
        const f4v v = {y[0], y[1], y[2], y[3]};
        __builtin_nontemporal_store(v, reinterpret_cast<__attribute__((address_space(1))) f4v*>(base + voff));
        voff += t == 3 ? step5 : step1;
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) a_cur[j] = a_nxt[j];
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

// Epilogue of the pipelined kernels.  Register r of a 32x32 accumulator fragment held
// by lane l is element (row 8*(r/4) + 4*(l/32) + r%4, column l%32).
template <typename OUT, int MT, int NT, typename ACC = v16i>
__device__ __forceinline__ void pipe_epilogue(ACC (&acc)[MT][NT], const float* sRow,
                                              const float* sCol, const float* sBias, int lane,
                                              int wm, int wn, int m0, int n0, int M, int N,
                                              const float* __restrict__ bias, OUT* __restrict__ Y,
                                              long long ld_y, int* __restrict__ acc_dump) {
  constexpr int BM = 64 * MT, BN = 64 * NT;
  const int ccol = lane & 31, rquad = (lane >> 5) * 4;
  const bool inside = m0 + BM <= M && n0 + BN <= N;
  if (inside && !acc_dump && (long long)(BM + 8) * ld_y < (1ll << 31) / (long long)sizeof(OUT)) {
    OUT* wtile = Y + (long long)(m0 + wm * 32 * MT) * ld_y + (n0 + wn * 32 * NT);
    if (bias)
      tile_store_fast<OUT, MT, NT, ACC, true>(acc, sRow, sCol, sBias, lane, wm, wn, wtile, ld_y);
    else
      tile_store_fast<OUT, MT, NT, ACC, false>(acc, sRow, sCol, sBias, lane, wm, wn, wtile, ld_y);
    return;
  }
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int cl = wn * 32 * NT + j * 32 + ccol;
      const int n = n0 + cl;
      const float ws = sCol[cl], bs = sBias[cl];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int rl = wm * 32 * MT + i * 32 + (r >> 2) * 8 + rquad + (r & 3);
        const int m = m0 + rl;
        if (m < M && n < N) {
          float y;
          if (acc_dump) {
            int a;
            if constexpr (std::is_same<ACC, v16i>::value) a = acc[i][j][r] >> 8;   // exact: 256 * acc
            else a = (int)acc[i][j][r];                                          // exact integer
            acc_dump[(long long)m * N + n] = a;
            y = ((float)a * sRow[rl]) * ws;
          } else {
            y = ((float)acc[i][j][r] * sRow[rl]) * ws;
          }
          if (bias) y = y + bs;
          store_out<OUT>(Y + (long long)m * ld_y + n, y);
        }
      }
    }
}

template <typename OUT, int MT, int NT>
__global__ __launch_bounds__(GEMM_THREADS, (MT * NT >= 16 ? 1 : 2)) void k_w4a4_gemm_pipe(
    const uint8_t* __restrict__ Qx, long long ld_q, const int* __restrict__ gid,
    const float* __restrict__ scale, int M, int T, int K, int N, int G,
    const uint8_t* __restrict__ Qw, long long ld_w, const float* __restrict__ w_scale,
    const float* __restrict__ bias, OUT* __restrict__ Y, long long ld_y, int* __restrict__ acc_dump,
    int m_tiles, int n_tiles) {
  constexpr int BM = 64 * MT, BN = 64 * NT, NB = MT + NT;
  constexpr int SLOT = (BM + BN) * BKB;      // bytes of one ring slot: A rows then B rows, 64 B each
  __shared__ __attribute__((aligned(1024))) uint8_t ring[3 * SLOT];
  __shared__ __attribute__((aligned(16))) float sRow[BM], sCol[BN], sBias[BN];

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
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int k_tiles = ((K + 1) / 2) / BKB;          // host guarantees K % 128 == 0

  // Scales of the epilogue.  The token-set ids are fetched first; the scales that
  // depend on them are fetched after the first stages' loads have been issued, so
  // the latencies overlap.
  int my_m[(BM + GEMM_THREADS - 1) / GEMM_THREADS], my_g[(BM + GEMM_THREADS - 1) / GEMM_THREADS];
#pragma unroll
  for (int u = 0; u < (BM + GEMM_THREADS - 1) / GEMM_THREADS; ++u) {
    const int m = m0 + tid + u * GEMM_THREADS;
    my_m[u] = m < M ? m : M - 1;
    my_g[u] = gid ? gid[my_m[u]] : 0;
  }

  // global source of this lane's piece of load i (rows 64 i + 16 w + (l >> 2))
  const uint8_t* pa[MT];
  const uint8_t* pb[NT];
  {
    const int rl0 = 16 * wave + (lane >> 2);
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const int rl = 64 * i + rl0;                            // row inside the tile
      const int c = (lane & 3) ^ ((rl >> 2) & 3);             // logical piece stored at position l & 3
      int r = m0 + rl;
      r = r < M ? r : M - 1;
      pa[i] = Qx + (long long)r * ld_q + c * 16;
    }
#pragma unroll
    for (int i = 0; i < NT; ++i) {
      const int rl = 64 * i + rl0;
      const int c = (lane & 3) ^ ((rl >> 2) & 3);
      int n = n0 + rl;
      n = n < N ? n : N - 1;
      pb[i] = Qw + (long long)n * ld_w + c * 16;
    }
  }
  const unsigned ring_base =
      (unsigned)(size_t)(__attribute__((address_space(3))) uint8_t*)ring;
  const unsigned dma_base = __builtin_amdgcn_readfirstlane(ring_base + wave * 1024);
  auto dma_piece = [&](int slot, int kt, int e) {     // slot, e compile-time; e = 0 .. NB-1
    const int kc = kt < k_tiles ? kt : k_tiles - 1;    // past the end: harmless re-load
    const long long ko = (long long)kc * BKB;
    if (e < MT)
      dma16(pa[e] + ko, dma_base + slot * SLOT + e * 4096);
    else
      dma16(pb[e - MT] + ko, dma_base + slot * SLOT + BM * BKB + (e - MT) * 4096);
  };

  // fragment reads: lane (row r' = l & 31, half h = l >> 5) of fragment e reads piece
  // 2 ks + h of row 32 e + r' (+ the wavefront's offset); the swizzle only depends on r'
  const int frow = lane & 31, fh = lane >> 5, swz = (frow >> 2) & 3;
  const int a_row = (wm * 32 * MT + frow) * 64, b_row = BM * BKB + (wn * 32 * NT + frow) * 64;
  const int off_k0 = ((0 + fh) ^ swz) * 16, off_k1 = ((2 + fh) ^ swz) * 16;
  auto read_piece = [&](Frags<MT, NT>& f, int slot, int ks, int e) {   // slot, ks, e compile-time
    const int off = ks == 0 ? off_k0 : off_k1;
    if (e < MT)
      f.a[e] = *reinterpret_cast<const uint4*>(&ring[slot * SLOT + a_row + e * 2048 + off]);
    else
      f.b[e - MT] =
          *reinterpret_cast<const uint4*>(&ring[slot * SLOT + b_row + (e - MT) * 2048 + off]);
  };

  v16i acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
  Frags<MT, NT> f0, f1;
  Operands<MT, NT> s0, s1;
  u32 hi;                                   // 0xF0F0F0F0 in a scalar register
  asm volatile("s_mov_b32 %0, 0xf0f0f0f0" : "=s"(hi));
#pragma unroll
  for (int e = 0; e < NB; ++e) dma_piece(0, 0, e);
#pragma unroll
  for (int e = 0; e < NB; ++e) dma_piece(1, 1, e);
#pragma unroll
  for (int u = 0; u < (BM + GEMM_THREADS - 1) / GEMM_THREADS; ++u) {
    const int i = tid + u * GEMM_THREADS;
    if (i < BM) {
      const float rs = scale[(long long)(my_m[u] / T) * G + my_g[u]];
      // the accumulators carry a factor 256; folding 2^-8 into the row scale is exact
      sRow[i] = acc_dump ? rs : rs * 0.00390625f;
    }
  }
  for (int j = tid; j < BN; j += GEMM_THREADS) {
    const int n = n0 + j;
    sCol[j] = n < N ? w_scale[n] : 0.f;
    sBias[j] = (bias && n < N) ? bias[n] : 0.f;
  }
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NB) : "memory");      // stage 0 has landed
  __syncthreads();
#pragma unroll
  for (int e = 0; e < NB; ++e) read_piece(f0, 0, 0, e);
#pragma unroll
  for (int e = 0; e < NB; ++e) expand_one<0>(s0, f0, e, hi);

  // One stage: CUR holds stage kt, NXT stage kt + 1 (in flight until the barrier),
  // LD receives stage kt + 2 (the slot that held stage kt - 1).  The body is
  // branch-free so that its bundles stay in one scheduling region: stages past the
  // end re-load the last one into an idle slot that nobody reads.
#define TDQ_STAGE(kt, CUR, NXT, LD)                                                              \
  do {                                                                                           \
    __builtin_amdgcn_sched_barrier(0);                                                           \
    half_slab<1>(acc, s0, s1, f0, hi, [&](int b) { read_piece(f1, CUR, 1, b); });       /* X0 */ \
    half_slab<0>(acc, s1, s0, f1, hi, [&](int b) { dma_piece(LD, (kt) + 2, b); });      /* Y0 */ \
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NB) : "memory");                                    \
    __syncthreads();                                                                             \
    __builtin_amdgcn_sched_barrier(0);                                                           \
    half_slab<1>(acc, s0, s1, f1, hi, [&](int b) { read_piece(f0, NXT, 0, b); });       /* X1 */ \
    half_slab<0>(acc, s1, s0, f0, hi, [&](int) {});                                     /* Y1 */ \
  } while (0)

  int kt = 0;
  for (; kt + 2 < k_tiles; kt += 3) {
    TDQ_STAGE(kt, 0, 1, 2);
    TDQ_STAGE(kt + 1, 1, 2, 0);
    TDQ_STAGE(kt + 2, 2, 0, 1);
  }
  if (kt < k_tiles) TDQ_STAGE(kt, 0, 1, 2);
  if (kt + 1 < k_tiles) TDQ_STAGE(kt + 1, 1, 2, 0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // nothing of ours may still be landing
#undef TDQ_STAGE

  pipe_epilogue<OUT, MT, NT>(acc, sRow, sCol, sBias, lane, wm, wn, m0, n0, M, N, bias, Y, ld_y,
                             acc_dump);
}

// ---------------------------------------------------------------------------
// Wide-stage variant of the pipelined kernel (K a multiple of 256 codes): a stage is
// 128 bytes = one whole cache line of every operand row, so a line is fetched once
// (the 64-byte stages above fetch each line twice, two stages apart, and the L1
// cannot hold 512 lines in between), and the workgroup meets at one barrier per 256
// codes instead of two.  256 x 256 tile, 2 x 2 wavefronts of 4 x 4 blocks, two LDS
// slots of 64 KiB.  Per stage (4 slabs of 64 codes; Xs/Ys as above):
//   X0 | LDS reads of slab 1        Y0 | loads 8..15 of stage + 1
//   X1 | LDS reads of slab 2        Y1
//   X2 | LDS reads of slab 3        Y2
//   wait for stage + 1 (all of this thread's loads), barrier
//   X3 | LDS reads of slab 0 of stage + 1      Y3 | loads 0..7 of stage + 2
// The loads of stage + 2 go into the slot of the stage that is ending: its last
// fragment reads (slab 3) were issued before the barrier, and every wavefront drains
// its LDS reads before it arrives there.  LDS rows are 128 bytes, piece c of row r at
// position c ^ ((r >> 1) & 7): 16 consecutive rows fall on 16 different bank groups.
// ---------------------------------------------------------------------------
template <typename OUT>
__global__ __launch_bounds__(GEMM_THREADS, 1) void k_w4a4_gemm_wide(
    const uint8_t* __restrict__ Qx, long long ld_q, const int* __restrict__ gid,
    const float* __restrict__ scale, int M, int T, int K, int N, int G,
    const uint8_t* __restrict__ Qw, long long ld_w, const float* __restrict__ w_scale,
    const float* __restrict__ bias, OUT* __restrict__ Y, long long ld_y, int* __restrict__ acc_dump,
    int m_tiles, int n_tiles) {
  constexpr int MT = 4, NT = 4, BM = 256, BN = 256, NB = MT + NT;
  constexpr int BKW = 128;                     // packed bytes of K per stage (256 codes)
  constexpr int SLOT = (BM + BN) * BKW;        // 64 KiB: A rows then B rows, 128 B each
  __shared__ __attribute__((aligned(1024))) uint8_t ring[2 * SLOT];
  __shared__ __attribute__((aligned(16))) float sRow[BM], sCol[BN], sBias[BN];

  const int bid = blockIdx.x;
  const int xcd = bid % XCDS, idx = bid / XCDS;
  const int m_tile = (idx / n_tiles) * XCDS + xcd;
  const int n_tile = idx % n_tiles;
  if (m_tile >= m_tiles) return;
  const int m0 = m_tile * BM, n0 = n_tile * BN;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int k_tiles = (K / 2) / BKW;                // host guarantees K % 256 == 0

  const int my_m = m0 + tid < M ? m0 + tid : M - 1;
  const int my_g = gid ? gid[my_m] : 0;

  // global source of this lane's piece of load i: rows 32 i + 8 w + (l >> 3), 8 per load
  const uint8_t* pa[2 * MT];
  const uint8_t* pb[2 * NT];
  {
    const int rl0 = 8 * wave + (lane >> 3);
    const int c = (lane & 7) ^ ((rl0 >> 1) & 7);      // logical piece stored at position l & 7
#pragma unroll
    for (int i = 0; i < 2 * MT; ++i) {
      int r = m0 + 32 * i + rl0;
      r = r < M ? r : M - 1;
      pa[i] = Qx + (long long)r * ld_q + c * 16;
    }
#pragma unroll
    for (int i = 0; i < 2 * NT; ++i) {
      int n = n0 + 32 * i + rl0;
      n = n < N ? n : N - 1;
      pb[i] = Qw + (long long)n * ld_w + c * 16;
    }
  }
  const unsigned ring_base =
      (unsigned)(size_t)(__attribute__((address_space(3))) uint8_t*)ring;
  const unsigned dma_base = __builtin_amdgcn_readfirstlane(ring_base + wave * 1024);
  auto dma_piece = [&](int slot, int kt, int e) {     // slot, e compile-time; e = 0 .. 15
    const int kc = kt < k_tiles ? kt : k_tiles - 1;    // past the end: harmless re-load
    const long long ko = (long long)kc * BKW;
    if (e < 2 * MT)
      dma16(pa[e] + ko, dma_base + slot * SLOT + e * 4096);
    else
      dma16(pb[e - 2 * MT] + ko, dma_base + slot * SLOT + BM * BKW + (e - 2 * MT) * 4096);
  };

  // fragment reads: lane (row r' = l & 31, half h = l >> 5) of fragment e reads piece
  // 2 ks + h of row 32 e + r' (+ the wavefront's offset); the swizzle only depends on r'
  const int frow = lane & 31, fh = lane >> 5, swz = (frow >> 1) & 7;
  const int a_row = (wm * 128 + frow) * BKW, b_row = BM * BKW + (wn * 128 + frow) * BKW;
  const int off0 = ((0 + fh) ^ swz) * 16, off1 = ((2 + fh) ^ swz) * 16;
  const int off2 = ((4 + fh) ^ swz) * 16, off3 = ((6 + fh) ^ swz) * 16;
  auto read_piece = [&](Frags<MT, NT>& f, int slot, int ks, int e) {   // slot, ks, e compile-time
    const int off = ks == 0 ? off0 : ks == 1 ? off1 : ks == 2 ? off2 : off3;
    if (e < MT)
      f.a[e] = *reinterpret_cast<const uint4*>(&ring[slot * SLOT + a_row + e * 4096 + off]);
    else
      f.b[e - MT] =
          *reinterpret_cast<const uint4*>(&ring[slot * SLOT + b_row + (e - MT) * 4096 + off]);
  };

  v16i acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
  Frags<MT, NT> f0, f1;
  Operands<MT, NT> s0, s1;
  u32 hi;                                   // 0xF0F0F0F0 in a scalar register
  asm volatile("s_mov_b32 %0, 0xf0f0f0f0" : "=s"(hi));
#pragma unroll
  for (int e = 0; e < 2 * NB; ++e) dma_piece(0, 0, e);
#pragma unroll
  for (int e = 0; e < NB; ++e) dma_piece(1, 1, e);
  {
    const float rs = scale[(long long)(my_m / T) * G + my_g];
    // the accumulators carry a factor 256; folding 2^-8 into the row scale is exact
    sRow[tid] = acc_dump ? rs : rs * 0.00390625f;
    const int n = n0 + tid;
    sCol[tid] = n < N ? w_scale[n] : 0.f;
    sBias[tid] = (bias && n < N) ? bias[n] : 0.f;
  }
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NB) : "memory");      // stage 0 has landed
  __syncthreads();
#pragma unroll
  for (int e = 0; e < NB; ++e) read_piece(f0, 0, 0, e);
#pragma unroll
  for (int e = 0; e < NB; ++e) expand_one<0>(s0, f0, e, hi);

#define TDQ_WSTAGE(kt, CUR, OTH)                                                                 \
  do {                                                                                           \
    __builtin_amdgcn_sched_barrier(0);                                                           \
    half_slab<1>(acc, s0, s1, f0, hi, [&](int b) { read_piece(f1, CUR, 1, b); });       /* X0 */ \
    half_slab<0>(acc, s1, s0, f1, hi, [&](int b) { dma_piece(OTH, (kt) + 1, NB + b); }); /* Y0 */ \
    half_slab<1>(acc, s0, s1, f1, hi, [&](int b) { read_piece(f0, CUR, 2, b); });       /* X1 */ \
    half_slab<0>(acc, s1, s0, f0, hi, [&](int) {});                                     /* Y1 */ \
    half_slab<1>(acc, s0, s1, f0, hi, [&](int b) { read_piece(f1, CUR, 3, b); });       /* X2 */ \
    half_slab<0>(acc, s1, s0, f1, hi, [&](int) {});                                     /* Y2 */ \
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");                                  \
    __syncthreads();                                                                             \
    __builtin_amdgcn_sched_barrier(0);                                                           \
    half_slab<1>(acc, s0, s1, f1, hi, [&](int b) { read_piece(f0, OTH, 0, b); });       /* X3 */ \
    half_slab<0>(acc, s1, s0, f0, hi, [&](int b) { dma_piece(CUR, (kt) + 2, b); });     /* Y3 */ \
  } while (0)

  int kt = 0;
  for (; kt + 1 < k_tiles; kt += 2) {
    TDQ_WSTAGE(kt, 0, 1);
    TDQ_WSTAGE(kt + 1, 1, 0);
  }
  if (kt < k_tiles) TDQ_WSTAGE(kt, 0, 1);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // nothing of ours may still be landing
#undef TDQ_WSTAGE

  pipe_epilogue<OUT, MT, NT>(acc, sRow, sCol, sBias, lane, wm, wn, m0, n0, M, N, bias, Y, ld_y,
                             acc_dump);
}

// ---------------------------------------------------------------------------
// Rolling variant of the wide-stage kernel for shapes of many whole tiles (M and N
// multiples of 256, an even number, at least four, of 256-code stages): a workgroup is
// persistent and walks its share of the tiles, and the stream of stages never drains
// between tiles -- the loads of the next tile's first two stages are issued during the
// current tile's last two, like any other stage's, and the next tile's token-set ids and
// scales are fetched during those two stages by direct loads into LDS.  What a tile
// boundary still costs is the output phase itself (the matrix pipe idles while a single
// wavefront per SIMD converts and stores 256 results per lane, tile_store_cols4); the
// workgroup launch, the two dependent loads of the scales and the first stage's load
// latency are gone.
//
// Operand addresses are a uniform 64-bit base (tile, stage) plus a 32-bit per-lane offset
// that does not depend on the tile, so changing tile costs no vector work.
// Stores and loads share one in-order counter (vmcnt): the only wait for loads that has
// output stores before it is the first stage barrier of the next tile, about a hundred
// matrix instructions after the last store was issued.
// Tile order: as in the other kernels every XCD takes whole rows of tiles; inside an XCD
// consecutive workgroups take consecutive tiles, so at any time an XCD's CUs work on a
// few rows of tiles whose operands its L2 holds.
// ---------------------------------------------------------------------------
template <typename OUT>
__global__ __launch_bounds__(GEMM_THREADS, 1) void k_w4a4_gemm_roll(
    const uint8_t* __restrict__ Qx, long long ld_q, const int* __restrict__ gid,
    const float* __restrict__ scale, int M, int T, int K, int N, int G,
    const uint8_t* __restrict__ Qw, long long ld_w, const float* __restrict__ w_scale,
    const float* __restrict__ bias, OUT* __restrict__ Y, long long ld_y, int m_tiles, int n_tiles,
    double inv_T) {
  constexpr int MT = 4, NT = 4, BM = 256, BN = 256, NB = MT + NT;
  constexpr int BKW = 128;                     // packed bytes of K per stage (256 codes)
  constexpr int SLOT = (BM + BN) * BKW;        // 64 KiB: A rows then B rows, 128 B each
  __shared__ __attribute__((aligned(1024))) uint8_t ring[2 * SLOT];
  // scales of the tile being computed and of the next one (sets alternate from tile to
  // tile), and the next tile's token-set ids
  __shared__ __attribute__((aligned(256))) float sRow[2][BM], sCol[2][BN], sBias[2][BN];
  __shared__ __attribute__((aligned(256))) int sGid[BM];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int k_tiles = (K / 2) / BKW;           // even, >= 2 (host)

  // this workgroup's tiles: index list of its XCD, every (gridDim / 8)-th entry
  const int xcd = blockIdx.x % XCDS, wslot = blockIdx.x / XCDS, per_xcd = gridDim.x / XCDS;
  const int xcd_tiles = (m_tiles / XCDS) * n_tiles;          // m_tiles is a multiple of 8 (host)
  const int n_my = wslot < xcd_tiles ? (xcd_tiles - wslot + per_xcd - 1) / per_xcd : 0;
  if (n_my == 0) return;
  auto tile_m0 = [&](int it) { return (((wslot + it * per_xcd) / n_tiles) * XCDS + xcd) * BM; };
  auto tile_n0 = [&](int it) { return ((wslot + it * per_xcd) % n_tiles) * BN; };

  // per-lane byte offsets of this lane's piece of load i (rows 32 i + 8 w + (l >> 3))
  unsigned offA[2 * MT], offB[2 * NT];
  {
    const int rl0 = 8 * wave + (lane >> 3);
    const int c = (lane & 7) ^ ((rl0 >> 1) & 7);      // logical piece stored at position l & 7
#pragma unroll
    for (int i = 0; i < 2 * MT; ++i) offA[i] = (unsigned)((32 * i + rl0) * ld_q + c * 16);
    // Weight rows are dealt to the column blocks: LDS row 128 wn + 32 j + c' of the B part
    // (column block j of wavefront column wn, matrix column c') holds weight row
    // 128 wn + 4 c' + j, so that a lane's four column blocks are four adjacent outputs
    // (tile_store_cols4).  The swizzle goes by the LDS row, as for A.
#pragma unroll
    for (int i = 0; i < 2 * NT; ++i) {
      const int lrow = 32 * i + rl0;                                   // LDS row, 0 .. 255
      const int wrow = (lrow & 128) + 4 * (lrow & 31) + ((lrow >> 5) & 3);
      offB[i] = (unsigned)(wrow * ld_w + c * 16);
    }
  }
  const unsigned ring_base =
      (unsigned)(size_t)(__attribute__((address_space(3))) uint8_t*)ring;
  const unsigned dma_base = __builtin_amdgcn_readfirstlane(ring_base + wave * 1024);

  // uniform operand bases of the current and the next tile
  const uint8_t* curA = Qx + (long long)tile_m0(0) * ld_q;
  const uint8_t* curB = Qw + (long long)tile_n0(0) * ld_w;
  const uint8_t* nxtA = curA;
  const uint8_t* nxtB = curB;
  // stage `rel` counted from the current tile's first: past its end it is a stage of the
  // next tile (or, after the last tile, a harmless re-load into a slot nobody reads)
  auto dma_piece = [&](int slot, int rel, int e) {      // slot, e compile-time; e = 0 .. 15
    const bool next = rel >= k_tiles;
    const long long ko = (long long)(next ? rel - k_tiles : rel) * BKW;
    if (e < 2 * MT)
      dma16s((next ? nxtA : curA) + ko, offA[e], dma_base + slot * SLOT + e * 4096);
    else
      dma16s((next ? nxtB : curB) + ko, offB[e - 2 * MT],
             dma_base + slot * SLOT + BM * BKW + (e - 2 * MT) * 4096);
  };

  // Fragment reads.  Lane (row r' = l & 31, half h = l >> 5) of fragment e reads piece
  // 2 ks + h of row 32 e + r' (+ the wavefront's offset); the swizzle only depends on r'.
  // The per-lane LDS address of (operand, ks) is kept in a register; slot and fragment are
  // added as one opaque base per half-slab plus an immediate, so that the compiler cannot
  // turn the 64 (slot, ks, fragment) addresses into 64 registers hoisted out of the loops.
  const int frow = lane & 31, fh = lane >> 5, swz = (frow >> 1) & 7;
  unsigned a_ks[4], b_ks[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const int off = ((2 * ks + fh) ^ swz) * 16;
    a_ks[ks] = (unsigned)((wm * 128 + frow) * BKW + off);
    b_ks[ks] = (unsigned)(BM * BKW + (wn * 128 + frow) * BKW + off);
  }
  unsigned rd_a = 0, rd_b = 0;               // bases of the half-slab's reads (bytes into the ring)
  auto read_base = [&](int slot, int ks) {    // slot, ks compile-time
    rd_a = a_ks[ks] + (unsigned)(slot * SLOT);
    rd_b = b_ks[ks] + (unsigned)(slot * SLOT);
    asm volatile("" : "+v"(rd_a), "+v"(rd_b));
  };
  auto read_piece = [&](Frags<MT, NT>& f, int e) {   // e compile-time
    if (e < MT)
      f.a[e] = *reinterpret_cast<const uint4*>(&ring[rd_a + (unsigned)(e * 4096)]);
    else
      f.b[e - MT] = *reinterpret_cast<const uint4*>(&ring[rd_b + (unsigned)((e - MT) * 4096)]);
  };

  Frags<MT, NT> f0;                         // the two that cross a tile boundary: the first
  Operands<MT, NT> s0;                      // slab of the next stage, read and half expanded
  u32 hi;                                   // 0xF0F0F0F0 in a scalar register
  asm volatile("s_mov_b32 %0, 0xf0f0f0f0" : "=s"(hi));

  // sources that are valid to load from whether or not the optional arrays exist
  const float* bias_src = bias ? bias : w_scale;
  const float* gid_src = reinterpret_cast<const float*>(gid ? gid : reinterpret_cast<const int*>(scale));
  // Scalars of a tile -- token-set id and scale of row tid, scale and bias of column tid --
  // travel global -> LDS by direct loads as well, so no register holds them while the
  // matrix stream runs: `ids` and the column entries first; one stage later (the ids have
  // landed) the row scales that depend on them.  Image of a row: floor((m + 1/2) / T) in
  // binary64, exact for m, T < 2^31.  The id is clamped into range before it indexes the
  // scales.
  const unsigned lds_of_wave = (unsigned)(wave * 256);
  auto lds_addr = [&](const void* ptr) {
    return __builtin_amdgcn_readfirstlane(
        (unsigned)(size_t)(__attribute__((address_space(3))) const uint8_t*)ptr + lds_of_wave);
  };
  auto fetch_ids_cols = [&](int set, int m_first, int n_first) {
    dma4s(gid_src, gid ? (unsigned)(m_first + tid) * 4u : 0u, lds_addr(sGid));
    dma4s(w_scale, (unsigned)(n_first + tid) * 4u, lds_addr(sCol[set]));
    dma4s(bias_src, (unsigned)(n_first + tid) * 4u, lds_addr(sBias[set]));
  };
  auto fetch_row_scales = [&](int set, int m_first) {
    int g = gid ? sGid[tid] : 0;
    g = g < 0 ? 0 : (g > G - 1 ? G - 1 : g);
    const int img = (int)(((double)(m_first + tid) + 0.5) * inv_T);
    dma4s(scale, (unsigned)(img * G + g) * 4u, lds_addr(sRow[set]));
  };

  // ---- first tile: fill the stream
  {
#pragma unroll
    for (int e = 0; e < 2 * NB; ++e) dma_piece(0, 0, e);
#pragma unroll
    for (int e = 0; e < NB; ++e) dma_piece(1, 1, e);
    fetch_ids_cols(0, tile_m0(0), tile_n0(0));
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    fetch_row_scales(0, tile_m0(0));
    read_base(0, 0);
#pragma unroll
    for (int e = 0; e < NB; ++e) read_piece(f0, e);
#pragma unroll
    for (int e = 0; e < NB; ++e) expand_one<0>(s0, f0, e, hi);
  }

  // One stage; see k_w4a4_gemm_wide.  FIRST: the tile's first stage (fresh accumulators).
#define TDQ_RSTAGE(kt, CUR, OTH, FIRST, AFTER_BARRIER)                                            \
  do {                                                                                           \
    __builtin_amdgcn_sched_barrier(0);                                                           \
    read_base(CUR, 1);                                                                           \
    half_slab<1, MT, NT, FIRST>(acc, s0, s1, f0, hi, [&](int b) { read_piece(f1, b); });         \
    half_slab<0>(acc, s1, s0, f1, hi, [&](int b) { dma_piece(OTH, (kt) + 1, NB + b); });         \
    read_base(CUR, 2);                                                                           \
    half_slab<1>(acc, s0, s1, f1, hi, [&](int b) { read_piece(f0, b); });                        \
    half_slab<0>(acc, s1, s0, f0, hi, [&](int) {});                                              \
    read_base(CUR, 3);                                                                           \
    half_slab<1>(acc, s0, s1, f0, hi, [&](int b) { read_piece(f1, b); });                        \
    half_slab<0>(acc, s1, s0, f1, hi, [&](int) {});                                              \
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");                                  \
    __syncthreads();                                                                             \
    __builtin_amdgcn_sched_barrier(0);                                                           \
    AFTER_BARRIER;                                                                               \
    read_base(OTH, 0);                                                                           \
    __builtin_amdgcn_sched_barrier(0);                                                           \
    half_slab<1>(acc, s0, s1, f1, hi, [&](int b) { read_piece(f0, b); });                        \
    half_slab<0>(acc, s1, s0, f0, hi, [&](int b) { dma_piece(CUR, (kt) + 2, b); });              \
  } while (0)

  for (int it = 0; it < n_my; ++it) {
    v16i acc[MT][NT];                       // started afresh by the tile's first half-slab
    Frags<MT, NT> f1;
    Operands<MT, NT> s1;
    const int m0 = tile_m0(it), n0 = tile_n0(it);
    const bool more = it + 1 < n_my;
    if (more) {
      nxtA = Qx + (long long)tile_m0(it + 1) * ld_q;
      nxtB = Qw + (long long)tile_n0(it + 1) * ld_w;
    }
    // The next tile's scalars are fetched in this tile's last two stages (straight-line
    // code: the stages before and inside the loop simply carry no fetch) and land before the
    // next tile's first stage barrier, long before its output phase.  After the last tile
    // they re-fetch its own.
    const int set = it & 1;
    const int nm0 = tile_m0(more ? it + 1 : it), nn0 = tile_n0(more ? it + 1 : it);
    TDQ_RSTAGE(0, 0, 1, true, (void)0);
    TDQ_RSTAGE(1, 1, 0, false, (void)0);
    for (int kt = 2; kt < k_tiles - 2; kt += 2) {
      TDQ_RSTAGE(kt, 0, 1, false, (void)0);
      TDQ_RSTAGE(kt + 1, 1, 0, false, (void)0);
    }
    // the tile's last two stages carry the fetches: ids and column entries first, one stage
    // (and its barrier's wait for every load) later the row scales that read the ids
    TDQ_RSTAGE(k_tiles - 2, 0, 1, false, fetch_ids_cols(set ^ 1, nm0, nn0));
    TDQ_RSTAGE(k_tiles - 1, 1, 0, false, fetch_row_scales(set ^ 1, nm0));
    // Output phase of this tile (whole tiles only).  The lane index is made opaque per
    // tile: everything the output phase derives from it would otherwise be hoisted out of
    // the tile loop and live in (spilled) registers throughout the matrix stream.
    {
      int lane_o = lane;
      asm volatile("" : "+v"(lane_o));
      OUT* wtile = Y + (long long)(m0 + wm * 128) * ld_y + (n0 + wn * 128);
      if (bias)
        tile_store_cols4<OUT, true>(acc, sRow[set], sCol[set], sBias[set], lane_o, wm, wn, wtile, ld_y);
      else
        tile_store_cols4<OUT, false>(acc, sRow[set], sCol[set], sBias[set], lane_o, wm, wn, wtile, ld_y);
    }
    curA = nxtA;
    curB = nxtB;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // nothing of ours may still be landing
#undef TDQ_RSTAGE
}

template <typename OUT, int MT, int NT>
static void launch_tile(const uint8_t* Qx, long long ld_q, const int* gid, const float* scale, int M,
                        int T, int K, int N, int G, const uint8_t* Qw, long long ld_w,
                        const float* w_scale, const float* bias, void* Y, long long ld_y,
                        int* acc_dump, hipStream_t st) {
  constexpr int BM = 64 * MT, BN = 64 * NT;
  const int m_tiles = (M + BM - 1) / BM, n_tiles = (N + BN - 1) / BN;
  const long long m_groups = (m_tiles + XCDS - 1) / XCDS;
  const unsigned grid = (unsigned)(m_groups * XCDS * n_tiles);
  hipLaunchKernelGGL((k_w4a4_gemm<OUT, MT, NT>), dim3(grid), dim3(GEMM_THREADS), 0, st, Qx, ld_q,
                     gid, scale, M, T, K, N, G, Qw, ld_w, w_scale, bias, static_cast<OUT*>(Y), ld_y,
                     acc_dump, m_tiles, n_tiles);
}

template <typename OUT, int MT, int NT>
static void launch_pipe(const uint8_t* Qx, long long ld_q, const int* gid, const float* scale, int M,
                        int T, int K, int N, int G, const uint8_t* Qw, long long ld_w,
                        const float* w_scale, const float* bias, void* Y, long long ld_y,
                        int* acc_dump, hipStream_t st) {
  constexpr int BM = 64 * MT, BN = 64 * NT;
  const int m_tiles = (M + BM - 1) / BM, n_tiles = (N + BN - 1) / BN;
  const long long m_groups = (m_tiles + XCDS - 1) / XCDS;
  const unsigned grid = (unsigned)(m_groups * XCDS * n_tiles);
  hipLaunchKernelGGL((k_w4a4_gemm_pipe<OUT, MT, NT>), dim3(grid), dim3(GEMM_THREADS), 0, st, Qx,
                     ld_q, gid, scale, M, T, K, N, G, Qw, ld_w, w_scale, bias, static_cast<OUT*>(Y),
                     ld_y, acc_dump, m_tiles, n_tiles);
}

template <typename OUT>
static void launch_wide(const uint8_t* Qx, long long ld_q, const int* gid, const float* scale, int M,
                        int T, int K, int N, int G, const uint8_t* Qw, long long ld_w,
                        const float* w_scale, const float* bias, void* Y, long long ld_y,
                        int* acc_dump, hipStream_t st) {
  const int m_tiles = (M + 255) / 256, n_tiles = (N + 255) / 256;
  const long long m_groups = (m_tiles + XCDS - 1) / XCDS;
  const unsigned grid = (unsigned)(m_groups * XCDS * n_tiles);
  hipLaunchKernelGGL((k_w4a4_gemm_wide<OUT>), dim3(grid), dim3(GEMM_THREADS), 0, st, Qx, ld_q, gid,
                     scale, M, T, K, N, G, Qw, ld_w, w_scale, bias, static_cast<OUT*>(Y), ld_y,
                     acc_dump, m_tiles, n_tiles);
}

// Compute units of the current device (0 if the query fails), looked up once per device.
static int compute_units() {
  static int cached[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
  int cu = __atomic_load_n(&cached[dev], __ATOMIC_RELAXED);
  if (cu == 0) {
    if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    __atomic_store_n(&cached[dev], cu, __ATOMIC_RELAXED);
  }
  return cu;
}

template <typename OUT>
static void launch_roll(const uint8_t* Qx, long long ld_q, const int* gid, const float* scale, int M,
                        int T, int K, int N, int G, const uint8_t* Qw, long long ld_w,
                        const float* w_scale, const float* bias, void* Y, long long ld_y, int wgs,
                        hipStream_t st) {
  hipLaunchKernelGGL((k_w4a4_gemm_roll<OUT>), dim3(wgs), dim3(GEMM_THREADS), 0, st, Qx, ld_q, gid,
                     scale, M, T, K, N, G, Qw, ld_w, w_scale, bias, static_cast<OUT*>(Y), ld_y,
                     M / 256, N / 256, 1.0 / (double)T);
}

hipError_t launch_w4a4_gemm(const uint8_t* Qx, long long ld_q, const int* gid, const float* scale,
                            int M, int T, int K, int N, int G, const uint8_t* Qw, long long ld_w,
                            const float* w_scale, const float* bias, void* Y, tdq_dtype y_dt,
                            long long ld_y, int* acc_dump, hipStream_t st) {
  const long long big_tiles = (long long)((M + 255) / 256) * ((N + 255) / 256);
  // Whole tiles only, an even number of 256-code stages, rows of tiles in multiples of the
  // 8 XCDs, and at least 8 tiles for each of one persistent workgroup per CU: the rolling
  // kernel.  (One workgroup fits a CU, so more workgroups than CUs would run in turns.)
  if (!acc_dump && M % 256 == 0 && N % 256 == 0 && K % 512 == 0 && K >= 1024 && (M / 256) % XCDS == 0 &&
      256ll * ld_q < (1ll << 32) && 256ll * ld_w < (1ll << 32) && ld_y % 4 == 0 &&
      132ll * ld_y * (y_dt == TDQ_F32 ? 4 : 2) < (1ll << 32) &&      // 32-bit store offsets inside 128 rows
      reinterpret_cast<uintptr_t>(Y) % (y_dt == TDQ_F32 ? 16 : 8) == 0) {
    const int wgs = (compute_units() / XCDS) * XCDS;
    if (wgs >= XCDS && big_tiles >= 8ll * wgs) {
      if (y_dt == TDQ_F32)
        launch_roll<float>(Qx, ld_q, gid, scale, M, T, K, N, G, Qw, ld_w, w_scale, bias, Y, ld_y, wgs, st);
      else
        launch_roll<_Float16>(Qx, ld_q, gid, scale, M, T, K, N, G, Qw, ld_w, w_scale, bias, Y, ld_y,
                              wgs, st);
      return hipGetLastError();
    }
  }
  // big tiles once they can fill the 256 CUs at least twice over; the pipelined kernels
  // need whole stages of K: 256 codes (measured 2 to 3 % faster), else 128
  const int mode = big_tiles >= 512 ? (K % 256 == 0 ? 3 : K % 128 == 0 ? 2 : 1) : 0;
#define TDQ_GEMM(OUT, MT, NT)                                                                   \
  launch_tile<OUT, MT, NT>(Qx, ld_q, gid, scale, M, T, K, N, G, Qw, ld_w, w_scale, bias, Y, ld_y, \
                           acc_dump, st)
#define TDQ_GEMM_MODES(OUT)                                                                      \
  switch (mode) {                                                                                \
    case 3:                                                                                      \
      launch_wide<OUT>(Qx, ld_q, gid, scale, M, T, K, N, G, Qw, ld_w, w_scale, bias, Y, ld_y,    \
                       acc_dump, st);                                                            \
      break;                                                                                     \
    case 2:                                                                                      \
      launch_pipe<OUT, 4, 4>(Qx, ld_q, gid, scale, M, T, K, N, G, Qw, ld_w, w_scale, bias, Y,    \
                             ld_y, acc_dump, st);                                                \
      break;                                                                                     \
    case 1: TDQ_GEMM(OUT, 4, 4); break;                                                          \
    default: TDQ_GEMM(OUT, 2, 2); break;                                                         \
  }
  if (y_dt == TDQ_F32) { TDQ_GEMM_MODES(float) } else { TDQ_GEMM_MODES(_Float16) }
#undef TDQ_GEMM_MODES
#undef TDQ_GEMM
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Block-scaled contraction for the paper-literal granularity (Supp. Algorithm 1, step 10
// with one step Delta[m, kb] per token m and block kb of g = 32 channels):
//   Y[m, n] = s_w[n] * sum_kb Delta[m, kb] * acc_kb[m, n],
//   acc_kb[m, n] = sum_{i in block kb} Qx[m, i] * Qw[n, i]   (|acc_kb| <= 32 * 64)
// The int32 accumulation cannot run over the whole of K any more: one matrix
// instruction (K = 32) is exactly one block, and its 16 results per lane are converted
// and folded into a binary32 accumulator with the block's step,
//   f <- fma(float(acc_kb), Delta[m, kb], f),   kb ascending,
// i.e. 32 vector operations per matrix instruction: this kernel is bound by the vector
// unit, not by the matrix cores (which idle three quarters of the time).  The factor 256
// of the nibble expansion is taken out once at the end (a power of two: exact).
//
// Workgroup = 2 x 2 wavefronts, wavefront tile 64 x 64, 128 x 128 per workgroup, two
// workgroups per CU; a stage is SBY packed bytes (SBY / 16 blocks) of K per row,
// register-staged and double-buffered.  LDS rows are SBY + 8 bytes apart: the 8-byte
// fragment reads of 32 consecutive rows then fall on 32 different bank pairs.  The steps
// of a stage sit in LDS block-major so that the 4 consecutive rows a lane owns are one
// 16-byte read.
// ---------------------------------------------------------------------------
template <typename OUT, int SBY>
__global__ __launch_bounds__(GEMM_THREADS, 2) void k_w4a4_gemm_blocks(
    const uint8_t* __restrict__ Qx, long long ld_q, const float* __restrict__ bscale, long long ld_s,
    int M, int K, int N, const uint8_t* __restrict__ Qw, long long ld_w,
    const float* __restrict__ w_scale, const float* __restrict__ bias, OUT* __restrict__ Y,
    long long ld_y, int m_tiles, int n_tiles) {
  constexpr int MT = 2, NT = 2, BM = 128, BN = 128;
  constexpr int SB = SBY / 16;                         // blocks (= 16-byte pieces) per stage
  constexpr int STRIDE = SBY + 8;
  constexpr int RPP = GEMM_THREADS / SB;               // rows per staging pass
  constexpr int PASSES = BM / RPP;
  constexpr int DPT = SB / 2;                          // steps per thread and stage
  __shared__ __attribute__((aligned(16))) uint8_t sA[2][BM * STRIDE];
  __shared__ __attribute__((aligned(16))) uint8_t sB[2][BN * STRIDE];
  __shared__ __attribute__((aligned(16))) float sD[2][SB][BM];
  __shared__ float sCol[BN], sBias[BN];

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
  const int KB = (K + 31) / 32;
  const int k_tiles = (kbytes + SBY - 1) / SBY;

  for (int j = tid; j < BN; j += GEMM_THREADS) {
    const int n = n0 + j;
    sCol[j] = n < N ? w_scale[n] : 0.f;
    sBias[j] = (bias && n < N) ? bias[n] : 0.f;
  }

  // staging: thread t owns the 16-byte piece t % SB of rows t / SB + RPP i of both
  // operands, and DPT consecutive steps of row t / 2
  const int pr0 = tid / SB, pc = (tid % SB) * 16;
  const uint8_t* pa[PASSES];
  const uint8_t* pb[PASSES];
#pragma unroll
  for (int i = 0; i < PASSES; ++i) {
    int r = m0 + pr0 + RPP * i;
    r = r < M ? r : M - 1;
    pa[i] = Qx + (long long)r * ld_q + pc;
    r = n0 + pr0 + RPP * i;
    r = r < N ? r : N - 1;
    pb[i] = Qw + (long long)r * ld_w + pc;
  }
  const int drow = tid >> 1, dcol = (tid & 1) * DPT;
  const bool d_row_ok = m0 + drow < M;
  const float* pd = bscale + (long long)(m0 + (d_row_ok ? drow : 0)) * ld_s + dcol;

  uint4 ga[PASSES], gb[PASSES];
  float gd[DPT];
  auto load_stage = [&](int kt) {
    const int kb = kt * SBY + pc;          // first packed byte of this piece
    if ((kt + 1) * SBY <= kbytes) {        // a whole stage inside the rows (uniform)
#pragma unroll
      for (int i = 0; i < PASSES; ++i) {
        ga[i] = *reinterpret_cast<const uint4*>(pa[i] + (long long)kt * SBY);
        gb[i] = *reinterpret_cast<const uint4*>(pb[i] + (long long)kt * SBY);
      }
    } else if (kb < kbytes) {
#pragma unroll
      for (int i = 0; i < PASSES; ++i) {
        ga[i] = *reinterpret_cast<const uint4*>(pa[i] + (long long)kt * SBY);
        gb[i] = *reinterpret_cast<const uint4*>(pb[i] + (long long)kt * SBY);
      }
      if (kb + 16 > kbytes) {              // piece straddles the end of the row: zero the rest
        const int keep = kbytes - kb;
#pragma unroll
        for (int i = 0; i < PASSES; ++i) {
          mask_piece(ga[i], keep);
          mask_piece(gb[i], keep);
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < PASSES; ++i) {
        ga[i] = make_uint4(0, 0, 0, 0);
        gb[i] = make_uint4(0, 0, 0, 0);
      }
    }
    // 4-byte loads, not 16-byte ones: every lane pair reads its own row here, and a
    // 16-byte load whose 64 lanes fall on 64 different 128-byte lines was measured to
    // slow the whole kernel down tenfold on this chip.
    const int b0 = kt * SB + dcol;         // first block of this thread's steps
#pragma unroll
    for (int j = 0; j < DPT; ++j) gd[j] = (d_row_ok && b0 + j < KB) ? pd[kt * SB + j] : 0.f;
  };
  auto store_stage = [&](int buf) {
#pragma unroll
    for (int i = 0; i < PASSES; ++i) {
      uint2* d = reinterpret_cast<uint2*>(&sA[buf][(pr0 + RPP * i) * STRIDE + pc]);
      d[0] = make_uint2(ga[i].x, ga[i].y);
      d[1] = make_uint2(ga[i].z, ga[i].w);
      d = reinterpret_cast<uint2*>(&sB[buf][(pr0 + RPP * i) * STRIDE + pc]);
      d[0] = make_uint2(gb[i].x, gb[i].y);
      d[1] = make_uint2(gb[i].z, gb[i].w);
    }
#pragma unroll
    for (int j = 0; j < DPT; ++j) sD[buf][dcol + j][drow] = gd[j];
  };

  float accf[MT][NT][16];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) accf[i][j][r] = 0.f;

  load_stage(0);
  store_stage(0);
  __syncthreads();

  // Lane l feeds row (l & 31) of a 32-row fragment and, of each 16-byte block of K, the
  // 8 bytes at offset 8 (l >> 5); it owns column l & 31 and rows 8 q + 4 (l >> 5) + 0..3,
  // q = 0..3, of every 32 x 32 result.
  const int frow = lane & 31, fhalf = (lane >> 5) * 8;
  const int a_off = (wm * 32 * MT + frow) * STRIDE + fhalf;
  const int b_off = (wn * 32 * NT + frow) * STRIDE + fhalf;
  const int d_off = wm * 32 * MT + (lane >> 5) * 4;
  const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  for (int kt = 0; kt < k_tiles; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < k_tiles) load_stage(kt + 1);
    // one block at a time: unrolled further, the loads of all blocks are hoisted and
    // the accumulators spill
#pragma unroll 1
    for (int kb = 0; kb < SB; ++kb) {
      v4i a[MT], b[NT];
      float dl[MT][16];
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        const uint2 f = *reinterpret_cast<const uint2*>(&sA[cur][a_off + i * 32 * STRIDE + kb * 16]);
        a[i] = expand(f.x, f.y);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float4 d4 = *reinterpret_cast<const float4*>(&sD[cur][kb][d_off + i * 32 + q * 8]);
          dl[i][4 * q] = d4.x; dl[i][4 * q + 1] = d4.y; dl[i][4 * q + 2] = d4.z; dl[i][4 * q + 3] = d4.w;
        }
      }
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const uint2 f = *reinterpret_cast<const uint2*>(&sB[cur][b_off + j * 32 * STRIDE + kb * 16]);
        b[j] = expand(f.x, f.y);
      }
      v16i t[MT][NT];
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
          t[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], zero, 0, 0, 0);
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            accf[i][j][r] = __builtin_fmaf((float)t[i][j][r], dl[i][r], accf[i][j][r]);
    }
    if (kt + 1 < k_tiles) store_stage(cur ^ 1);
    __syncthreads();
  }

  const int ccol = lane & 31, rquad = (lane >> 5) * 4;
  if (m0 + BM <= M && n0 + BN <= N && (long long)(BM + 8) * ld_y < (1ll << 31) / (long long)sizeof(OUT)) {
    // whole tile inside Y: a wavefront-uniform row pointer plus one per-lane offset, two
    // rows at a time, the NT column blocks of a row back to back (whole lines of Y)
    const unsigned lane_offu = (unsigned)(rquad * (int)ld_y + ccol);
    auto body = [&](auto with_bias) {
      float ws[NT], bs[NT];
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        ws[j] = sCol[wn * 32 * NT + j * 32 + ccol];
        bs[j] = sBias[wn * 32 * NT + j * 32 + ccol];
      }
      OUT* wtile = Y + (long long)(m0 + wm * 32 * MT) * ld_y + (n0 + wn * 32 * NT);
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          OUT* row0 = wtile + (long long)(i * 32 + (r >> 2) * 8 + (r & 3)) * ld_y + lane_offu;
          OUT* row1 = row0 + ld_y;
          float y0[NT], y1[NT];
#pragma unroll
          for (int j = 0; j < NT; ++j) {
            y0[j] = (accf[i][j][r] * 0.00390625f) * ws[j];
            y1[j] = (accf[i][j][r + 1] * 0.00390625f) * ws[j];
            if (decltype(with_bias)::value) {
              y0[j] = y0[j] + bs[j];
              y1[j] = y1[j] + bs[j];
            }
          }
          if constexpr (sizeof(OUT) == 2) {
            h2v p[NT];
#pragma unroll
            for (int j = 0; j < NT; ++j) p[j] = round_pair_to_half(y0[j], y1[j]);
#pragma unroll
            for (int j = 0; j < NT; ++j) __builtin_nontemporal_store(p[j][0], row0 + j * 32);
#pragma unroll
            for (int j = 0; j < NT; ++j) __builtin_nontemporal_store(p[j][1], row1 + j * 32);
          } else {
#pragma unroll
            for (int j = 0; j < NT; ++j) store_out<OUT>(row0 + j * 32, y0[j]);
#pragma unroll
            for (int j = 0; j < NT; ++j) store_out<OUT>(row1 + j * 32, y1[j]);
          }
        }
    };
    if (bias)
      body(std::true_type{});
    else
      body(std::false_type{});
    return;
  }
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int rl = wm * 32 * MT + i * 32 + (r >> 2) * 8 + rquad + (r & 3);
      const int m = m0 + rl;
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int cl = wn * 32 * NT + j * 32 + ccol;
        const int n = n0 + cl;
        if (m < M && n < N) {
          float y = (accf[i][j][r] * 0.00390625f) * sCol[cl];
          if (bias) y = y + sBias[cl];
          store_out<OUT>(Y + (long long)m * ld_y + n, y);
        }
      }
    }
}

constexpr int kBlkStageBytes = 128;      // packed bytes of K per stage of the block-scaled kernel
hipError_t launch_w4a4_gemm_blocks(const uint8_t* Qx, long long ld_q, const float* bscale,
                                   long long ld_s, int M, int K, int N, const uint8_t* Qw,
                                   long long ld_w, const float* w_scale, const float* bias, void* Y,
                                   tdq_dtype y_dt, long long ld_y, hipStream_t st) {
  const int m_tiles = (M + 127) / 128, n_tiles = (N + 127) / 128;
  const long long m_groups = (m_tiles + XCDS - 1) / XCDS;
  const unsigned grid = (unsigned)(m_groups * XCDS * n_tiles);
  if (y_dt == TDQ_F32)
    hipLaunchKernelGGL((k_w4a4_gemm_blocks<float, kBlkStageBytes>), dim3(grid), dim3(GEMM_THREADS), 0, st, Qx, ld_q,
                       bscale, ld_s, M, K, N, Qw, ld_w, w_scale, bias, static_cast<float*>(Y), ld_y,
                       m_tiles, n_tiles);
  else
    hipLaunchKernelGGL((k_w4a4_gemm_blocks<_Float16, kBlkStageBytes>), dim3(grid), dim3(GEMM_THREADS), 0, st, Qx,
                       ld_q, bscale, ld_s, M, K, N, Qw, ld_w, w_scale, bias,
                       static_cast<_Float16*>(Y), ld_y, m_tiles, n_tiles);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// The contraction on the 6-bit matrix format of gfx950.  The sixteen int4 codes are all
// exactly representable in bf6 (e3m2: 1 sign, 3 exponent, 2 mantissa bits), products and
// sums of integers below 2^24 are exact in the binary32 accumulator, and
// v_mfma_scale_f32_32x32x64_f8f6f4 with unit scales runs at twice the int8 rate per
// instruction (K = 64 in the time the int8 instruction takes for K = 32) with no nibble
// expansion in the loop: measured register-only on random codes 5.3 POP/s against 3.2
// for the int8 instruction (the clock drops less under its load).
//
// Operand storage ("f6 fragments"): rows in blocks of 32, K in blocks of 64; the block
// (rb, kb) is 1536 contiguous bytes at ((rb * KB + kb) * 1536), KB = number of 64-blocks
// of K (even, zero-padded), holding the 64 lanes' operands of ONE matrix instruction in
// lane order: lane l = (row % 32) + 32 * ((k % 64) / 32) owns 24 bytes, code j = k % 32
// in bits [6 j, 6 j + 6) (little endian).  A workgroup's stage (128 codes of K for 256
// rows of each operand) is 16 chunks of 3072 contiguous bytes, copied by 48 direct-to-LDS
// loads of 1 KiB, and a lane reads its operand as three 8-byte LDS reads, 24 bytes apart
// from its neighbours': conflict-free without any swizzle.
// ---------------------------------------------------------------------------
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
constexpr int F6_FRAG = 1536;            // bytes of one (32 rows, 64 codes) block

// Packed nibbles [R, ld] -> f6 fragments.  One wavefront per fragment (32 rows x 64 codes),
// the four wavefronts of a workgroup on four consecutive fragments of the same rows, so
// that together they read whole 128-byte lines.  Lane l loads the 16 bytes of (row l / 2,
// half l % 2), the lane that owns (row, half) in the fragment's order fetches them with a
// lane permute, sign-extends the 32 nibbles, and one conversion instruction (even codes
// in its first operand, odd ones in its second) packs them.  Codes at and beyond K, rows
// at and beyond R are zero.
typedef int v6i_pack __attribute__((ext_vector_type(6)));
__global__ __launch_bounds__(256) void k_pack_f6(const uint8_t* __restrict__ Q, long long ld, int R,
                                                 int K, int KB, long long n_blocks, int vec_ok,
                                                 uint8_t* __restrict__ F) {
  const int l = threadIdx.x & 63;
  const long long blk = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (blk >= n_blocks) return;                             // whole wavefronts only
  const int kb = (int)(blk % KB);
  const long long rb = blk / KB;
  const long long row = rb * 32 + (l >> 1);
  const int k0 = kb * 64 + 32 * (l & 1);
  u32 n[4] = {0u, 0u, 0u, 0u};
  if (row < R && k0 < K) {
    const uint8_t* src = Q + row * ld + k0 / 2;
    const int live = K - k0;                               // codes of this piece that exist
    const int nb = live >= 32 ? 16 : (live + 1) / 2;       // bytes that hold them
    if (vec_ok && nb == 16) {
      const uint4 q = *reinterpret_cast<const uint4*>(src);
      n[0] = q.x; n[1] = q.y; n[2] = q.z; n[3] = q.w;
    } else {
      for (int j = 0; j < nb; ++j) n[j >> 2] |= (u32)src[j] << (8 * (j & 3));
    }
    if (live < 32) {                                       // the pad nibble of an odd K is not a code
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const int keep = live - 8 * w;
        n[w] &= keep >= 8 ? 0xFFFFFFFFu : (keep <= 0 ? 0u : (1u << (4 * keep)) - 1u);
      }
    }
  }
  const int from = (2 * (l & 31) + (l >> 5)) * 4;          // the lane that loaded this lane's piece
  u32 m[4];
#pragma unroll
  for (int w = 0; w < 4; ++w) m[w] = (u32)__builtin_amdgcn_ds_bpermute(from, (int)n[w]);
  v16f ev, od;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const u32 wd = m[i >> 2];
    const int sh = 8 * (i & 3);                            // codes 2 i and 2 i + 1: bits sh, sh + 4
    ev[i] = (float)((int)(wd << (28 - sh)) >> 28);
    od[i] = (float)((int)(wd << (24 - sh)) >> 28);
  }
  const v6i_pack r = __builtin_amdgcn_cvt_scalef32_2xpk16_bf6_f32(ev, od, 1.0f);
  uint2* dst = reinterpret_cast<uint2*>(F + (blk * 64 + l) * 24);
  dst[0] = make_uint2((u32)r[0], (u32)r[1]);
  dst[1] = make_uint2((u32)r[2], (u32)r[3]);
  dst[2] = make_uint2((u32)r[4], (u32)r[5]);
}

hipError_t launch_pack_f6(const uint8_t* Q, long long ld, int R, int K, uint8_t* F, hipStream_t st) {
  const int KB = 2 * ((K + 127) / 128);
  const long long n_blocks = (long long)((R + 31) / 32) * KB;
  const int vec_ok = ((reinterpret_cast<uintptr_t>(Q) & 15) == 0 && ld % 16 == 0) ? 1 : 0;
  hipLaunchKernelGGL(k_pack_f6, dim3((unsigned)((n_blocks + 3) / 4)), dim3(256), 0, st, Q, ld, R, K, KB,
                     n_blocks, vec_ok, F);
  return hipGetLastError();
}

template <typename OUT>
__global__ __launch_bounds__(GEMM_THREADS, 1) void k_w4a4_gemm_f6(
    const uint8_t* __restrict__ A6, const uint8_t* __restrict__ B6, int KB,
    const int* __restrict__ gid, const float* __restrict__ scale, int M, int T, int N, int G,
    const float* __restrict__ w_scale, const float* __restrict__ bias, OUT* __restrict__ Y,
    long long ld_y, int* __restrict__ acc_dump, int m_tiles, int n_tiles) {
  constexpr int MT = 4, NT = 4, BM = 256, BN = 256;
  constexpr int KS = 2;                          // 64-blocks of K per stage
  constexpr int CH = KS * F6_FRAG;               // one row block's bytes of a stage
  constexpr int SLOT = 16 * CH;                  // 8 row blocks of A, then 8 of B: 48 KiB
  constexpr int NDMA = SLOT / 1024 / 4;          // direct loads per wavefront and stage: 12
  __shared__ __attribute__((aligned(1024))) uint8_t ring[3 * SLOT];
  __shared__ __attribute__((aligned(16))) float sRow[BM], sCol[BN], sBias[BN];

  const int bid = blockIdx.x;
  const int xcd = bid % XCDS, idx = bid / XCDS;
  const int m_tile = (idx / n_tiles) * XCDS + xcd;
  const int n_tile = idx % n_tiles;
  if (m_tile >= m_tiles) return;
  const int m0 = m_tile * BM, n0 = n_tile * BN;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int stages = KB / KS;                    // KB is even
  const int MBk = (M + 31) / 32, NBk = (N + 31) / 32;

  // piece pi = wave + 4 e of a stage: chunk pi / 3 (row block), 1 KiB part pi % 3
  const uint8_t* src[NDMA];
#pragma unroll
  for (int e = 0; e < NDMA; ++e) {
    const int pi = wave + 4 * e;
    const int c = pi / 3, part = pi % 3;
    long long rb;
    const uint8_t* base;
    if (c < 8) {
      rb = (long long)m_tile * 8 + c;
      rb = rb < MBk ? rb : MBk - 1;              // past the end: a harmless re-read
      base = A6;
    } else {
      rb = (long long)n_tile * 8 + (c - 8);
      rb = rb < NBk ? rb : NBk - 1;
      base = B6;
    }
    src[e] = base + rb * KB * F6_FRAG + part * 1024 + lane * 16;
  }
  const unsigned ring_base = (unsigned)(size_t)(__attribute__((address_space(3))) uint8_t*)ring;
  {
    const int my_m = m0 + tid < M ? m0 + tid : M - 1;
    const int my_g = gid ? gid[my_m] : 0;
    sRow[tid] = scale[(long long)(my_m / T) * G + my_g];
    const int n = n0 + tid;
    sCol[tid] = n < N ? w_scale[n] : 0.f;
    sBias[tid] = (bias && n < N) ? bias[n] : 0.f;
  }

  v16f acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int a_off = wm * 4 * CH + lane * 24, b_off = (8 + wn * 4) * CH + lane * 24;
  // fragment f of a K block: f < 4 the wavefront's row blocks of A, else of B
  auto read_frag = [&](v8i (&fa)[MT], v8i (&fb)[NT], int slot, int kk, int f) {   // all compile-time
    const int off = (f < MT ? a_off + f * CH : b_off + (f - MT) * CH) + kk * F6_FRAG;
    const uint2* p = reinterpret_cast<const uint2*>(&ring[slot * SLOT + off]);
    const uint2 q0 = p[0], q1 = p[1], q2 = p[2];
    const v8i v = {(int)q0.x, (int)q0.y, (int)q1.x, (int)q1.y, (int)q2.x, (int)q2.y, 0, 0};
    if (f < MT) fa[f] = v; else fb[f - MT] = v;
  };
  auto mma = [&](const v8i (&fa)[MT], const v8i (&fb)[NT], int t) {               // t compile-time
    acc[t >> 2][t & 3] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
        fa[t >> 2], fb[t & 3], acc[t >> 2][t & 3], 3, 3, 0, 127, 0, 127);
  };
  // stage st (clamped to the last one: past the end a harmless re-load) -> slot
  auto dma_piece = [&](int slot, int st, int e) {                                  // slot, e compile-time
    const int sc = st < stages ? st : stages - 1;
    dma16(src[e] + (long long)sc * CH,
          __builtin_amdgcn_readfirstlane(ring_base + slot * SLOT + (wave + 4 * e) * 1024));
  };

  // Three slots.  The instruction stream of stage s (slot s % 3; two K blocks, 32 matrix
  // instructions) is laid out by hand in bundles fenced with sched_barrier — one
  // wavefront per SIMD, nothing else hides latency — and has no branch (a branch would
  // end the basic block and with it the order):
  //   K block 0, 16 matrix instructions: the 8 fragments of K block 1 are read;
  //   wait until stage s + 1 has landed (all but the newest 12 loads), barrier: now every
  //     wavefront has read the last of slot s % 3, and stage s + 1 is whole;
  //   K block 1, 16 matrix instructions: the 8 fragments of K block 0 of stage s + 1 are
  //     read and the 12 direct loads of stage s + 3 are issued into slot s % 3 — two full
  //     stages (about 2000 cycles) before anything reads them.
  v8i a0[MT], b0[NT], a1[MT], b1[NT];
#pragma unroll
  for (int e = 0; e < NDMA; ++e) dma_piece(0, 0, e);
#pragma unroll
  for (int e = 0; e < NDMA; ++e) dma_piece(1, 1, e);
#pragma unroll
  for (int e = 0; e < NDMA; ++e) dma_piece(2, 2, e);
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * NDMA) : "memory");                  // stage 0 has landed
  __syncthreads();
#pragma unroll
  for (int f = 0; f < MT + NT; ++f) read_frag(a0, b0, 0, 0, f);

#define TDQ_F6_STAGE(s, CUR, NXT)                                                                \
  do {                                                                                           \
    _Pragma("unroll") for (int t = 0; t < 16; ++t) {                                             \
      __builtin_amdgcn_sched_barrier(0);                                                         \
      mma(a0, b0, t);                                                                            \
      if ((t & 1) == 0) read_frag(a1, b1, CUR, 1, t >> 1);                                       \
    }                                                                                            \
    __builtin_amdgcn_sched_barrier(0);                                                           \
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(NDMA) : "memory");                       \
    __syncthreads();                                                                             \
    _Pragma("unroll") for (int t = 0; t < 16; ++t) {                                             \
      __builtin_amdgcn_sched_barrier(0);                                                         \
      mma(a1, b1, t);                                                                            \
      if ((t & 1) == 0) read_frag(a0, b0, NXT, 0, t >> 1);                                       \
      else if (t < 12) { dma_piece(CUR, (s) + 3, t - 1); dma_piece(CUR, (s) + 3, t); }           \
    }                                                                                            \
    __builtin_amdgcn_sched_barrier(0);                                                           \
  } while (0)

  int s = 0;
  for (; s + 2 < stages; s += 3) {
    TDQ_F6_STAGE(s, 0, 1);
    TDQ_F6_STAGE(s + 1, 1, 2);
    TDQ_F6_STAGE(s + 2, 2, 0);
  }
  if (s < stages) {
    TDQ_F6_STAGE(s, 0, 1);
    if (s + 1 < stages) TDQ_F6_STAGE(s + 1, 1, 2);
  }
#undef TDQ_F6_STAGE
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");         // nothing of ours may still be landing

  pipe_epilogue<OUT, MT, NT, v16f>(acc, sRow, sCol, sBias, lane, wm, wn, m0, n0, M, N, bias, Y, ld_y,
                                   acc_dump);
}

hipError_t launch_w4a4_gemm_f6(const uint8_t* A6, const uint8_t* B6, int K, const int* gid,
                               const float* scale, int M, int T, int N, int G, const float* w_scale,
                               const float* bias, void* Y, tdq_dtype y_dt, long long ld_y,
                               int* acc_dump, hipStream_t st) {
  const int KB = 2 * ((K + 127) / 128);
  const int m_tiles = (M + 255) / 256, n_tiles = (N + 255) / 256;
  const long long m_groups = (m_tiles + XCDS - 1) / XCDS;
  const unsigned grid = (unsigned)(m_groups * XCDS * n_tiles);
  if (y_dt == TDQ_F32)
    hipLaunchKernelGGL((k_w4a4_gemm_f6<float>), dim3(grid), dim3(GEMM_THREADS), 0, st, A6, B6, KB, gid,
                       scale, M, T, N, G, w_scale, bias, static_cast<float*>(Y), ld_y, acc_dump, m_tiles,
                       n_tiles);
  else
    hipLaunchKernelGGL((k_w4a4_gemm_f6<_Float16>), dim3(grid), dim3(GEMM_THREADS), 0, st, A6, B6, KB,
                       gid, scale, M, T, N, G, w_scale, bias, static_cast<_Float16*>(Y), ld_y, acc_dump,
                       m_tiles, n_tiles);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// The block-scaled contraction (one step per row and 32-code block) on f6 fragments.
// The 6-bit instruction covers 64 codes = two blocks, lanes 0-31 supplying the even
// block and lanes 32-63 the odd one of an operand; zeroing the other half of one operand
// makes it deliver one block's sum, already as a float, so the rescale is one fused
// multiply-add per element and block (16 per matrix instruction) instead of a conversion
// and a multiply-add on top of the nibble expansion (38).  Same arithmetic as
// k_w4a4_gemm_blocks (f <- fma(acc_kb, Delta[m, kb], f), kb ascending): same bits.
//
// The weights are the instruction's row operand and the activations its column operand,
// so a lane holds ONE activation row m (= lane % 32) and 16 output channels: Delta[m, kb]
// is one register per lane instead of sixteen.
//
// 128 x 128 tile, 2 x 2 wavefronts of 64 x 64; a stage is 128 codes of K = four scale
// blocks = four "rounds" of 4 matrix instructions + 64 multiply-adds per wavefront.  The
// kernel is bound by the vector unit, so the two must overlap inside a wavefront: a round
// consumes the four results of the round before, one at a time, and re-issues the matrix
// instruction into the result registers just freed, so every result has three quarters
// of a round (about 200 cycles) to arrive and the vector unit never waits for the matrix
// pipe.  Operands of a round are read from LDS during the round before.
//   Ring of three slots of 24 KiB + the stage's scales [4][128], all by direct-to-LDS
//   loads (8 per wavefront and stage, no staging registers).  Everything read from the
//   slot of stage s is read by round 2 of stage s; the barrier in that round publishes
//   stage s + 1, and right behind it the loads of stage s + 3 go into the slot of stage
//   s: two full stages of flight.  A half-zero operand is read as such: the lanes of the
//   unwanted half read 24 zero bytes (one multiply-add on the address, no selects on the
//   data).  No branch inside the stage: a branch would end the basic block and the
//   compiler would regroup the instructions.
// ---------------------------------------------------------------------------

template <typename OUT>
__global__ __launch_bounds__(GEMM_THREADS, 2) void k_w4a4_gemm_blocks_f6(
    const uint8_t* __restrict__ A6, const uint8_t* __restrict__ B6, int KB64,
    const float* __restrict__ bscale, long long ld_s, int M, int K, int N,
    const float* __restrict__ w_scale, const float* __restrict__ bias, OUT* __restrict__ Y,
    long long ld_y, int m_tiles, int n_tiles, int y_vec_ok) {
  // WM x 2 wavefronts of 64 x 64.  (WM = 4, one workgroup of 256 x 128 per CU, brings a
  // quarter less into the CU per stage, but was 3 % slower on both large shapes: with one
  // workgroup per CU nothing overlaps a tile's first loads and its output phase.)
  constexpr int WM = 2;
  constexpr int MT = 2, NT = 2, BM = WM * 64, BN = 128;
  constexpr int NW = 2 * WM, THREADS = NW * 64;
  constexpr int KS = 2;                          // 64-blocks of K per stage
  constexpr int SBK = 2 * KS;                    // scale blocks per stage
  constexpr int CH = KS * F6_FRAG;               // 3072 bytes per row block and stage
  constexpr int ACH = 2 * WM;                    // row blocks of A; then 4 of B
  constexpr int SLOT = (ACH + 4) * CH;
  constexpr int PIECES = SLOT / 1024;            // 1 KiB direct loads per stage: 24 or 36
  constexpr int NDMA = (PIECES + NW - 1) / NW;   // per wavefront: 6 or 5 (4 of the 40 twice)
  constexpr int NVM = NDMA + 2;                  // + 2 scale loads
  __shared__ __attribute__((aligned(1024))) uint8_t ring[3 * SLOT];
  __shared__ __attribute__((aligned(256))) float sD[3][BM][SBK];
  __shared__ __attribute__((aligned(16))) float sCol[BN], sBias[BN];
  __shared__ __attribute__((aligned(32))) unsigned sZero[8];
  typedef unsigned u2v __attribute__((ext_vector_type(2)));
  typedef const __attribute__((address_space(3))) u2v* lds_u2;

  const int bid = blockIdx.x;
  const int xcd = bid % XCDS, idx = bid / XCDS;
  const int m_tile = (idx / n_tiles) * XCDS + xcd;
  const int n_tile = idx % n_tiles;
  if (m_tile >= m_tiles) return;
  const int m0 = m_tile * BM, n0 = n_tile * BN;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;        // wm < WM
  const int stages = KB64 / KS;
  const int KB = (K + 31) / 32;                  // scale blocks that exist
  const int MBk = (M + 31) / 32, NBk = (N + 31) / 32;

  for (int j = tid; j < BN; j += THREADS) {
    const int n = n0 + j;
    sCol[j] = n < N ? w_scale[n] : 0.f;
    sBias[j] = (bias && n < N) ? bias[n] : 0.f;
  }
  if (tid < 8) sZero[tid] = 0u;

  // piece wave + NW e of a stage (past the last: one of the first again, the same bytes
  // to the same place): chunk (row block) piece / 3, 1 KiB part piece % 3
  const uint8_t* sbase[NDMA];
  int piece[NDMA];
#pragma unroll
  for (int e = 0; e < NDMA; ++e) {
    int pi = wave + NW * e;
    pi = pi < PIECES ? pi : pi - PIECES;
    piece[e] = pi;
    const int c = pi / 3, part = pi % 3;
    long long rb;
    const uint8_t* base;
    if (c < ACH) {
      rb = (long long)m_tile * ACH + c;
      rb = rb < MBk ? rb : MBk - 1;              // past the end: a harmless re-read
      base = A6;
    } else {
      rb = (long long)n_tile * 4 + (c - ACH);
      rb = rb < NBk ? rb : NBk - 1;
      base = B6;
    }
    sbase[e] = base + rb * KB64 * F6_FRAG + part * 1024;
  }
  const unsigned lane16 = lane * 16;
  const unsigned ring_base = (unsigned)(size_t)(__attribute__((address_space(3))) uint8_t*)ring;
  const unsigned sd_base = (unsigned)(size_t)(__attribute__((address_space(3))) float*)&sD[0][0][0];
  const unsigned zero_addr = (unsigned)(size_t)(__attribute__((address_space(3))) uint8_t*)sZero;
  // scales of a stage, [BM][4] in LDS: one load brings 16 rows x 4 blocks, four lanes per
  // row, so it touches 16 lines (a lane per row would touch 64 for the same 256 bytes,
  // and the L2 request rate is what this kernel runs against); BM / 16 = 2 NW loads,
  // wavefront w brings row groups w and w + NW.  Rows and blocks past the end are
  // clamped to real ones (their products are zero or unused); only the last stage can
  // have fewer than four blocks.
  const float* d_row0 = bscale + (long long)m0 * ld_s;
  const int last_real = KB - 1 - (stages - 1) * SBK;       // 0..3 (or more: no clamp)
  unsigned d_voff[2], d_voff_last[2];
#pragma unroll
  for (int hf = 0; hf < 2; ++hf) {
    int row = (wave + hf * NW) * 16 + (lane >> 2);
    row = m0 + row < M ? row : M - 1 - m0;
    const int b = lane & 3;
    d_voff[hf] = ((unsigned)row * (unsigned)ld_s + (unsigned)b) * 4u;
    d_voff_last[hf] = ((unsigned)row * (unsigned)ld_s + (unsigned)(b < last_real ? b : last_real)) * 4u;
  }
  // stage st (clamped to the last: past the end a harmless re-load) -> slot (run-time
  // 0, 1, 2 in turn: with compile-time slots the compiler hoists every LDS address out
  // of the loop and spills them)
  auto dma_stage = [&](int slot, int st) {
    const int sc = st < stages ? st : stages - 1;
#pragma unroll
    for (int e = 0; e < NDMA; ++e)
      dma16s(sbase[e] + (long long)sc * CH, lane16,
             __builtin_amdgcn_readfirstlane(ring_base + slot * SLOT + piece[e] * 1024));
    const bool last = sc == stages - 1;
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
      dma4s(d_row0 + sc * SBK, last ? d_voff_last[hf] : d_voff[hf],
            __builtin_amdgcn_readfirstlane(sd_base + (slot * BM + (wave + hf * NW) * 16) * SBK * 4));
  };

  // operand reads.  x (activations): lanes of half h read their 24 bytes, the others the
  // zeros: address = base + flag * offset, one instruction, kept where it is written.
  const bool lower = lane < 32;
  const unsigned x_lane = ring_base + (wm * 2 * CH + lane * 24);
  const unsigned w_lane = ring_base + ((ACH + wn * 2) * CH + lane * 24);
  const unsigned x_base[2] = {lower ? x_lane : zero_addr, lower ? zero_addr : x_lane};
  const unsigned x_flag[2] = {lower ? 1u : 0u, lower ? 0u : 1u};
  const unsigned d_lane = sd_base + (wm * 64 + (lane & 31)) * SBK * 4;
  auto read24 = [&](unsigned addr) {
    const lds_u2 p = (lds_u2)(size_t)addr;
    const u2v q0 = p[0], q1 = p[1], q2 = p[2];
    const v8i v = {(int)q0.x, (int)q0.y, (int)q1.x, (int)q1.y, (int)q2.x, (int)q2.y, 0, 0};
    return v;
  };
  auto read_x = [&](v8i (&dst)[MT], int slot, int kk, int h) {          // kk, h compile-time
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const unsigned off = (unsigned)(slot * SLOT + i * CH + kk * F6_FRAG);   // scalar
      unsigned addr;
      asm volatile("v_mad_u32_u24 %0, %1, %2, %3" : "=v"(addr) : "v"(x_flag[h]), "s"(off), "v"(x_base[h]));
      dst[i] = read24(addr);
    }
  };
  auto read_w = [&](v8i (&dst)[NT], int slot, int kk) {
    const unsigned w_slot = w_lane + (unsigned)(slot * SLOT);
#pragma unroll
    for (int j = 0; j < NT; ++j) dst[j] = read24(w_slot + (unsigned)(j * CH + kk * F6_FRAG));
  };
  typedef float f4v __attribute__((ext_vector_type(4)));
  typedef const __attribute__((address_space(3))) f4v* lds_f4;
  auto read_dl = [&](f4v (&dst)[MT], int slot) {           // the lane's rows, the stage's 4 blocks
    const lds_f4 p = (lds_f4)(size_t)(d_lane + (unsigned)(slot * SBK * BM * 4));
#pragma unroll
    for (int i = 0; i < MT; ++i) dst[i] = p[i * 32];
  };

  float accf[MT][NT][16];
  v16f t[MT][NT];
  f4v dcur[MT];                                  // the stage's scales of the lane's rows
  float dlast[MT];                               // those of the previous stage's last block
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    dlast[i] = 0.f;
    dcur[i] = f4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        accf[i][j][r] = 0.f;
        t[i][j][r] = 0.f;
      }
  }
  const v16f zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  auto consume = [&](int i, int j, float d) {
#pragma unroll
    for (int r = 0; r < 16; ++r) accf[i][j][r] = __builtin_fmaf(t[i][j][r], d, accf[i][j][r]);
  };

  v8i xbuf[2][MT], wbuf[2][NT];                  // activations by half h, weights by kk
  dma_stage(0, 0);
  dma_stage(1, 1);
  dma_stage(2, 2);
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * NVM) : "memory");   // stage 0 has landed
  __syncthreads();
  read_x(xbuf[0], 0, 0, 0);
  read_w(wbuf[0], 0, 0);

  // Round R of the stage in slot CUR (NXT: the next stage's).  R and the register
  // indices are compile-time constants.  Round 0 consumes the last group of the stage
  // before (scale kept in dlast) and reads this stage's scales; round R > 0 consumes
  // group R - 1.
#define TDQ_BF6_SLOT(R, I, J)                                                                     \
  do {                                                                                            \
    __builtin_amdgcn_sched_barrier(0);                                                            \
    consume(I, J, (R) == 0 ? dlast[I] : dcur[I][((R) + 3) & 3]);                                  \
    t[I][J] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wbuf[(R) >> 1][J], xbuf[(R) & 1][I], \
                                                              zero, 3, 3, 0, 127, 0, 127);        \
  } while (0)
#define TDQ_BF6_ROUND(s, CUR, NXT, R)                                                             \
  do {                                                                                            \
    /* the next round's activations first: four slots until they are used */                     \
    __builtin_amdgcn_sched_barrier(0);                                                            \
    if ((R) < 3) read_x(xbuf[((R) + 1) & 1], CUR, ((R) + 1) >> 1, ((R) + 1) & 1);                 \
    else read_x(xbuf[0], NXT, 0, 0);                                                              \
    TDQ_BF6_SLOT(R, 0, 0);                                                                        \
    if ((R) == 0) {                                                                               \
      read_dl(dcur, CUR);                         /* the old ones were spent in round 3 */        \
      read_w(wbuf[1], CUR, 1);                    /* for rounds 2 and 3 */                        \
    }                                                                                             \
    TDQ_BF6_SLOT(R, 0, 1);                                                                        \
    TDQ_BF6_SLOT(R, 1, 0);                                                                        \
    if ((R) == 2) {                                                                               \
      __builtin_amdgcn_sched_barrier(0);                                                          \
      asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(NVM) : "memory");                       \
      __builtin_amdgcn_s_barrier();                                                               \
      dma_stage(CUR, (s) + 3);                                                                    \
      read_w(wbuf[0], NXT, 0);                    /* for rounds 0 and 1 of the next stage */      \
    }                                                                                             \
    TDQ_BF6_SLOT(R, 1, 1);                                                                        \
    if ((R) == 3) {                                                                               \
      dlast[0] = dcur[0][3];                                                                      \
      dlast[1] = dcur[1][3];                                                                      \
    }                                                                                             \
    __builtin_amdgcn_sched_barrier(0);                                                            \
  } while (0)

  int cur = 0, nxt = 1, nn = 2;
#pragma unroll 1
  for (int s = 0; s < stages; ++s) {
    TDQ_BF6_ROUND(s, cur, nxt, 0);
    TDQ_BF6_ROUND(s, cur, nxt, 1);
    TDQ_BF6_ROUND(s, cur, nxt, 2);
    TDQ_BF6_ROUND(s, cur, nxt, 3);
    const int o = cur;
    cur = nxt;
    nxt = nn;
    nn = o;
  }
#undef TDQ_BF6_ROUND
#undef TDQ_BF6_SLOT
  consume(0, 0, dlast[0]);                       // the last round's results
  consume(0, 1, dlast[0]);
  consume(1, 0, dlast[1]);
  consume(1, 1, dlast[1]);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");         // nothing of ours may still be landing

  // Register r of result (i, j) is row m = 32 i + lane % 32 of the wavefront's 64 and
  // channel 32 j + 8 (r / 4) + 4 (lane / 32) + r % 4: a lane holds short runs of 32 rows,
  // which as stores would touch 32 lines with 8 or 16 bytes each.  So the wavefront's
  // 64 x 64 results (already scaled) go, 32 rows at a time, through its own 8.5 KiB of the
  // ring, now free, and leave row-major: every store instruction writes whole 128-byte lines.
  __syncthreads();                               // every wavefront's loads have landed
  constexpr int TP = 68;                         // pitch in floats: 16-byte aligned rows, staggered banks
  float* T = reinterpret_cast<float*>(ring) + wave * (32 * TP);
  const int ml = lane & 31, nq = (lane >> 5) * 4;
  constexpr int W = 16 / (int)sizeof(OUT);       // outputs per 16-byte store: 4 or 8
  constexpr int LPR = 64 / W;                    // lanes per row of 64
  constexpr int RPI = 64 / LPR;                  // rows per store instruction
  const int rsub = lane / LPR, col = (lane % LPR) * W;
  const int nbase = n0 + wn * 64 + col;
#pragma unroll
  for (int i = 0; i < MT; ++i) {                 // 32 rows at a time
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        const int cw = j * 32 + rq * 8 + nq;     // channel within the wavefront's 64
        const float4 sc4 = *reinterpret_cast<const float4*>(&sCol[wn * 64 + cw]);
        const float4 bi4 = *reinterpret_cast<const float4*>(&sBias[wn * 64 + cw]);
        float4 y = make_float4(accf[i][j][4 * rq] * sc4.x, accf[i][j][4 * rq + 1] * sc4.y,
                               accf[i][j][4 * rq + 2] * sc4.z, accf[i][j][4 * rq + 3] * sc4.w);
        if (bias) {
          y.x = y.x + bi4.x;
          y.y = y.y + bi4.y;
          y.z = y.z + bi4.z;
          y.w = y.w + bi4.w;
        }
        *reinterpret_cast<float4*>(&T[ml * TP + cw]) = y;
      }
#pragma unroll
    for (int it = 0; it < 32 / RPI; ++it) {
      const int row = it * RPI + rsub;
      const int m = m0 + wm * 64 + i * 32 + row;
      float y[W];
#pragma unroll
      for (int q = 0; q < W / 4; ++q) {
        const float4 v = *reinterpret_cast<const float4*>(&T[row * TP + col + 4 * q]);
        y[4 * q] = v.x; y[4 * q + 1] = v.y; y[4 * q + 2] = v.z; y[4 * q + 3] = v.w;
      }
      if (m < M) {
        OUT* yp = Y + (long long)m * ld_y + nbase;
        if (y_vec_ok && nbase + W - 1 < N) {
          store_out_vec<OUT>(yp, y);
        } else {
#pragma unroll
          for (int e = 0; e < W; ++e)
            if (nbase + e < N) store_out<OUT>(yp + e, y[e]);
        }
      }
    }
  }
}

hipError_t launch_w4a4_gemm_blocks_f6(const uint8_t* A6, const uint8_t* B6, const float* bscale,
                                      long long ld_s, int M, int K, int N, const float* w_scale,
                                      const float* bias, void* Y, tdq_dtype y_dt, long long ld_y,
                                      hipStream_t st) {
  const int KB64 = 2 * ((K + 127) / 128);
  const int m_tiles = (M + 127) / 128, n_tiles = (N + 127) / 128;
  const long long m_groups = (m_tiles + XCDS - 1) / XCDS;
  const unsigned grid = (unsigned)(m_groups * XCDS * n_tiles);
  // 16-byte stores where every row of Y starts on a 16-byte boundary
  const int per16 = y_dt == TDQ_F32 ? 4 : 8;
  const int y_vec_ok = (reinterpret_cast<uintptr_t>(Y) % 16 == 0 && ld_y % per16 == 0) ? 1 : 0;
  if (y_dt == TDQ_F32)
    hipLaunchKernelGGL((k_w4a4_gemm_blocks_f6<float>), dim3(grid), dim3(GEMM_THREADS), 0, st, A6, B6,
                       KB64, bscale, ld_s, M, K, N, w_scale, bias, static_cast<float*>(Y), ld_y, m_tiles,
                       n_tiles, y_vec_ok);
  else
    hipLaunchKernelGGL((k_w4a4_gemm_blocks_f6<_Float16>), dim3(grid), dim3(GEMM_THREADS), 0, st, A6, B6,
                       KB64, bscale, ld_s, M, K, N, w_scale, bias, static_cast<_Float16*>(Y), ld_y,
                       m_tiles, n_tiles, y_vec_ok);
  return hipGetLastError();
}

}  // namespace tdq
