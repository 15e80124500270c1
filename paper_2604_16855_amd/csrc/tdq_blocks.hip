// Paper-literal granularity of DSTG + DCRP (Sec. 4.2, Eq. direct_sum; Supp. Algorithm 1
// steps 1-9): every token's channel axis, zero-padded to a multiple of g = 32, is cut
// into blocks of g channels, and every (token, block) is a quantization group of its
// own: base radius = block maximum (or the rank quantile Q_p), sigma = population std of
// the 32 values (padding zeros included, as Algorithm 1 pads before it reduces),
// threshold = the ceil(zr g)-th smallest magnitude, Eq. (dcrp), quantize, pack.  With 32
// values per group nothing needs a histogram or a second pass: ONE sweep of X.
//
// Four adjacent lanes (a quad) own a block, 8 values each.  Block-wide quantities are
// combined over the quad with DPP quad permutes, which leave the result in all four
// lanes.  For binary16 input a lane serves TWO blocks at once (block i and block i + 16
// of the 32 consecutive blocks of its wavefront, so both 16-byte loads of the wavefront
// are contiguous kilobytes) and keeps the two blocks' magnitude keys in the two halves
// of its registers: every packed 16-bit min / max then works on both blocks.
//
// The k-th smallest of 32 keys for k <= 8 (zr <= 0.25; the paper's zr = 0.2 gives k = 7):
//   1. each lane sorts its 8 keys (19 compare-exchanges);
//   2. lanes l and l ^ 1 keep the 8 smallest of their 16: min(a[i], b[7 - i]) is that
//      set as a bitonic sequence, which 12 compare-exchanges sort;
//   3. the same between lanes l and l ^ 2: the 8 smallest of the block, sorted; take
//      element k - 1.
// Any other rank (and the percentile base radius) is found by bisection on the key bits.
#include "tdq_device.hpp"

namespace tdq {

constexpr int kBlk = 32;                 // channels per block (the paper's g)

// ---------------------------------------------------------------------------
// quad exchanges (control = quad_perm selector; every lane of the wavefront is active
// wherever these are called)
// ---------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ u32 quad_u32(u32 v) {
  return (u32)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
constexpr int kQuadXor1 = 0xB1;          // [1, 0, 3, 2]
constexpr int kQuadXor2 = 0x4E;          // [2, 3, 0, 1]
constexpr int kQuadLane0 = 0x00;         // [0, 0, 0, 0]
constexpr int kQuadLane1 = 0x55;         // [1, 1, 1, 1]

template <int CTRL>
__device__ __forceinline__ float quad_f32(float v) {
  return __uint_as_float(quad_u32<CTRL>(__float_as_uint(v)));
}
template <int CTRL>
__device__ __forceinline__ double quad_f64(double v) {
  const unsigned long long b = __builtin_bit_cast(unsigned long long, v);
  const u32 lo = quad_u32<CTRL>((u32)b), hi = quad_u32<CTRL>((u32)(b >> 32));
  return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
}
__device__ __forceinline__ u32 quad_sum_u32(u32 v) {
  v += quad_u32<kQuadXor1>(v);
  v += quad_u32<kQuadXor2>(v);
  return v;
}
// Sum over the quad, the same bits in all four lanes: (x0 + x1) + (x2 + x3) with
// commutative additions only.
__device__ __forceinline__ double quad_sum_f64(double v) {
  v += quad_f64<kQuadXor1>(v);
  v += quad_f64<kQuadXor2>(v);
  return v;
}

// ---------------------------------------------------------------------------
// keys: PK = two 15-bit keys per register (two blocks), else one 31-bit key
// ---------------------------------------------------------------------------
typedef short s2b __attribute__((ext_vector_type(2)));

template <bool PK>
__device__ __forceinline__ u32 kmin(u32 a, u32 b) {
  if constexpr (PK)
    return __builtin_bit_cast(
        u32, __builtin_elementwise_min(__builtin_bit_cast(us2, a), __builtin_bit_cast(us2, b)));
  else
    return a < b ? a : b;
}
template <bool PK>
__device__ __forceinline__ u32 kmax(u32 a, u32 b) {
  if constexpr (PK)
    return __builtin_bit_cast(
        u32, __builtin_elementwise_max(__builtin_bit_cast(us2, a), __builtin_bit_cast(us2, b)));
  else
    return a > b ? a : b;
}
template <bool PK>
__device__ __forceinline__ void cmpx(u32& a, u32& b) {     // a <- min, b <- max
  const u32 lo = kmin<PK>(a, b), hi = kmax<PK>(a, b);
  a = lo;
  b = hi;
}
template <bool PK>
__device__ __forceinline__ void sort8(u32 (&k)[8]) {        // optimal 19-comparator network
  cmpx<PK>(k[0], k[1]); cmpx<PK>(k[2], k[3]); cmpx<PK>(k[4], k[5]); cmpx<PK>(k[6], k[7]);
  cmpx<PK>(k[0], k[2]); cmpx<PK>(k[1], k[3]); cmpx<PK>(k[4], k[6]); cmpx<PK>(k[5], k[7]);
  cmpx<PK>(k[1], k[2]); cmpx<PK>(k[5], k[6]); cmpx<PK>(k[0], k[4]); cmpx<PK>(k[3], k[7]);
  cmpx<PK>(k[1], k[5]); cmpx<PK>(k[2], k[6]);
  cmpx<PK>(k[1], k[4]); cmpx<PK>(k[3], k[6]);
  cmpx<PK>(k[2], k[4]); cmpx<PK>(k[3], k[5]);
  cmpx<PK>(k[3], k[4]);
}
template <bool PK>
__device__ __forceinline__ void sort8_bitonic(u32 (&k)[8]) {   // input: a bitonic sequence
  cmpx<PK>(k[0], k[4]); cmpx<PK>(k[1], k[5]); cmpx<PK>(k[2], k[6]); cmpx<PK>(k[3], k[7]);
  cmpx<PK>(k[0], k[2]); cmpx<PK>(k[1], k[3]); cmpx<PK>(k[4], k[6]); cmpx<PK>(k[5], k[7]);
  cmpx<PK>(k[0], k[1]); cmpx<PK>(k[2], k[3]); cmpx<PK>(k[4], k[5]); cmpx<PK>(k[6], k[7]);
}
// k[] sorted ascending in this lane and in its partner: the 8 smallest of both, sorted.
template <bool PK, int CTRL>
__device__ __forceinline__ void merge_low8(u32 (&k)[8]) {
  u32 o[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = quad_u32<CTRL>(k[7 - i]);
#pragma unroll
  for (int i = 0; i < 8; ++i) k[i] = kmin<PK>(k[i], o[i]);
  sort8_bitonic<PK>(k);
}

// The rank-th smallest (1-based, 1 <= rank <= 32) of the block's 32 keys by bisection on
// the key bits: the largest t with #{key < t} < rank.  PK: both blocks at once.
template <bool PK>
__device__ __forceinline__ u32 kth_by_bisection(const u32 (&key)[8], u32 rank) {
  u32 thr = 0;
  if constexpr (PK) {
#pragma unroll 1
    for (int bit = 14; bit >= 0; --bit) {
      const u32 cand = thr | (0x00010001u << bit);
      u32 cnt = 0;                                         // two counts, one per half
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        // keys and candidates are below 2^15: the 16-bit differences cannot overflow and
        // their sign bits say "key < candidate"
        const s2b d = __builtin_bit_cast(s2b, key[i]) - __builtin_bit_cast(s2b, cand);
        cnt += (__builtin_bit_cast(u32, d) >> 15) & 0x00010001u;
      }
      cnt = quad_sum_u32(cnt);
      const u32 take = ((cnt & 0xFFFFu) < rank ? 0x0000FFFFu : 0u) |
                       ((cnt >> 16) < rank ? 0xFFFF0000u : 0u);
      thr = (cand & take) | (thr & ~take);
    }
  } else {
#pragma unroll 1
    for (int bit = 30; bit >= 0; --bit) {
      const u32 cand = thr | (1u << bit);
      u32 cnt = 0;
#pragma unroll
      for (int i = 0; i < 8; ++i) cnt += key[i] < cand ? 1u : 0u;
      cnt = quad_sum_u32(cnt);
      thr = cnt < rank ? cand : thr;
    }
  }
  return thr;
}

// ---------------------------------------------------------------------------
// One block per quad (two for binary16, in the halves of the key registers): raw[s] holds
// this lane's 8 values of block s as loaded.  Returns the 8 packed codes of each block
// and, in every lane of the quad, its clip radius and step.  Every lane of the wavefront
// must take part (quad exchanges).
// ---------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void block_core(const u32 (&raw)[sizeof(T) == 2 ? 2 : 1][sizeof(T) == 2 ? 4 : 8],
                                           int ql, int kq, int kp, const Scalars& sc,
                                           u32 (&word)[sizeof(T) == 2 ? 2 : 1],
                                           float (&cs)[sizeof(T) == 2 ? 2 : 1],
                                           float (&ds)[sizeof(T) == 2 ? 2 : 1]) {
  constexpr bool PK = sizeof(T) == 2;
  constexpr int NB = PK ? 2 : 1;
  // values, moments (binary64, as the set statistics of the token-set path)
  float v[NB][8];
  double s1[NB], s2[NB];
#pragma unroll
  for (int s = 0; s < NB; ++s) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if constexpr (PK) v[s][i] = h2f((raw[s][i >> 1] >> (16 * (i & 1))) & 0xFFFFu);
      else v[s][i] = __uint_as_float(raw[s][i]);
    }
    double a1 = 0.0, a2 = 0.0;
    if constexpr (PK) {
      // sum x^2 - n mu^2 in binary64: binary16 values that differ at all differ by at
      // least 2^-11 relative, so the variance is no smaller than 1e-8 mu^2 and the
      // cancellation costs 8 of the 16 digits at most
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const double x = (double)v[s][i];
        a1 += x;
        a2 = fma(x, x, a2);
      }
      s1[s] = quad_sum_f64(a1);
      s2[s] = quad_sum_f64(a2);
    } else {
      // binary32 values can sit within 1e-7 of their mean: centre first
#pragma unroll
      for (int i = 0; i < 8; ++i) a1 += (double)v[s][i];
      s1[s] = quad_sum_f64(a1);
      const double mu = s1[s] / (double)kBlk;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const double e = (double)v[s][i] - mu;
        a2 = fma(e, e, a2);
      }
      s2[s] = quad_sum_f64(a2);                            // sum (x - mu)^2
    }
  }

  // keys: PK packs element i of block 0 (low half) with element i of block 1 (high half)
  u32 key[8];
  if constexpr (PK) {
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const u32 a = raw[0][w] & 0x7FFF7FFFu, b = raw[1][w] & 0x7FFF7FFFu;
      key[2 * w] = __builtin_amdgcn_perm(b, a, 0x05040100u);       // [a.lo16, b.lo16]
      key[2 * w + 1] = __builtin_amdgcn_perm(b, a, 0x07060302u);   // [a.hi16, b.hi16]
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) key[i] = raw[0][i] & 0x7FFFFFFFu;
  }

  u32 top = key[0];
#pragma unroll
  for (int i = 1; i < 8; ++i) top = kmax<PK>(top, key[i]);
  top = kmax<PK>(top, quad_u32<kQuadXor1>(top));
  top = kmax<PK>(top, quad_u32<kQuadXor2>(top));
  if (kp < kBlk) top = kth_by_bisection<PK>(key, (u32)kp);         // percentile base radius

  u32 thr;
  if (kq <= 8) {
    u32 k[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) k[i] = key[i];
    sort8<PK>(k);
    merge_low8<PK, kQuadXor1>(k);
    merge_low8<PK, kQuadXor2>(k);
    thr = k[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) thr = kq == i + 1 ? k[i] : thr;
  } else {
    thr = kth_by_bisection<PK>(key, (u32)kq);
  }

  // Eq. (dcrp) in binary32 with the eps floors of the supplementary conventions.  Lane s
  // of the quad does block s; the results travel to the other lanes afterwards.
  const int mine = (PK && ql == 1) ? 1 : 0;
  const double S1 = mine ? s1[NB - 1] : s1[0], S2 = mine ? s2[NB - 1] : s2[0];
  const u32 my_top = PK ? (mine ? top >> 16 : top & 0xFFFFu) : top;
  const u32 my_thr = PK ? (mine ? thr >> 16 : thr & 0xFFFFu) : thr;
  double var;
  if constexpr (PK) {
    const double mu = S1 / (double)kBlk;
    var = S2 / (double)kBlk - mu * mu;
    var = var > 0.0 ? var : 0.0;
  } else {
    var = S2 / (double)kBlk;
  }
  const float sigma = (float)(sqrt(var) + sc.eps_std);
  const float c_base = Elem<T>::key_to_float(my_top);
  const float c_tau = sc.qmax_tau * sigma;                         // q_max tau sigma
  const float c_zr = sc.two_qmax * Elem<T>::key_to_float(my_thr);  // 2 q_max Q_zr(|x|)
  float c = c_base;
  if ((sc.flags & TDQ_FLAG_C1) && c_tau < c) c = c_tau;
  if ((sc.flags & TDQ_FLAG_C2) && c_zr < c) c = c_zr;
  if (!(c > sc.eps_scale)) c = sc.eps_scale;
  float d = c / sc.qmax;
  d = d > sc.eps_scale ? d : sc.eps_scale;
  const float rcp = 1.0f / d;                                      // correctly rounded

  float rs[NB];
  cs[0] = quad_f32<kQuadLane0>(c);
  ds[0] = quad_f32<kQuadLane0>(d);
  rs[0] = quad_f32<kQuadLane0>(rcp);
  if constexpr (PK) {
    cs[1] = quad_f32<kQuadLane1>(c);
    ds[1] = quad_f32<kQuadLane1>(d);
    rs[1] = quad_f32<kQuadLane1>(rcp);
  }

#pragma unroll
  for (int s = 0; s < NB; ++s) {
    if constexpr (PK) {
      // c <= 7 Delta (1 + 2^-24) by construction: the clamp of the code is implied
      word[s] = quant8_f16<false>(make_uint4(raw[s][0], raw[s][1], raw[s][2], raw[s][3]), cs[s], ds[s],
                                  rs[s]);
    } else {
      word[s] = 0;
#pragma unroll
      for (int i = 0; i < 8; ++i) word[s] |= quant_nibble(v[s][i], cs[s], ds[s], rs[s]) << (4 * i);
    }
  }
}

// Stores the 8 codes of one lane (4 bytes at byte b0 of the row) and, from lane `owner`
// of the quad, the block's step and radius.
__device__ __forceinline__ void block_store(u32 word, float c, float d, bool owner, long long row,
                                            int kb, int ql, int C, int q_vec_ok,
                                            uint8_t* __restrict__ Q, long long ld_q,
                                            float* __restrict__ bscale, float* __restrict__ bclip,
                                            long long ld_s) {
  if (owner) {
    bscale[row * ld_s + kb] = d;
    if (bclip) bclip[row * ld_s + kb] = c;
  }
  // 8 codes = 4 bytes at byte 16 kb + 4 ql of the row; a row holds ceil(C / 2) bytes
  const int b0 = kb * (kBlk / 2) + ql * 4;
  uint8_t* qp = Q + row * ld_q + b0;
  const int nbytes = (C + 1) / 2 - b0;                             // bytes of the row from here on
  if (q_vec_ok && nbytes >= 4) {
    *reinterpret_cast<u32*>(qp) = word;
  } else {
    for (int i = 0; i < 4 && i < nbytes; ++i) qp[i] = (uint8_t)(word >> (8 * i));
  }
}

// ---------------------------------------------------------------------------
// the sweep
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_quantize_blocks(
    const T* __restrict__ X, long long ld, u32 total, int C, int KB, int vec_ok, int q_vec_ok,
    int kq, int kp, Scalars sc, uint8_t* __restrict__ Q, long long ld_q, float* __restrict__ bscale,
    float* __restrict__ bclip, long long ld_s) {
  constexpr bool PK = sizeof(T) == 2;
  constexpr int NB = PK ? 2 : 1;                           // blocks per lane
  constexpr int W = PK ? 4 : 8;                            // 32-bit words of 8 elements
  const u32 wave_first =
      (u32)__builtin_amdgcn_readfirstlane((int)((blockIdx.x * 4u + (threadIdx.x >> 6)) * (16u * NB)));
  if (wave_first >= total) return;                         // whole wavefronts only
  const int lane = threadIdx.x & 63, quad = lane >> 2, ql = lane & 3;
  const u32 row0 = wave_first / (u32)KB, kb0 = wave_first - row0 * (u32)KB;

  bool live[NB];
  long long row[NB];
  int kb[NB];
  u32 raw[NB][W];
#pragma unroll
  for (int s = 0; s < NB; ++s) {
    const u32 off = (u32)quad + 16u * s;
    live[s] = wave_first + off < total;
    // a quad without a block works on the wavefront's first block and stores nothing
    const u32 t = kb0 + (live[s] ? off : 0u);
    u32 wrap;
    if (KB >= 16 * NB) wrap = t >= (u32)KB ? 1u : 0u;      // t < KB + 16 NB <= 2 KB
    else wrap = t / (u32)KB;
    row[s] = (long long)(row0 + wrap);
    kb[s] = (int)(t - wrap * (u32)KB);
    const int c0 = kb[s] * kBlk + ql * 8;                  // first channel of this lane
    const T* xp = X + row[s] * ld + c0;
    if (vec_ok && c0 + 8 <= C) {
      const uint4 q0 = *reinterpret_cast<const uint4*>(xp);
      raw[s][0] = q0.x; raw[s][1] = q0.y; raw[s][2] = q0.z; raw[s][3] = q0.w;
      if constexpr (!PK) {
        const uint4 q1 = *reinterpret_cast<const uint4*>(xp + 4);
        raw[s][4] = q1.x; raw[s][5] = q1.y; raw[s][6] = q1.z; raw[s][7] = q1.w;
      }
    } else {
      // row tail or unaligned rows; channels at and beyond C are the zero padding
#pragma unroll
      for (int w = 0; w < W; ++w) raw[s][w] = 0;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (c0 + i < C) {
          if constexpr (PK) raw[s][i >> 1] |= (u32)xp[i] << (16 * (i & 1));
          else raw[s][i] = __float_as_uint(xp[i]);
        }
      }
    }
  }

  u32 word[NB];
  float cs[NB], ds[NB];
  block_core<T>(raw, ql, kq, kp, sc, word, cs, ds);
#pragma unroll
  for (int s = 0; s < NB; ++s)
    if (live[s])
      block_store(word[s], cs[s], ds[s], ql == s, row[s], kb[s], ql, C, q_vec_ok, Q, ld_q, bscale,
                  bclip, ld_s);
}

template <typename T>
static hipError_t quantize_blocks_t(const T* X, long long M, int C, long long ld, int kq, int kp,
                                    const Scalars& sc, uint8_t* Q, long long ld_q, float* bscale,
                                    float* bclip, long long ld_s, hipStream_t st) {
  const int KB = (C + kBlk - 1) / kBlk;
  const int V = 16 / (int)sizeof(T);
  const int per_wave = sizeof(T) == 2 ? 32 : 16;
  const int vec_ok = ((reinterpret_cast<uintptr_t>(X) & 15) == 0 && ld % V == 0) ? 1 : 0;
  const int q_vec_ok = ((reinterpret_cast<uintptr_t>(Q) & 3) == 0 && ld_q % 4 == 0) ? 1 : 0;
  const long long total = M * KB;                          // checked by the caller: < 2^31
  const unsigned grid = (unsigned)((total + 4 * per_wave - 1) / (4 * per_wave));
  hipLaunchKernelGGL((k_quantize_blocks<T>), dim3(grid), dim3(256), 0, st, X, ld, (u32)total, C, KB,
                     vec_ok, q_vec_ok, kq, kp, sc, Q, ld_q, bscale, bclip, ld_s);
  return hipGetLastError();
}

hipError_t launch_quantize_blocks(const void* X, tdq_dtype dt, long long M, int C, long long ld,
                                  int kq, int kp, const Scalars& sc, uint8_t* Q, long long ld_q,
                                  float* bscale, float* bclip, long long ld_s, hipStream_t st) {
  if (dt == TDQ_F16)
    return quantize_blocks_t<u16>(static_cast<const u16*>(X), M, C, ld, kq, kp, sc, Q, ld_q, bscale,
                                  bclip, ld_s, st);
  return quantize_blocks_t<float>(static_cast<const float*>(X), M, C, ld, kq, kp, sc, Q, ld_q,
                                  bscale, bclip, ld_s, st);
}

// ---------------------------------------------------------------------------
// The sweep writing the operand format of the 6-bit contraction (f6 fragments of 32 rows
// x 64 codes, see k_quantize_f6) instead of packed nibbles; steps and radii as before.
// A workgroup owns 32 rows x 16 blocks (8 fragments): every wavefront pass runs
// block_core on NB rows x 16 blocks (reads of 1 KiB per row), the nibble words go to LDS,
// and after a barrier every thread turns two (row, block) entries -- 32 codes, 16 bytes
// of nibbles -- into 24 bytes of bf6 patterns: sign-extending extract, integer -> float,
// one conversion instruction for the 32 (even codes in its first operand, odd ones in its
// second).  A fragment leaves as 1536 contiguous bytes.  Rows past M and blocks past
// ceil(C / 32) are zero codes.
// ---------------------------------------------------------------------------
typedef float blk_v16f __attribute__((ext_vector_type(16)));
typedef int blk_v6i __attribute__((ext_vector_type(6)));

template <typename T>
__global__ __launch_bounds__(256) void k_quantize_blocks_f6(
    const T* __restrict__ X, long long ld, long long M, int C, int KB, int KB64, int k_tiles,
    int vec_ok, int kq, int kp, Scalars sc, uint8_t* __restrict__ F, float* __restrict__ bscale,
    float* __restrict__ bclip, long long ld_s) {
  constexpr bool PK = sizeof(T) == 2;
  constexpr int NB = PK ? 2 : 1;                           // blocks per lane = rows per pass
  constexpr int W = PK ? 4 : 8;
  constexpr int TBK = 16;                                  // blocks per tile
  constexpr int PITCH = TBK * 4 + 4;                       // words per tile row: 16-byte reads on disjoint banks
  constexpr int PASSES = 32 / NB / 4;                      // per wavefront
  __shared__ __attribute__((aligned(16))) u32 sN[32 * PITCH];

  const long long rb = blockIdx.x / k_tiles;
  const int kt = blockIdx.x % k_tiles;
  const long long row0 = rb * 32;
  const int kbt0 = kt * TBK;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, quad = lane >> 2, ql = lane & 3;
  const int kb = kbt0 + quad;
  const int c0 = kb * kBlk + ql * 8;                       // first channel of this lane

#pragma unroll 1
  for (int p = 0; p < PASSES; ++p) {
    bool live[NB];
    long long row[NB];
    int r_in[NB];
    u32 raw[NB][W];
#pragma unroll
    for (int s = 0; s < NB; ++s) {
      r_in[s] = (wave * PASSES + p) * NB + s;
      row[s] = row0 + r_in[s];
      live[s] = row[s] < M && kb < KB;
#pragma unroll
      for (int w = 0; w < W; ++w) raw[s][w] = 0;
      if (live[s]) {
        const T* xp = X + row[s] * ld + c0;
        if (vec_ok && c0 + 8 <= C) {
          const uint4 q0 = *reinterpret_cast<const uint4*>(xp);
          raw[s][0] = q0.x; raw[s][1] = q0.y; raw[s][2] = q0.z; raw[s][3] = q0.w;
          if constexpr (!PK) {
            const uint4 q1 = *reinterpret_cast<const uint4*>(xp + 4);
            raw[s][4] = q1.x; raw[s][5] = q1.y; raw[s][6] = q1.z; raw[s][7] = q1.w;
          }
        } else {
          // row tail or unaligned rows; channels at and beyond C are the zero padding
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            if (c0 + i < C) {
              if constexpr (PK) raw[s][i >> 1] |= (u32)xp[i] << (16 * (i & 1));
              else raw[s][i] = __float_as_uint(xp[i]);
            }
          }
        }
      }
    }
    u32 word[NB];
    float cs[NB], ds[NB];
    block_core<T>(raw, ql, kq, kp, sc, word, cs, ds);      // (a quad without a block works on zeros)
#pragma unroll
    for (int s = 0; s < NB; ++s) {
      if (live[s] && ql == s) {
        bscale[row[s] * ld_s + kb] = ds[s];
        if (bclip) bclip[row[s] * ld_s + kb] = cs[s];
      }
      sN[r_in[s] * PITCH + quad * 4 + ql] = live[s] ? word[s] : 0u;
    }
  }
  __syncthreads();

#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int e = threadIdx.x + 256 * k;
    const int f = e >> 6, l = e & 63;                      // fragment of the tile, lane of the fragment
    const int kb64 = kbt0 / 2 + f;
    if (kb64 >= KB64) continue;
    const uint4 w4 = *reinterpret_cast<const uint4*>(&sN[(l & 31) * PITCH + (2 * f + (l >> 5)) * 4]);
    const u32 w[4] = {w4.x, w4.y, w4.z, w4.w};
    blk_v16f ev, od;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const u32 wd = w[i >> 2];
      const int sh = 8 * (i & 3);                          // codes 2 i and 2 i + 1: bits sh, sh + 4
      ev[i] = (float)((int)(wd << (28 - sh)) >> 28);
      od[i] = (float)((int)(wd << (24 - sh)) >> 28);
    }
    const blk_v6i r = __builtin_amdgcn_cvt_scalef32_2xpk16_bf6_f32(ev, od, 1.0f);
    uint2* dst = reinterpret_cast<uint2*>(F + ((rb * KB64 + kb64) * 64 + l) * 24);
    dst[0] = make_uint2((u32)r[0], (u32)r[1]);
    dst[1] = make_uint2((u32)r[2], (u32)r[3]);
    dst[2] = make_uint2((u32)r[4], (u32)r[5]);
  }
}

hipError_t launch_quantize_blocks_f6(const void* X, tdq_dtype dt, long long M, int C, long long ld,
                                     int kq, int kp, const Scalars& sc, uint8_t* F, float* bscale,
                                     float* bclip, long long ld_s, hipStream_t st) {
  const int KB = (C + kBlk - 1) / kBlk;
  const int KB64 = 2 * ((C + 127) / 128);
  const int k_tiles = (KB64 + 7) / 8;
  const long long n_rb = (M + 31) / 32;
  const unsigned grid = (unsigned)(n_rb * k_tiles);        // checked by the caller: < 2^31
  if (dt == TDQ_F16) {
    const int vec_ok = ((reinterpret_cast<uintptr_t>(X) & 15) == 0 && ld % 8 == 0) ? 1 : 0;
    hipLaunchKernelGGL((k_quantize_blocks_f6<u16>), dim3(grid), dim3(256), 0, st,
                       static_cast<const u16*>(X), ld, M, C, KB, KB64, k_tiles, vec_ok, kq, kp, sc, F,
                       bscale, bclip, ld_s);
  } else {
    const int vec_ok = ((reinterpret_cast<uintptr_t>(X) & 15) == 0 && ld % 4 == 0) ? 1 : 0;
    hipLaunchKernelGGL((k_quantize_blocks_f6<float>), dim3(grid), dim3(256), 0, st,
                       static_cast<const float*>(X), ld, M, C, KB, KB64, k_tiles, vec_ok, kq, kp, sc, F,
                       bscale, bclip, ld_s);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// The same sweep over a convolutional feature map X[B, C, T] (T = H W tokens, contiguous;
// Supp. "Implementation details", the 4-D branch): a group is the block of 32 channels
// of one pixel.  A workgroup owns TT consecutive tokens of one image and walks the
// channel axis in tiles of TC channels: 16-byte loads along the token axis into LDS,
// then every quad gathers its block(s) of one token from the tile (2- or 4-byte LDS
// reads; rows 8 bytes longer than the data keep them to two-way bank conflicts) and
// runs block_core.  Codes and steps are token-major, as from the token-major sweep.
// ---------------------------------------------------------------------------
template <typename T, int TC>
__global__ __launch_bounds__(256) void k_quantize_blocks_chw(
    const T* __restrict__ X, long long ld_c, long long ld_b, int C, int T_, int vin_ok, int q_vec_ok,
    int kq, int kp, Scalars sc, uint8_t* __restrict__ Q, long long ld_q, float* __restrict__ bscale,
    float* __restrict__ bclip, long long ld_s) {
  constexpr bool PK = sizeof(T) == 2;
  constexpr int NB = PK ? 2 : 1;
  constexpr int W = PK ? 4 : 8;
  constexpr int E = 16 / (int)sizeof(T);                   // elements per 16 bytes
  constexpr int TT = 16 * E;                               // tokens per tile
  constexpr int PITCH = TT + 8 / (int)sizeof(T);
  constexpr int QPT = TC / (kBlk * NB);                    // quads per token and tile
  __shared__ __attribute__((aligned(16))) T tile[TC][PITCH];

  const int t0 = blockIdx.x * TT, b = blockIdx.y;
  const int tid = threadIdx.x, ql = tid & 3;
  const T* xb = X + (long long)b * ld_b;
  const int KB = (C + kBlk - 1) / kBlk;

  for (int c0 = 0; c0 < C; c0 += TC) {
    {
      const int p = tid & 15;
      const int tok = t0 + p * E;
#pragma unroll
      for (int i = 0; i < TC / 16; ++i) {
        const int ch = (tid >> 4) + 16 * i;
        const int c = c0 + ch;
        __attribute__((aligned(16))) T v[E];
        if (c < C && vin_ok && tok + E <= T_) {
          *reinterpret_cast<uint4*>(v) = *reinterpret_cast<const uint4*>(xb + (long long)c * ld_c + tok);
        } else {
          // channels at and beyond C are the zero padding of the last block
#pragma unroll
          for (int k = 0; k < E; ++k)
            v[k] = (c < C && tok + k < T_) ? xb[(long long)c * ld_c + tok + k] : (T)0;
        }
        uint2* d = reinterpret_cast<uint2*>(&tile[ch][p * E]);
        const uint2* sp = reinterpret_cast<const uint2*>(v);
        d[0] = sp[0];
        d[1] = sp[1];
      }
    }
    __syncthreads();
#pragma unroll 1
    for (int pass = 0; pass < TT * QPT / 64; ++pass) {
      const int qd = (tid >> 2) + 64 * pass;
      const int tl = qd / QPT, sub = qd % QPT;
      u32 raw[NB][W];
#pragma unroll
      for (int s = 0; s < NB; ++s) {
        const int chb = (sub * NB + s) * kBlk + ql * 8;
#pragma unroll
        for (int w = 0; w < W; ++w) {
          if constexpr (PK) {
            const u32 lo = tile[chb + 2 * w][tl], hi = tile[chb + 2 * w + 1][tl];
            raw[s][w] = lo | (hi << 16);
          } else {
            raw[s][w] = __float_as_uint(tile[chb + w][tl]);
          }
        }
      }
      u32 word[NB];
      float cs[NB], ds[NB];
      block_core<T>(raw, ql, kq, kp, sc, word, cs, ds);
      const bool tok_ok = t0 + tl < T_;
      const long long row = (long long)b * T_ + t0 + tl;
#pragma unroll
      for (int s = 0; s < NB; ++s) {
        const int kb = c0 / kBlk + sub * NB + s;
        if (tok_ok && kb < KB)
          block_store(word[s], cs[s], ds[s], ql == s, row, kb, ql, C, q_vec_ok, Q, ld_q, bscale,
                      bclip, ld_s);
      }
    }
    __syncthreads();
  }
}

template <typename T>
static hipError_t quantize_blocks_chw_t(const T* X, int B, int C, int T_, long long ld_c,
                                        long long ld_b, int kq, int kp, const Scalars& sc,
                                        uint8_t* Q, long long ld_q, float* bscale, float* bclip,
                                        long long ld_s, hipStream_t st) {
  constexpr int E = 16 / (int)sizeof(T);
  const int vin_ok =
      ((reinterpret_cast<uintptr_t>(X) & 15) == 0 && ld_c % E == 0 && ld_b % E == 0) ? 1 : 0;
  const int q_vec_ok = ((reinterpret_cast<uintptr_t>(Q) & 3) == 0 && ld_q % 4 == 0) ? 1 : 0;
  const dim3 grid((unsigned)((T_ + 16 * E - 1) / (16 * E)), (unsigned)B);
  // 128-channel tiles: 256-channel ones (whole 128-byte lines of codes per token) measured
  // 20 % slower, with half as many workgroups per CU to hide the tile loads
  hipLaunchKernelGGL((k_quantize_blocks_chw<T, 128>), grid, dim3(256), 0, st, X, ld_c, ld_b, C, T_,
                     vin_ok, q_vec_ok, kq, kp, sc, Q, ld_q, bscale, bclip, ld_s);
  return hipGetLastError();
}

hipError_t launch_quantize_blocks_chw(const void* X, tdq_dtype dt, int B, int C, int T, long long ld_c,
                                      long long ld_b, int kq, int kp, const Scalars& sc, uint8_t* Q,
                                      long long ld_q, float* bscale, float* bclip, long long ld_s,
                                      hipStream_t st) {
  if (dt == TDQ_F16)
    return quantize_blocks_chw_t<u16>(static_cast<const u16*>(X), B, C, T, ld_c, ld_b, kq, kp, sc, Q,
                                      ld_q, bscale, bclip, ld_s, st);
  return quantize_blocks_chw_t<float>(static_cast<const float*>(X), B, C, T, ld_c, ld_b, kq, kp, sc, Q,
                                      ld_q, bscale, bclip, ld_s, st);
}

}  // namespace tdq
