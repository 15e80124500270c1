// Rank select of the zr quantile for binary16 activations in ONE sweep of X
// (constraint C2 of DCRP, Eq. zr_constraint: the k-th smallest |x| of every
// (image, token set), k = ceil(zr n), Supp. "Quantile Implementation").
//
// The magnitude key of a binary16 value has 15 bits.  A radix select over LDS
// histograms needs two sweeps of X for that many bits.  Here a small sample of
// every set first says where to look:
//
//   k_bracket         one workgroup per set reads up to 16 Ki sampled elements and
//                     finds, in an LDS histogram of their top key bits, the sample
//                     order statistic whose sample rank corresponds to k.  The key
//                     interval [lo, lo + W) centred on it (W = as many one-key bins as
//                     the LDS histogram has per set) holds the true answer unless the
//                     sample is off by more than W/2 keys.
//   k_bracket_hist    one sweep of X: per set, the number of keys below lo and an LDS
//                     histogram, one bin per key, of the keys inside the interval.
//   k_bracket_finish  one workgroup per set: if below < k <= below + inside, the
//                     answer is the bin where the running count reaches k - below --
//                     the exact k-th smallest, no matter how the interval was chosen --
//                     and the set is projected.  Otherwise the set is counted as missed
//                     and the same workgroup resolves it with a two-level radix select
//                     over the set's own rows (exact as well, and rare).
//
// The result is therefore always the exact order statistic; the sample only decides
// which of the two routes computes it, i.e. how long it takes.
#include "tdq_device.hpp"

namespace tdq {

constexpr int kSampleThreads = 256;                             // one wavefront per SIMD
constexpr int kSampleWaves = kSampleThreads / 64;
constexpr int kSamplePerThread = 64;
constexpr int kRunLen = 32;                                     // channels per run (64 bytes)
constexpr int kSampleMax = kSampleThreads * kSamplePerThread;   // 16 Ki keys per set
constexpr int kSampleRuns = kSampleMax / kRunLen;               // 512 runs
constexpr int kSampleTokens = kSampleRuns;                      // at most one run per token
constexpr int kSampleBits = 10;                                 // key bits the sample histogram resolves
constexpr int kSweepThreads = 1024;

// ---------------------------------------------------------------------------
// k_bracket
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kSampleThreads) void k_bracket(
    const u16* __restrict__ X, long long ld, int T, int C, int G, int W, int vec,
    const int* __restrict__ gid, const SetAcc* __restrict__ part, int S, Scalars sc, int pass,
    int keep_base, GroupWork* __restrict__ grp, Bracket* __restrict__ br,
    u32* __restrict__ bhist) {
  __shared__ int sel[kSampleTokens];                 // drawn token of every stratum
  __shared__ long long run_base[kSampleRuns];        // element offset of every run's first channel
  __shared__ int run_len[kSampleRuns];               // channels of the run (<= kRunLen)
  __shared__ u32 shist[1 << kSampleBits];            // sample histogram over the top key bits
  __shared__ u32 wtot[kSampleWaves];
  __shared__ u32 s_bin;
  const int idx = blockIdx.x;
  const int b = idx / G, j = idx - b * G;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // the set ids of the first batch of tokens are on their way while the records are merged
  constexpr int kRankBatch = 16;
  const int* gb = gid + (long long)b * T;
  int gv[kRankBatch];
#pragma unroll
  for (int u = 0; u < kRankBatch; ++u) {
    const int t = u * kSampleThreads + tid;
    gv[u] = t < T ? gb[t] : -1;
  }
  // every thread merges the assignment's partial records of this set (same loads, same
  // order, same result); one of them stores the working record for the later kernels
  GroupWork w = merge_partials(part, b, j, S, G, C, sc, pass);
  if (keep_base) w.c_base = grp[idx].c_base;     // left by the base-radius pass (only this
                                                 // field is read; thread 0 rewrites it unchanged)
  if (tid == 0) grp[idx] = w;

  // the sweep adds into this set's histogram and counter: clear them here
  for (int i = tid; i < W; i += kSampleThreads) bhist[(size_t)idx * W + i] = 0;
  if (w.tokens == 0) {
    if (tid == 0) {
      Bracket e;
      e.lo = 0; e.width = 0; e.below = 0; e.pad = 0;
      br[idx] = e;
    }
    return;
  }

  // Sample geometry.  The set's tokens, in index order, are cut into strata of
  // `stride` tokens (at most kSampleTokens strata) and one token is drawn from each
  // at a hashed position: a regular stride would alias with any period the token
  // sequence has (image rows).  Of each drawn token `rpt` runs of kRunLen consecutive
  // channels are read, the first at a hashed offset, so that all channels are
  // represented; a row that fits is read whole.
  const int tokens = (int)w.tokens;
  const int stride = (tokens + kSampleTokens - 1) / kSampleTokens;
  const int n_sel = (tokens + stride - 1) / stride;         // <= kSampleTokens
  const int row_runs = (C + kRunLen - 1) / kRunLen;
  int rpt = kSampleRuns / n_sel;                            // runs per drawn token, >= 1
  rpt = rpt < row_runs ? rpt : row_runs;
  const int cw = rpt == row_runs ? C : rpt * kRunLen;       // channels read per drawn token
  const int n_runs = n_sel * rpt;                           // <= kSampleRuns
  const long long m = (long long)n_sel * cw;                // sample size, <= kSampleMax

  // Rank of every token inside its set -> the drawn tokens' indices.  Tokens are taken
  // kRankBatch rounds of kSampleThreads at a time: all set ids of a batch are loaded
  // together, every wavefront counts its matches of every round (ballot), the counts meet
  // in LDS once, and every thread turns them into the rank offsets of its own wavefront --
  // two barriers per batch instead of two per round.
  __shared__ u32 wcnt[kRankBatch * kSampleWaves];
  u32 base = 0;
  for (int t0 = 0; t0 < T; t0 += kRankBatch * kSampleThreads) {
    if (t0 > 0) {
#pragma unroll
      for (int u = 0; u < kRankBatch; ++u) {
        const int t = t0 + u * kSampleThreads + tid;
        gv[u] = t < T ? gb[t] : -1;
      }
    }
    u32 within[kRankBatch];
#pragma unroll
    for (int u = 0; u < kRankBatch; ++u) {
      const unsigned long long mask = __ballot(gv[u] == j);
      within[u] = (u32)__popcll(mask & ((1ull << lane) - 1ull));
      if (lane == 0) wcnt[u * kSampleWaves + wave] = (u32)__popcll(mask);
    }
    __syncthreads();
    u32 run = base;
#pragma unroll
    for (int u = 0; u < kRankBatch; ++u) {
      u32 mine = 0;
#pragma unroll
      for (int w2 = 0; w2 < kSampleWaves; ++w2) {
        const u32 v = wcnt[u * kSampleWaves + w2];
        mine = w2 == wave ? run : mine;
        run += v;
      }
      if (gv[u] == j) {
        const int t = t0 + u * kSampleThreads + tid;
        const u32 rank = mine + within[u];
        const u32 stratum = rank / (u32)stride, first = stratum * (u32)stride;
        const u32 len = (u32)tokens - first < (u32)stride ? (u32)tokens - first : (u32)stride;
        const u32 pick =
            first + (((stratum + 1u) * 2246822519u + (u32)idx * 3266489917u) >> 12) % len;
        if (rank == pick) sel[stratum] = t;
      }
    }
    base = run;
    __syncthreads();                     // wcnt is rewritten by the next batch; sel is read below
  }
  // table of runs, so that the load loop below has no division in it
  for (int q = tid; q < kSampleRuns; q += kSampleThreads) {
    long long rb = 0;
    int rl = 0;
    if (q < n_runs) {
      const int slot = q / rpt, run = q - slot * rpt;
      const int t = sel[slot];
      // (whole 16-byte pieces when the rows allow 16-byte loads: C, cw and the offset are
      // then multiples of 8 channels)
      const u32 off = vec ? (((u32)t * 2654435761u >> 8) % (u32)((C - cw) / 8 + 1)) * 8u
                          : ((u32)t * 2654435761u >> 8) % (u32)(C - cw + 1);
      rb = ((long long)b * T + t) * ld + off + run * kRunLen;
      rl = cw - run * kRunLen;
      rl = rl < kRunLen ? rl : kRunLen;
    } else {
      rb = ((long long)b * T + sel[0]) * ld;          // a valid address; the key is discarded
    }
    run_base[q] = rb;
    run_len[q] = rl;
  }
  __syncthreads();

  // The sample.  Every live key adds one to an LDS histogram of its top kSampleBits bits.
  // Loads are issued unconditionally (from a clamped, valid address) so that they overlap.
  for (int i = tid; i < (1 << kSampleBits); i += kSampleThreads) shist[i] = 0;
  if (vec) {
    // 16-byte pieces of 8 channels: piece p = 256 e + tid is part p % 4 of run p / 4, so a
    // wavefront's load instruction fetches 16 whole runs of 64 bytes; a run's pieces are
    // all live or (runs past the end of the table) all dead.
    constexpr int kPieces = kSampleMax / 8 / kSampleThreads;      // 8 per thread
    uint4 v[kPieces];
    bool live[kPieces];
#pragma unroll
    for (int e = 0; e < kPieces; ++e) {
      const int p = e * kSampleThreads + tid;
      const int q = p >> 2, part = p & 3;
      live[e] = part * 8 < run_len[q];
      v[e] = *reinterpret_cast<const uint4*>(X + run_base[q] + (live[e] ? part * 8 : 0));
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < kPieces; ++e) {
      if (live[e]) {
        const u32 wd[4] = {v[e].x, v[e].y, v[e].z, v[e].w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          atomicAdd(&shist[(wd[i] & 0x7FFFu) >> (15 - kSampleBits)], 1u);
          atomicAdd(&shist[((wd[i] >> 16) & 0x7FFFu) >> (15 - kSampleBits)], 1u);
        }
      }
    }
  } else {
    // element e of lane l of wavefront w is channel l % 32 of run 8 e + 2 w + l / 32
    u32 key[kSamplePerThread];
    const int half = lane >> 5, cl = lane & 31;
#pragma unroll
    for (int e = 0; e < kSamplePerThread; ++e) {
      const int q = e * (2 * kSampleWaves) + 2 * wave + half;
      const int rl = run_len[q];
      const int ch = cl < rl ? cl : (rl > 0 ? rl - 1 : 0);
      const u32 x = X[run_base[q] + ch];
      key[e] = cl < rl ? (x & 0x7FFFu) : 0xFFFFu;
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < kSamplePerThread; ++e)
      if (key[e] != 0xFFFFu) atomicAdd(&shist[key[e] >> (15 - kSampleBits)], 1u);
  }
  __syncthreads();

  // Sample rank that corresponds to rank k of the set, and the histogram bin that
  // holds that order statistic (the low key bits do not matter to the interval).
  const double n = (double)w.n, kd = (double)w.k_rem;
  long long r = (long long)(kd / n * (double)m + 0.5);
  r = r < 1 ? 1 : (r > m ? m : r);
  constexpr int kBinsPerThread = (1 << kSampleBits) / kSampleThreads;
  u32 c[kBinsPerThread], mine = 0;
#pragma unroll
  for (int i = 0; i < kBinsPerThread; ++i) {
    c[i] = shist[tid * kBinsPerThread + i];
    mine += c[i];
  }
  u32 incl = mine;                           // inclusive scan over the wavefront
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const u32 o = (u32)__shfl_up((int)incl, d, 64);
    if (lane >= d) incl += o;
  }
  if (lane == 63) wtot[wave] = incl;
  __syncthreads();
  u32 before = 0;
#pragma unroll
  for (int w2 = 0; w2 < kSampleWaves; ++w2) before += w2 < wave ? wtot[w2] : 0u;
  incl += before;
  if ((long long)(incl - mine) < r && r <= (long long)incl) {     // exactly one thread
    u32 cum = incl - mine;
    int i = 0;
    for (; i < kBinsPerThread - 1; ++i) {
      if ((long long)(cum + c[i]) >= r) break;
      cum += c[i];
    }
    s_bin = (u32)(tid * kBinsPerThread + i);
  }
  __syncthreads();
  const u32 v = s_bin << (15 - kSampleBits);

  if (tid == 0) {
    // v <= estimate < v + 2^(15 - kSampleBits): centre the interval on the middle
    const u32 mid = v + (1u << (14 - kSampleBits));
    Bracket e;
    e.below = 0; e.pad = 0;
    e.lo = mid > (u32)W / 2 ? mid - (u32)W / 2 : 0u;
    e.width = (u32)W;
    br[idx] = e;
  }
}

hipError_t launch_bracket(const void* X, int B, int T, int C, long long ld, int G, int W,
                          const int* gid, const void* part, const Scalars& sc, int pass,
                          bool keep_base, GroupWork* grp, Bracket* br, unsigned* bhist,
                          hipStream_t st) {
  // 16-byte sample loads need rows of whole, aligned 16-byte pieces
  const int vec = ((reinterpret_cast<uintptr_t>(X) & 15) == 0 && ld % 8 == 0 && C % 8 == 0) ? 1 : 0;
  hipLaunchKernelGGL(k_bracket, dim3(B * G), dim3(kSampleThreads), 0, st,
                     static_cast<const u16*>(X), ld, T, C, G, W, vec, gid,
                     static_cast<const SetAcc*>(part), assign_split(T), sc, pass,
                     keep_base ? 1 : 0, grp, br, bhist);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// k_bracket_hist: the one sweep
// ---------------------------------------------------------------------------
typedef short s2v __attribute__((ext_vector_type(2)));

template <int L>
__global__ __launch_bounds__(kSweepThreads) void k_bracket_hist(
    const u16* __restrict__ X, long long ld, int T_, int C, int G, int W, int vec_ok,
    const int* __restrict__ gid, Bracket* __restrict__ br, u32* __restrict__ bhist,
    int rows_per_block) {
  extern __shared__ u32 lds[];                    // [G][W] bins, then per set: below, lo, width
  // walks X backwards: it runs right after the forward statistics sweep, so the end of
  // X is what the last-level cache still holds
  const int b = (int)(gridDim.y - 1 - blockIdx.y);
  const int chunk = (int)(gridDim.x - 1 - blockIdx.x);
  const int tid = threadIdx.x;
  const int nwords = G * W;
  u32* s_below = lds + nwords;
  u32* s_lo = s_below + G;
  u32* s_width = s_lo + G;
  for (int i = tid; i < nwords + G; i += kSweepThreads) lds[i] = 0;
  for (int g = tid; g < G; g += kSweepThreads) {
    const Bracket e = br[(long long)b * G + g];
    s_lo[g] = e.lo;
    s_width[g] = e.width;
  }
  __syncthreads();

  const int row0 = chunk * rows_per_block;
  int nrows = T_ - row0;
  nrows = nrows < rows_per_block ? nrows : rows_per_block;
  constexpr int SLOTS = kSweepThreads / L;
  const int slot = tid / L, lr = tid % L;
  const int nvec = vec_ok ? C / 8 : 0;
  for (int rr = slot; rr < nrows; rr += SLOTS) {
    const long long row = (long long)b * T_ + row0 + rr;
    const int g = gid[row];
    const u32 lo = s_lo[g], width = s_width[g];
    const u32 lo2 = lo | (lo << 16);
    u32* h = lds + g * W;
    const u16* xp = X + row * ld;
    u32 below = 0;
#pragma unroll 2
    for (int v = lr; v < nvec; v += L) {
      const uint4 q = *reinterpret_cast<const uint4*>(xp + (long long)v * 8);
      const u32 wd[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        // both halves at once: keys and lo are below 2^15, so the 16-bit differences
        // cannot overflow and their sign bits say "key < lo"
        const s2v d = __builtin_bit_cast(s2v, wd[i] & 0x7FFF7FFFu) - __builtin_bit_cast(s2v, lo2);
        const u32 d2 = __builtin_bit_cast(u32, d);
        below += (u32)__builtin_popcount(d2 & 0x80008000u);
        const u32 dl = d2 & 0xFFFFu, dh = d2 >> 16;       // negative ones are >= 2^15 > width
        if (dl < width) atomicAdd(&h[dl], 1u);
        if (dh < width) atomicAdd(&h[dh], 1u);
      }
    }
    for (int c = nvec * 8 + lr; c < C; c += L) {
      const u32 k = xp[c] & 0x7FFFu;
      below += k < lo ? 1u : 0u;
      const u32 d = k - lo;
      if (k >= lo && d < width) atomicAdd(&h[d], 1u);
    }
    below = group_sum_u32<L>(below);                       // total in the row's last lane
    if (lr == L - 1 && below) atomicAdd(&s_below[g], below);
  }
  __syncthreads();
  u32* gh = bhist + (size_t)b * G * W;
  for (int i = tid; i < nwords; i += kSweepThreads) {
    const u32 v = lds[i];
    if (v) atomicAdd(&gh[i], v);
  }
  for (int g = tid; g < G; g += kSweepThreads) {
    const u32 v = s_below[g];
    if (v) atomicAdd(&br[(long long)b * G + g].below, v);
  }
}

hipError_t launch_bracket_hist(const void* Xv, int B, int T_, int C, long long ld, int G, int W,
                               const int* gid, Bracket* br, unsigned* bhist, hipStream_t st) {
  const u16* X = static_cast<const u16*>(Xv);
  const int vec_ok = ((reinterpret_cast<uintptr_t>(X) & 15) == 0 && ld % 8 == 0) ? 1 : 0;
  const int L = lanes_per_row(C, 8);
  // two workgroups per CU (measured best of 256 / 384 / 512 / 1024 / 2048: every
  // workgroup flushes up to G * W bins with global atomics), but at least ~64 Ki
  // elements each
  long long rows_min = (65536 + C - 1) / C;
  long long target_blocks = 512 / (B > 0 ? B : 1);
  if (target_blocks < 1) target_blocks = 1;
  long long rpb = (T_ + target_blocks - 1) / target_blocks;
  if (rpb < rows_min) rpb = rows_min;
  if (rpb > T_) rpb = T_;
  const unsigned chunks = (unsigned)((T_ + rpb - 1) / rpb);
  const size_t lds_bytes = ((size_t)G * W + 3 * (size_t)G) * sizeof(u32);
#define TDQ_BH(LL)                                                                              \
  case LL:                                                                                      \
    if (lds_bytes > 65536)                                                                      \
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_bracket_hist<LL>),             \
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);    \
    hipLaunchKernelGGL((k_bracket_hist<LL>), dim3(chunks, B), dim3(kSweepThreads), lds_bytes,   \
                       st, X, ld, T_, C, G, W, vec_ok, gid, br, bhist, (int)rpb);               \
    break;
  switch (L) { TDQ_BH(1) TDQ_BH(2) TDQ_BH(4) TDQ_BH(8) TDQ_BH(16) TDQ_BH(32) TDQ_BH(64) }
#undef TDQ_BH
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// k_bracket_finish: one workgroup per set.  Its first wavefront verifies the interval
// and, on a hit, finishes the set; on a miss the whole workgroup runs the exact
// two-level radix select (8 + 7 key bits, LDS histogram) over the set's own rows.
// ---------------------------------------------------------------------------
constexpr int kFinishThreads = 256;

__global__ __launch_bounds__(kFinishThreads) void k_bracket_finish(
    const u16* __restrict__ X, long long ld, int T, int C, int G, int vec_ok,
    const int* __restrict__ gid, const u32* __restrict__ bhist, int W, int force_miss, Scalars sc,
    int pass, GroupWork* __restrict__ grp, const Bracket* __restrict__ br,
    float* __restrict__ clip, float* __restrict__ scale, tdq_group_stats* __restrict__ stats,
    const u32* __restrict__ img_flag, int B, u32* __restrict__ status) {
  __shared__ u32 h[256];
  __shared__ int list[kFinishThreads];
  __shared__ u32 wtot[kFinishThreads / 64];
  __shared__ u32 s_ok, s_digit;
  __shared__ unsigned long long s_rem;
  const int idx = blockIdx.x;
  const int b = idx / G, j = idx - b * G;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  if (idx == 0 && wave == 0 && pass == kPassZr) {   // fold the per-image flags into the status word
    u32 f = 0;
    for (int bb = lane; bb < B; bb += 64) f |= img_flag[bb];
    const unsigned long long any = __ballot(f != 0);
    if (lane == 0) status[0] = any ? TDQ_DEV_NONFINITE : 0u;
  }
  const GroupWork w = grp[idx];
  if (w.tokens == 0) {
    if (tid == 0 && pass == kPassZr) project_store(idx, w, 0u, true, sc, clip, scale, stats);
    return;
  }
  if (wave == 0) {
    bool ok = false;
    unsigned long long need = 0, mine = 0, incl = 0;
    const u32* hb = bhist + (size_t)idx * W;
    const int per = W / 64;                     // W is a multiple of 64
    const int first = lane * per;
    Bracket e;
    e.lo = 0; e.width = 0; e.below = 0; e.pad = 0;
    if (!force_miss) {
      e = br[idx];
      const unsigned long long k = (unsigned long long)w.k_rem;
      for (int i = 0; i < per; ++i) mine += hb[first + i];
      incl = mine;                              // inclusive scan over lanes
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const unsigned long long o = __shfl_up(incl, d, 64);
        if (lane >= d) incl += o;
      }
      const unsigned long long inside = __shfl(incl, 63, 64);
      ok = k > e.below && k - e.below <= inside;
      need = k - e.below;
    }
    if (ok) {                                   // wavefront-uniform
      const unsigned long long hit = __ballot(incl >= need);
      const int src = __ffsll((long long)hit) - 1;        // hit != 0 because need <= inside
      if (lane == src) {
        unsigned long long cum = incl - mine;
        int i = 0;
        for (; i < per - 1; ++i) {
          const unsigned long long c = hb[first + i];
          if (cum + c >= need) break;
          cum += c;
        }
        const u32 key = e.lo + (u32)(first + i);
        if (pass == kPassBase)
          grp[idx].c_base = h2f(key);            // the set's base radius Q_p(|x|)
        else
          project_store(idx, w, key, true, sc, clip, scale, stats);
      }
    }
    if (lane == 0) s_ok = ok ? 1u : 0u;
  }
  __syncthreads();
  if (s_ok) return;

  // The interval missed rank k (or the validation switch asked for this route).
  if (tid == 0) atomicAdd(&status[1 + pass], 1u);
  const int* gb = gid + (long long)b * T;
  unsigned long long k = (unsigned long long)w.k_rem;
  u32 prefix = 0;
  const int nvec = vec_ok ? C / 8 : 0;
  for (int level = 0; level < 2; ++level) {
    const int shift = level == 0 ? 7 : 0;
    const u32 mask = level == 0 ? 255u : 127u;
    h[tid] = 0;                                 // kFinishThreads == 256 bins
    __syncthreads();
    for (int t0 = 0; t0 < T; t0 += kFinishThreads) {
      // the set's tokens among t0 .. t0 + 255, compacted into `list`
      const int t = t0 + tid;
      const bool match = t < T && gb[t] == j;
      const unsigned long long m = __ballot(match);
      if (lane == 0) wtot[wave] = (u32)__popcll(m);
      __syncthreads();
      u32 before = 0, n_list = 0;
#pragma unroll
      for (int w2 = 0; w2 < kFinishThreads / 64; ++w2) {
        before += w2 < wave ? wtot[w2] : 0u;
        n_list += wtot[w2];
      }
      if (match) list[before + (u32)__popcll(m & ((1ull << lane) - 1ull))] = t;
      __syncthreads();
      for (u32 i = wave; i < n_list; i += kFinishThreads / 64) {     // one wavefront per row
        const u16* xp = X + ((long long)b * T + list[i]) * ld;
        for (int v = lane; v < nvec; v += 64) {
          const uint4 q = *reinterpret_cast<const uint4*>(xp + (long long)v * 8);
          const u32 wd[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const u32 k0 = wd[c] & 0x7FFFu, k1 = (wd[c] >> 16) & 0x7FFFu;
            if (level == 0 || (k0 >> 7) == prefix) atomicAdd(&h[(k0 >> shift) & mask], 1u);
            if (level == 0 || (k1 >> 7) == prefix) atomicAdd(&h[(k1 >> shift) & mask], 1u);
          }
        }
        for (int c = nvec * 8 + lane; c < C; c += 64) {
          const u32 k0 = xp[c] & 0x7FFFu;
          if (level == 0 || (k0 >> 7) == prefix) atomicAdd(&h[(k0 >> shift) & mask], 1u);
        }
      }
      __syncthreads();                          // `list` and `wtot` are reused
    }
    if (tid == 0) {
      unsigned long long cum = 0;
      const int nb = level == 0 ? 256 : 128;
      int bin = 0;
      for (; bin < nb - 1; ++bin) {
        if (cum + h[bin] >= k) break;
        cum += h[bin];
      }
      s_digit = (u32)bin;
      s_rem = k - cum;
    }
    __syncthreads();
    prefix = level == 0 ? s_digit : ((prefix << 7) | s_digit);
    k = s_rem;
    __syncthreads();
  }
  if (tid == 0) {
    if (pass == kPassBase)
      grp[idx].c_base = h2f(prefix);
    else
      project_store(idx, w, prefix, true, sc, clip, scale, stats);
  }
}

hipError_t launch_bracket_finish(const void* Xv, int B, int T, int C, long long ld, int G, int W,
                                 const int* gid, const unsigned* bhist, bool force_miss,
                                 const Scalars& sc, int pass, GroupWork* grp, const Bracket* br,
                                 float* clip, float* scale, tdq_group_stats* stats,
                                 const unsigned* img_flag, unsigned* status, hipStream_t st) {
  const u16* X = static_cast<const u16*>(Xv);
  const int vec_ok = ((reinterpret_cast<uintptr_t>(X) & 15) == 0 && ld % 8 == 0) ? 1 : 0;
  hipLaunchKernelGGL(k_bracket_finish, dim3(B * G), dim3(kFinishThreads), 0, st, X, ld, T, C, G,
                     vec_ok, gid, bhist, W, force_miss ? 1 : 0, sc, pass, grp, br, clip, scale, stats,
                     img_flag, B, status);
  return hipGetLastError();
}

}  // namespace tdq
