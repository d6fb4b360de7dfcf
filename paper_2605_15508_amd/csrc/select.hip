// Online mask generation for STS (gfx950): draft attention scores -> per-head top-k token
// index sets, remapped to the target heads (paper Section 4.2; Section 4.3: one mask per
// speculative batch).
//
// Three ways through, chosen on the host from the shape; one row = one (batch, draft head):
//  * long rows, any budget -- every kernel on a (chunk, row) grid of 8192-token chunks:
//      clear  zero the three digit histograms and the chunk flags of every row
//      agg    A[n] = ((P[0,n] + P[1,n]) + ...) in fp32, stored; histogram of the top 11 key bits
//      hist1  find the first digit of the k-th largest key, histogram the next 11 bits of the
//             keys that share it
//      hist2  same for the last 10 bits
//      write  the k-th largest key T is now known, with r = how many keys equal to T are kept.
//             Ordered compaction: token n is kept iff key > T, or key == T and fewer than r
//             equal keys precede it; its output position is (#greater before n) + min(#equal
//             before n, r). The counts of the chunks before this one come from the words those
//             chunks publish. The list is written to every target head mapped to the draft head.
//  * long rows, small budgets (chunks * budget small enough for one workgroup's LDS, see the
//    host's rule) -- two launches, nothing to clear:
//      local  aggregate a chunk, keep its keys in registers, and rank them inside the chunk: the
//             chunk's own top-k (same tie rule) goes to a pool, in token order. Every token of
//             the row's top-k is in the top-k of its chunk.
//      pool   one workgroup per row ranks the pooled candidates out of LDS and writes the list.
//  * short rows -- one workgroup per row does everything out of LDS (select_small_kernel).
// Keys are the usual order-preserving map of fp32 to uint32 (with -0 folded onto +0), so the
// whole selection is integer arithmetic: the index sets are exact, ties go to the lower token.
// Histograms use LDS atomics per workgroup and integer global atomics to merge (order-free).
#include "common.h"

namespace {

__device__ __forceinline__ uint32_t key_of_bits(uint32_t u) {
  if (u == 0x80000000u) u = 0u;                       // -0 == +0
  // ascending with the float order: negative values have all bits flipped, the others the sign bit set
  return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
}
__device__ __forceinline__ uint32_t key_of(float x) { return key_of_bits(__builtin_bit_cast(uint32_t, x)); }

// exp(s - lse) through the hardware base-2 exponential (about 1 ulp; the product with log2(e)
// adds a relative error below 1e-6 for |s - lse| < 40, far inside the stage-wise tolerance)
__device__ __forceinline__ float prob_of(float s, float lse) {
  return __builtin_amdgcn_exp2f((s - lse) * 1.44269504088896340736f);
}

__device__ __forceinline__ int row_len(const SelectArgs &A, int bt) {
  int nb = A.seq_lens ? A.seq_lens[bt] : A.N;
  return min(max(nb, 0), A.N);
}

// number of ranked units (tokens, or blocks of `page` tokens) in the row of batch bt
__device__ __forceinline__ int src_len(const SelectArgs &A, int bt) {
  return (row_len(A, bt) + A.page - 1) / A.page;
}

// Inclusive prefix sum over the 64 lanes of a wave with data-parallel-primitive moves (no LDS
// round trips): shifts by 1, 2, 4, 8 inside each row of 16 lanes (a lane whose source lies
// outside its row adds 0), then lane 15 of row 0 / 2 is added to row 1 / 3, then lane 31 to
// rows 2 and 3.
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
  int x = (int)v;
  x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, false);   // row_shr:1
  x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, false);   // row_shr:2
  x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xf, 0xf, false);   // row_shr:4
  x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xf, 0xf, false);   // row_shr:8
  x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
  x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
  return (uint32_t)x;
}

// exclusive prefix sum of one value per thread over a THREADS-thread block; also returns the
// total. lds_wave_tot needs THREADS/64 words.
template <int THREADS = SEL_THREADS>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t *lds_wave_tot, uint32_t &total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t incl = wave_incl_scan(v);
  if (lane == 63) lds_wave_tot[wave] = incl;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < THREADS / 64; ++w) {
    const uint32_t t = lds_wave_tot[w];
    if (w < wave) base += t;
    tot += t;
  }
  __syncthreads();
  total = tot;
  return base + incl - v;
}

// Walk a digit histogram from the top: the digit holding the krem-th largest key of the
// candidates, and how many keys of that digit are still wanted. Requires 1 <= krem <= total.
// lds_tmp needs THREADS/64 + 2 words; the result lands in its last two.
template <int NBINS, int THREADS = SEL_THREADS>
__device__ __forceinline__ void find_digit(const uint32_t *hist, uint32_t krem, uint32_t *lds_tmp,
                                           uint32_t &digit, uint32_t &krem_next) {
  constexpr int PER = NBINS / THREADS;
  constexpr int RES = THREADS / 64;
  uint32_t loc[PER], sum = 0;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    loc[i] = hist[threadIdx.x * PER + i];
    sum += loc[i];
  }
  uint32_t total;
  const uint32_t excl = block_excl_scan<THREADS>(sum, lds_tmp, total);
  uint32_t above = total - excl - sum;   // keys in bins owned by higher threads
#pragma unroll
  for (int i = PER - 1; i >= 0; --i) {
    if (above < krem && above + loc[i] >= krem) {
      lds_tmp[RES] = threadIdx.x * PER + i;
      lds_tmp[RES + 1] = krem - above;
    }
    above += loc[i];
  }
  __syncthreads();
  digit = lds_tmp[RES];
  krem_next = lds_tmp[RES + 1];
  __syncthreads();
}

// ------------------------------------------------------------------- aggregation of a row
// The Tq score rows of one (batch, draft head), reduced per token strictly in row order.
struct AggRow {
  const void *P;    // [Tq][N] fp32, or bf16 bit patterns
  const float *L;   // [Tq] natural-log normalisers (scaled-logit input) or nullptr
  int Tq, N;
  bool bf16, logits, use_max;
};

__device__ __forceinline__ AggRow agg_row(const SelectArgs &A, int row) {
  AggRow R;
  const size_t off = (size_t)row * A.Tq * A.N;
  R.bf16 = A.scores_bf16 != 0;
  R.P = R.bf16 ? static_cast<const void *>(static_cast<const uint16_t *>(A.scores) + off)
               : static_cast<const void *>(static_cast<const float *>(A.scores) + off);
  R.L = A.lse ? A.lse + (size_t)row * A.Tq : nullptr;
  R.Tq = A.Tq;
  R.N = A.N;
  R.logits = A.kind == STS_SCORES_LOGITS_LSE;
  R.use_max = A.reduce == STS_REDUCE_MAX;
  return R;
}

// One score (V = float) or four consecutive ones (V = f32x4, n % 4 == 0) of row i, as stored:
// the raw load, and its exact widening to fp32. Nontemporal: every score is read exactly once.
template <class V, bool BF16>
struct ScoreLoad;
template <>
struct ScoreLoad<float, false> {
  typedef float raw;
  static __device__ __forceinline__ raw load(const AggRow &R, int i, int n) {
    return __builtin_nontemporal_load(static_cast<const float *>(R.P) + (size_t)i * R.N + n);
  }
  static __device__ __forceinline__ float widen(raw x) { return x; }
};
template <>
struct ScoreLoad<f32x4, false> {
  typedef f32x4 raw;
  static __device__ __forceinline__ raw load(const AggRow &R, int i, int n) {
    return __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(static_cast<const float *>(R.P) + (size_t)i * R.N + n));
  }
  static __device__ __forceinline__ f32x4 widen(raw x) { return x; }
};
template <>
struct ScoreLoad<float, true> {
  typedef uint16_t raw;
  static __device__ __forceinline__ raw load(const AggRow &R, int i, int n) {
    return __builtin_nontemporal_load(static_cast<const uint16_t *>(R.P) + (size_t)i * R.N + n);
  }
  static __device__ __forceinline__ float widen(raw x) { return __builtin_bit_cast(float, (uint32_t)x << 16); }
};
template <>
struct ScoreLoad<f32x4, true> {
  typedef u32x2 raw;   // four bf16 values, 8-byte aligned
  static __device__ __forceinline__ raw load(const AggRow &R, int i, int n) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(static_cast<const uint16_t *>(R.P) + (size_t)i * R.N + n));
  }
  static __device__ __forceinline__ f32x4 widen(raw x) {
    return f32x4{__builtin_bit_cast(float, x[0] << 16), __builtin_bit_cast(float, x[0] & 0xffff0000u),
                 __builtin_bit_cast(float, x[1] << 16), __builtin_bit_cast(float, x[1] & 0xffff0000u)};
  }
};

// NROWS consecutive score rows, from row i on, of the token(s) at each of the NPOS positions n[]:
// all loads first (their latencies overlap), then the reduction strictly in row order. FIRST: row
// i is row 0 and initialises the accumulators.
template <int NROWS, bool FIRST, bool BF16, int NPOS, class V>
__device__ __forceinline__ void agg_rows(const AggRow &R, int i, const int (&n)[NPOS], V (&acc)[NPOS]) {
  typedef ScoreLoad<V, BF16> SL;
  typename SL::raw raw[NPOS][NROWS];
#pragma unroll
  for (int x = 0; x < NPOS; ++x)
#pragma unroll
    for (int u = 0; u < NROWS; ++u) raw[x][u] = SL::load(R, i + u, n[x]);
#pragma unroll
  for (int x = 0; x < NPOS; ++x)
#pragma unroll
    for (int u = 0; u < NROWS; ++u) {
      V p = SL::widen(raw[x][u]);
      if (R.logits) {
        const float l = R.L[i + u];
        if constexpr (sizeof(V) == sizeof(float)) {
          p = prob_of(p, l);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) p[e] = prob_of(p[e], l);
        }
      }
      if (FIRST && u == 0) {
        acc[x] = p;
      } else if (R.use_max) {
        if constexpr (sizeof(V) == sizeof(float)) {
          acc[x] = fmaxf(acc[x], p);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[x][e] = fmaxf(acc[x][e], p[e]);
        }
      } else {
        acc[x] = acc[x] + p;
      }
    }
}

template <bool FIRST, bool BF16, int NPOS, class V>
__device__ __forceinline__ void agg_group(const AggRow &R, int i, int rows, const int (&n)[NPOS], V (&acc)[NPOS]) {
  switch (rows) {   // uniform: a scalar branch; every case is straight-line code
    case 1: agg_rows<1, FIRST, BF16>(R, i, n, acc); break;
    case 2: agg_rows<2, FIRST, BF16>(R, i, n, acc); break;
    case 3: agg_rows<3, FIRST, BF16>(R, i, n, acc); break;
    case 4: agg_rows<4, FIRST, BF16>(R, i, n, acc); break;
    case 5: agg_rows<5, FIRST, BF16>(R, i, n, acc); break;
    case 6: agg_rows<6, FIRST, BF16>(R, i, n, acc); break;
    case 7: agg_rows<7, FIRST, BF16>(R, i, n, acc); break;
    default: agg_rows<8, FIRST, BF16>(R, i, n, acc); break;
  }
}

// aggregated score(s) at NPOS positions at once: rows in groups of up to 8 loads per position in
// flight
template <class V, int NPOS>
__device__ __forceinline__ void agg_multi(const AggRow &R, const int (&n)[NPOS], V (&acc)[NPOS]) {
  if (R.bf16) {
    agg_group<true, true>(R, 0, min(R.Tq, 8), n, acc);
    for (int i = 8; i < R.Tq; i += 8) agg_group<false, true>(R, i, min(R.Tq - i, 8), n, acc);
  } else {
    agg_group<true, false>(R, 0, min(R.Tq, 8), n, acc);
    for (int i = 8; i < R.Tq; i += 8) agg_group<false, false>(R, i, min(R.Tq - i, 8), n, acc);
  }
}

// the same for a caller that knows Tq <= MAXG (MAXG <= 8): only those cases are compiled, so many
// positions in flight do not cost the registers of eight rows each
template <bool BF16, int MAXG, int NPOS, class V>
__device__ __forceinline__ void agg_group_lim(const AggRow &R, int rows, const int (&n)[NPOS], V (&acc)[NPOS]) {
  if constexpr (MAXG <= 1) {
    agg_rows<1, true, BF16>(R, 0, n, acc);
  } else {
    if (rows >= MAXG) agg_rows<MAXG, true, BF16>(R, 0, n, acc);
    else agg_group_lim<BF16, MAXG - 1>(R, rows, n, acc);
  }
}
template <class V, int NPOS, int MAXG>
__device__ __forceinline__ void agg_multi_lim(const AggRow &R, const int (&n)[NPOS], V (&acc)[NPOS]) {
  if constexpr (MAXG >= 8) {
    agg_multi<V, NPOS>(R, n, acc);
  } else {
    if (R.bf16) agg_group_lim<true, MAXG>(R, R.Tq, n, acc);
    else agg_group_lim<false, MAXG>(R, R.Tq, n, acc);
  }
}

template <class V>
__device__ __forceinline__ V agg_at(const AggRow &R, int n) {
  const int pos[1] = {n};
  V acc[1];
  agg_multi<V, 1>(R, pos, acc);
  return acc[0];
}

__device__ __forceinline__ f32x4 agg_quad(const AggRow &R, int n) { return agg_at<f32x4>(R, n); }
__device__ __forceinline__ float agg_one(const AggRow &R, int n) { return agg_at<float>(R, n); }

// Add a workgroup's LDS histogram to the row's global one. Two neighbouring 32-bit bins travel
// in one 64-bit atomic (a row holds fewer than 2^32 keys, so the low bin never carries into
// the high one), which halves the number of atomics.
template <int NBINS, int THREADS = SEL_THREADS>
__device__ __forceinline__ void flush_hist(uint32_t *global_bins, const uint32_t *lds_bins) {
  unsigned long long *g2 = reinterpret_cast<unsigned long long *>(global_bins);
  for (int i = threadIdx.x; i < NBINS / 2; i += THREADS) {
    const unsigned long long v = (unsigned long long)lds_bins[2 * i] | ((unsigned long long)lds_bins[2 * i + 1] << 32);
    if (v) atomicAdd(&g2[i], v);
  }
}

__global__ void __launch_bounds__(SEL_THREADS) select_clear_kernel(uint32_t *p, size_t n) {
  const size_t i = (size_t)blockIdx.x * SEL_THREADS + threadIdx.x;
  if (i < n) p[i] = 0u;
}

__global__ void __launch_bounds__(SEL_THREADS) select_clear16_kernel(u32x4 *p, size_t n) {
  const size_t i = (size_t)blockIdx.x * SEL_THREADS + threadIdx.x;
  if (i < n) p[i] = u32x4{0u, 0u, 0u, 0u};
}

// --------------------------------------------------------------------------- aggregation
template <bool VEC4>
__global__ void __launch_bounds__(SEL_THREADS) select_agg_kernel(const SelectArgs A) {
  __shared__ uint32_t h[SEL_BINS];
  const int row = blockIdx.y, chunk = blockIdx.x;
  const int bt = row / A.Hd;
  const int nb = row_len(A, bt);
  for (int i = threadIdx.x; i < SEL_BINS; i += SEL_THREADS) h[i] = 0u;
  __syncthreads();
  const AggRow R = agg_row(A, row);
  float *out = A.agg + (size_t)row * A.N;
  const int n0 = chunk * SEL_CHUNK;
  const int n1 = min(n0 + SEL_CHUNK, A.N);
  if (VEC4) {
    // The chunk's sums wait in registers and are stored in one burst after the last read: a
    // write stream mixed into the read stream costs this memory system far more than its bytes,
    // and with the workgroups of a launch running in step the two phases separate chip-wide.
    constexpr int IT = SEL_CHUNK / (SEL_THREADS * 4);
    f32x4 keep[IT];
#pragma clang loop unroll(full)
    for (int i = 0; i < IT; ++i) {
      const int n = n0 + (i * SEL_THREADS + (int)threadIdx.x) * 4;
      if (n < n1) {
        keep[i] = agg_quad(R, n);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (A.page == 1 && n + e < nb) atomicAdd(&h[key_of(keep[i][e]) >> (32 - SEL_BITS0)], 1u);
      }
    }
    if (!A.agg_is_input) {
#pragma clang loop unroll(full)
      for (int i = 0; i < IT; ++i) {
        const int n = n0 + (i * SEL_THREADS + (int)threadIdx.x) * 4;
        if (n < n1) {
          f32x4 o = keep[i];
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (n + e >= nb) o[e] = 0.f;          // the stored aggregate is 0 past the valid length
          *reinterpret_cast<f32x4 *>(out + n) = o;
        }
      }
    }
  } else {
    for (int n = n0 + threadIdx.x; n < n1; n += SEL_THREADS) {
      const float acc = agg_one(R, n);
      if (!A.agg_is_input) out[n] = n < nb ? acc : 0.f;
      if (A.page == 1 && n < nb) atomicAdd(&h[key_of(acc) >> (32 - SEL_BITS0)], 1u);
    }
  }
  __syncthreads();
  if (A.page != 1) return;   // block granularity: the block kernel builds the first histogram
  uint32_t *gh = A.hist + (size_t)row * 3 * SEL_BINS;
  flush_hist<SEL_BINS>(gh, h);
}

// ----------------------------------------------------------------------- block scores
// One thread per block: the block's aggregated scores added left to right in fp32 (tokens
// below the valid length only), stored, and counted into the first-digit histogram.
__global__ void __launch_bounds__(SEL_THREADS) select_block_kernel(const SelectArgs A) {
  __shared__ uint32_t h[SEL_BINS];
  const int row = blockIdx.y;
  const int bt = row / A.Hd;
  const int nb = row_len(A, bt);
  const int nblk = (nb + A.page - 1) / A.page;
  for (int i = threadIdx.x; i < SEL_BINS; i += SEL_THREADS) h[i] = 0u;
  __syncthreads();
  const float *a = A.agg + (size_t)row * A.N;
  float *out = A.blk + (size_t)row * A.srcN;
  const int m = blockIdx.x * SEL_THREADS + threadIdx.x;
  if (m < A.srcN) {
    float acc = 0.f;
    const int n0 = m * A.page;
    const int n1 = min(n0 + A.page, nb);
    for (int n = n0; n < n1; ++n) acc = (n == n0) ? a[n] : acc + a[n];
    out[m] = acc;
    if (m < nblk) atomicAdd(&h[key_of(acc) >> (32 - SEL_BITS0)], 1u);
  }
  __syncthreads();
  uint32_t *gh = A.hist + (size_t)row * 3 * SEL_BINS;
  flush_hist<SEL_BINS>(gh, h);
}

// Coalesced variant for page % 4 == 0, page <= 256, N % 4 == 0: every lane loads 4 consecutive
// tokens and the page/4 lanes of a block pass a running sum from left to right, so the
// additions happen in exactly the order of the one-thread-per-block kernel above.
__global__ void __launch_bounds__(SEL_THREADS) select_block_vec_kernel(const SelectArgs A) {
  __shared__ uint32_t h[SEL_BINS];
  const int row = blockIdx.y;
  const int bt = row / A.Hd;
  const int nb = row_len(A, bt);
  const int nblk = (nb + A.page - 1) / A.page;
  for (int i = threadIdx.x; i < SEL_BINS; i += SEL_THREADS) h[i] = 0u;
  __syncthreads();
  const float *a = A.agg + (size_t)row * A.N;
  float *out = A.blk + (size_t)row * A.srcN;
  const int L = A.page >> 2;                       // lanes per block (1..64, power of two)
  const int lane = threadIdx.x & 63;
  const int pos_in_blk = lane & (L - 1);
  // SEL_CHUNK tokens per workgroup, 1024 per sweep
  for (int n = blockIdx.x * SEL_CHUNK + threadIdx.x * 4; n < min((blockIdx.x + 1) * SEL_CHUNK, A.N);
       n += SEL_THREADS * 4) {
    const f32x4 x = *reinterpret_cast<const f32x4 *>(a + n);
    float run = 0.f;
    bool have = false;                             // whether `run` holds at least one term
    for (int s = 0; s < L; ++s) {
      if (pos_in_blk == s) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (n + e < nb) {
            run = have ? run + x[e] : x[e];
            have = true;
          }
      }
      if (s + 1 < L) {
        const float up = __shfl_up(run, 1, 64);
        const int hup = __shfl_up((int)have, 1, 64);
        if (pos_in_blk == s + 1) {
          run = up;
          have = hup != 0;
        }
      }
    }
    if (pos_in_blk == L - 1) {
      const int m = n / A.page;
      out[m] = run;                                // blocks past the valid length hold 0
      if (m < nblk) atomicAdd(&h[key_of(run) >> (32 - SEL_BITS0)], 1u);
    }
  }
  __syncthreads();
  uint32_t *gh = A.hist + (size_t)row * 3 * SEL_BINS;
  flush_hist<SEL_BINS>(gh, h);
}

// Aggregation and block sums in one pass (page % 4 == 0, page <= 256, N % page == 0, 16-byte
// aligned scores): every lane aggregates 4 consecutive tokens in registers and the page/4
// lanes of a block pass the running sum from left to right, exactly as above; the per-token
// aggregate is stored only when the caller asks for it. With A.hist == nullptr no histogram is
// built (the blocks are ranked out of LDS afterwards).
__global__ void __launch_bounds__(SEL_THREADS) select_aggblock_kernel(const SelectArgs A) {
  __shared__ uint32_t h[SEL_BINS];
  const int row = blockIdx.y;
  const int bt = row / A.Hd;
  const int nb = row_len(A, bt);
  const int nblk = (nb + A.page - 1) / A.page;
  const bool want_hist = A.hist != nullptr;
  if (want_hist) {
    for (int i = threadIdx.x; i < SEL_BINS; i += SEL_THREADS) h[i] = 0u;
    __syncthreads();
  }
  const AggRow R = agg_row(A, row);
  float *tok_out = A.agg ? A.agg + (size_t)row * A.N : nullptr;
  float *out = A.blk + (size_t)row * A.srcN;
  const int L = A.page >> 2;                       // lanes per block (1..64, power of two)
  const int lane = threadIdx.x & 63;
  const int pos_in_blk = lane & (L - 1);
  for (int n = blockIdx.x * SEL_CHUNK + threadIdx.x * 4; n < min((blockIdx.x + 1) * SEL_CHUNK, A.N);
       n += SEL_THREADS * 4) {
    const f32x4 x = agg_quad(R, n);
    if (tok_out) {
      f32x4 o = x;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (n + e >= nb) o[e] = 0.f;
      *reinterpret_cast<f32x4 *>(tok_out + n) = o;
    }
    float run = 0.f;
    bool have = false;                             // whether `run` holds at least one term
    for (int s = 0; s < L; ++s) {
      if (pos_in_blk == s) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (n + e < nb) {
            run = have ? run + x[e] : x[e];
            have = true;
          }
      }
      if (s + 1 < L) {
        const float up = __shfl_up(run, 1, 64);
        const int hup = __shfl_up((int)have, 1, 64);
        if (pos_in_blk == s + 1) {
          run = up;
          have = hup != 0;
        }
      }
    }
    if (pos_in_blk == L - 1) {
      const int m = n / A.page;
      out[m] = run;                                // blocks past the valid length hold 0
      if (want_hist && m < nblk) atomicAdd(&h[key_of(run) >> (32 - SEL_BITS0)], 1u);
    }
  }
  if (!want_hist) return;
  __syncthreads();
  flush_hist<SEL_BINS>(A.hist + (size_t)row * 3 * SEL_BINS, h);
}

// ------------------------------------------------------------------ refinement histograms
// PASS 1: digit 1 (bits 20..10) of keys whose digit 0 matches; PASS 2: digit 2 (bits 9..0)
// of keys whose digits 0 and 1 match.
template <int PASS, bool VEC4>
__global__ void __launch_bounds__(SEL_THREADS) select_hist_kernel(const SelectArgs A) {
  __shared__ uint32_t h[SEL_BINS];
  __shared__ uint32_t tmp[16];
  const int row = blockIdx.y;
  const int chunk0 = blockIdx.x * A.hist_cpw;      // this workgroup takes hist_cpw consecutive chunks
  const int bt = row / A.Hd;
  const int nb = src_len(A, bt);
  const uint32_t c = (uint32_t)min(A.kh[row % A.Hd], nb);
  if (c == 0) return;
  uint32_t *st = A.state + (size_t)row * 8;
  const uint32_t *gh = A.hist + (size_t)row * 3 * SEL_BINS;
  const float *a = A.src + (size_t)row * A.srcN;
  // The first chunk's loads do not depend on the digit search: issue them first so that their
  // latency hides behind it. They are unconditional (a branch around a load makes the compiler
  // wait for it at the join): the address is clamped into the row, out-of-range quads are
  // ignored when counting.
  constexpr int IT = SEL_CHUNK / (SEL_THREADS * 4);
  f32x4 x[IT];
  if (VEC4) {
#pragma unroll
    for (int i = 0; i < IT; ++i) {
      const int n = chunk0 * SEL_CHUNK + (i * SEL_THREADS + (int)threadIdx.x) * 4;
      x[i] = *reinterpret_cast<const f32x4 *>(a + min(n, A.srcN - 4));
    }
  }
  for (int i = threadIdx.x; i < SEL_BINS; i += SEL_THREADS) h[i] = 0u;
  uint32_t prefix, shift, dmask;
  if (PASS == 1) {
    uint32_t d0, k1;
    find_digit<(1 << SEL_BITS0)>(gh, c, tmp, d0, k1);
    if (chunk0 == 0 && threadIdx.x == 0) { st[0] = d0; st[1] = k1; st[6] = c; }
    prefix = d0;
    shift = SEL_BITS1 + SEL_BITS2;
    dmask = (1u << SEL_BITS1) - 1;
  } else {
    const uint32_t d0 = st[0], k1 = st[1];
    uint32_t d1, k2;
    find_digit<(1 << SEL_BITS1)>(gh + SEL_BINS, k1, tmp, d1, k2);
    if (chunk0 == 0 && threadIdx.x == 0) { st[2] = d1; st[3] = k2; }
    prefix = (d0 << SEL_BITS1) | d1;
    shift = SEL_BITS2;
    dmask = (1u << SEL_BITS2) - 1;
  }
  const uint32_t dshift = (PASS == 1) ? SEL_BITS2 : 0;
  // (the barriers inside find_digit have published the zeroed histogram)
  for (int cc = 0; cc < A.hist_cpw; ++cc) {
    const int n0 = (chunk0 + cc) * SEL_CHUNK;
    const int n1 = min(min(n0 + SEL_CHUNK, A.srcN), nb);
    if (n0 >= n1) break;
    if (VEC4) {
      if (cc > 0) {
#pragma unroll
        for (int i = 0; i < IT; ++i) {
          const int n = n0 + (i * SEL_THREADS + (int)threadIdx.x) * 4;
          x[i] = *reinterpret_cast<const f32x4 *>(a + min(n, A.srcN - 4));
        }
      }
#pragma unroll
      for (int i = 0; i < IT; ++i) {
        const int n = n0 + (i * SEL_THREADS + (int)threadIdx.x) * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t key = key_of(x[i][e]);
          if (n + e < n1 && (key >> shift) == prefix) atomicAdd(&h[(key >> dshift) & dmask], 1u);
        }
      }
    } else {
      for (int n = n0 + threadIdx.x; n < n1; n += SEL_THREADS) {
        const uint32_t key = key_of(a[n]);
        if ((key >> shift) == prefix) atomicAdd(&h[(key >> dshift) & dmask], 1u);
      }
    }
  }
  __syncthreads();
  uint32_t *go = A.hist + ((size_t)row * 3 + PASS) * SEL_BINS;
  flush_hist<SEL_BINS>(go, h);
}

// ------------------------------------------------------ ordered compaction + head remap
// The chunk's scores are loaded coalesced into LDS, then every thread takes 32 consecutive
// tokens, so one block scan of (greater, equal) counts gives every token its rank in token
// order. The kept tokens of a chunk occupy one contiguous range of the output list: they are
// staged in LDS at their local rank and copied out with coalesced stores, once per target.
template <bool VEC4>
__global__ void __launch_bounds__(SEL_THREADS, 4) select_write_kernel(const SelectArgs A) {   // <= 128 VGPRs: 4 workgroups per CU
  constexpr int PER = SEL_CHUNK / SEL_THREADS;   // 32 tokens per thread
  constexpr int PITCH = PER + 1;                 // odd pitch: conflict-free per-thread rows
  __shared__ uint32_t tmp[16];
  __shared__ uint32_t buf[SEL_THREADS * PITCH];  // keys first, then the staged token ids
  const int row = blockIdx.y, chunk = blockIdx.x;
  const int bt = row / A.Hd, j = row % A.Hd;
  const int nb = src_len(A, bt);
  const uint32_t c = (uint32_t)min(A.kh[j], nb);
  const int t0 = A.targets.off[j], t1 = A.targets.off[j + 1];
  if (chunk == 0) {
    // tail padding and counts for every target head of this draft head
    for (int ti = t0; ti < t1; ++ti) {
      const int tgt = A.targets.tgt[ti];
      int32_t *dst = A.indices + ((size_t)bt * A.Hq + tgt) * A.k;
      for (uint32_t p = c + threadIdx.x; p < (uint32_t)A.k; p += SEL_THREADS) dst[p] = -1;
      if (A.counts && threadIdx.x == 0) A.counts[(size_t)bt * A.Hq + tgt] = (int32_t)c;
    }
  }
  if (c == 0 || t0 == t1) return;
  const int n0 = chunk * SEL_CHUNK;
  if (n0 >= nb) return;
  const uint32_t *st = A.state + (size_t)row * 8;
  const float *a = A.src + (size_t)row * A.srcN;

  uint32_t *cc = A.chunk_cnt + (size_t)row * A.nchunks * SEL_FLAG_PITCH;
  // Everything this workgroup needs from memory is asked for at once, before anything is used:
  // the chunk (coalesced, clamped addresses, unconditional), a first look at the counts the
  // earlier chunks publish (they are often there already), and, inside find_digit, the last
  // digit's histogram.
  constexpr int IT = SEL_CHUNK / (SEL_THREADS * 4);
  f32x4 x[IT];
  if (VEC4) {
#pragma unroll
    for (int i = 0; i < IT; ++i)
      x[i] = *reinterpret_cast<const f32x4 *>(a + min(n0 + (i * SEL_THREADS + (int)threadIdx.x) * 4, A.srcN - 4));
  }
  uint32_t early = 0;
  if ((int)threadIdx.x < chunk)
    early = __hip_atomic_load(&cc[threadIdx.x * SEL_FLAG_PITCH], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

  // threshold key and tie quota of the row
  uint32_t d2, r;
  find_digit<(1 << SEL_BITS2)>(A.hist + ((size_t)row * 3 + 2) * SEL_BINS, st[3], tmp, d2, r);
  const uint32_t T = (st[0] << (SEL_BITS1 + SEL_BITS2)) | (st[2] << SEL_BITS2) | d2;

  // token n0 + i lands at buf[(i / PER) * PITCH + i % PER]
  if (VEC4) {
#pragma unroll
    for (int i = 0; i < IT; ++i) {
      const int t = (i * SEL_THREADS + (int)threadIdx.x) * 4;
#pragma unroll
      for (int e = 0; e < 4; ++e) buf[((t + e) / PER) * PITCH + (t + e) % PER] = key_of(x[i][e]);   // srcN % 4 == 0
    }
  } else {
    for (int i = threadIdx.x; i < SEL_CHUNK; i += SEL_THREADS)
      buf[(i / PER) * PITCH + i % PER] = (n0 + i < nb) ? key_of(a[n0 + i]) : 0u;
  }
  __syncthreads();

  const int base_n = n0 + threadIdx.x * PER;
  uint32_t keys[PER];
  uint32_t cg = 0, ce = 0;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    keys[i] = buf[threadIdx.x * PITCH + i];
    const bool in = base_n + i < nb;        // tokens past the valid length never count
    cg += (in && keys[i] > T) ? 1u : 0u;
    ce += (in && keys[i] == T) ? 1u : 0u;
  }
  uint32_t total;
  const uint32_t excl = block_excl_scan(cg | (ce << 16), tmp, total);   // barriers: buf is free
  const uint32_t chunk_gt = total & 0xffffu, chunk_eq = total >> 16;

  // keys greater / equal in the chunks before this one
  uint32_t pre = 0, pre_eq = 0;
  {
    // Every chunk publishes its own counts in one word (flag | equal << 14 | greater) with a
    // device-scope atomic store and reads the words of the chunks before it, one per thread.
    // The payload travels inside the flag, so no fence is involved. A chunk whose word does
    // not show up within the poll limit is simply recounted from the scores by this workgroup,
    // so the wait is bounded and no workgroup depends on another one being scheduled.
    uint32_t *miss = reinterpret_cast<uint32_t *>(buf);   // list of chunks to recount
    if (threadIdx.x == 0) {
      __hip_atomic_store(&cc[chunk * SEL_FLAG_PITCH], 0x80000000u | (chunk_eq << 14) | chunk_gt, __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
      tmp[8] = 0;                                          // number of entries in miss
    }
    __syncthreads();
    uint32_t g = 0, e = 0;
    for (int ch = threadIdx.x; ch < chunk; ch += SEL_THREADS) {
      uint32_t f = early;                                  // the first look, taken at the start
      if (ch != (int)threadIdx.x || !(f >> 31))
        f = __hip_atomic_load(&cc[ch * SEL_FLAG_PITCH], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      for (int spin = 0; !(f >> 31) && spin < A.spin_limit; ++spin) {
        __builtin_amdgcn_s_sleep(8);
        f = __hip_atomic_load(&cc[ch * SEL_FLAG_PITCH], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      if (f >> 31) {
        g += f & 0x3fffu;
        e += (f >> 14) & 0x3fffu;
      } else {
        const uint32_t slot = atomicAdd(&tmp[8], 1u);
        if (slot < (uint32_t)(SEL_THREADS * PITCH)) {
          miss[slot] = (uint32_t)ch;
        } else {   // list full (only with thousands of chunks per row): this thread recounts alone
          for (int i = 0; i < SEL_CHUNK; ++i) {
            const uint32_t key = key_of(a[ch * SEL_CHUNK + i]);
            g += key > T ? 1u : 0u;
            e += key == T ? 1u : 0u;
          }
        }
      }
    }
    __syncthreads();
    const uint32_t nmiss = min(tmp[8], (uint32_t)(SEL_THREADS * PITCH));
    for (uint32_t mi = 0; mi < nmiss; ++mi) {
      // recount chunk miss[mi] (it lies wholly below nb: it precedes this chunk)
      const int m0 = (int)miss[mi] * SEL_CHUNK;
      uint32_t packed = 0;
      for (int i = threadIdx.x; i < SEL_CHUNK; i += SEL_THREADS) {
        const uint32_t key = key_of(a[m0 + i]);
        packed += (key > T ? 1u : 0u) + (key == T ? 0x10000u : 0u);
      }
      // one thread per wave carries the wave's sum into the running totals
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) packed += __shfl_xor(packed, off, 64);
      if ((threadIdx.x & 63) == 0) {
        g += packed & 0xffffu;
        e += packed >> 16;
      }
    }
    // block totals of both counts (a row holds fewer than 2^31 tokens: two 32-bit sums)
    const uint32_t wg = wave_incl_scan(g), we = wave_incl_scan(e);
    if ((threadIdx.x & 63) == 63) {
      tmp[2 * (threadIdx.x >> 6)] = wg;
      tmp[2 * (threadIdx.x >> 6) + 1] = we;
    }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < SEL_THREADS / 64; ++w) {
      pre += tmp[2 * w];
      pre_eq += tmp[2 * w + 1];
    }
    __syncthreads();
  }
  uint32_t g = pre + (excl & 0xffffu), q = pre_eq + (excl >> 16);
  // output range of this chunk: [first, last)
  const uint32_t first = pre + min(pre_eq, r);
  const uint32_t last = min((pre + chunk_gt) + min(pre_eq + chunk_eq, r), c);
  int32_t *staged = reinterpret_cast<int32_t *>(buf);
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const bool in = base_n + i < nb;
    const bool is_gt = in && keys[i] > T;
    const bool is_eq = in && keys[i] == T;
    if (is_gt || (is_eq && q < r)) {
      const uint32_t pos = g + min(q, r);
      // always inside [first, last) for a consistent threshold; the test keeps a bad state
      // inside the staging buffer
      if (pos >= first && pos - first < (uint32_t)SEL_CHUNK) staged[pos - first] = base_n + i;
    }
    g += is_gt ? 1u : 0u;
    q += is_eq ? 1u : 0u;
  }
  __syncthreads();
  if (last > first) {
    const uint32_t cnt = min(last - first, (uint32_t)SEL_CHUNK);
    for (int ti = t0; ti < t1; ++ti) {
      int32_t *dst = A.indices + ((size_t)bt * A.Hq + A.targets.tgt[ti]) * A.k + first;
      for (uint32_t p = threadIdx.x; p < cnt; p += SEL_THREADS) dst[p] = staged[p];
    }
  }
}

// ------------------------------------------------------- ranking keys that sit in LDS
constexpr int SMALL_THREADS = 1024;
__device__ __forceinline__ int small_slot(int n) { return n + (n >> 5); }   // pad 1 word per 32: conflict-free strided reads

// The c-th largest of keys[small_slot(0 .. m)) and the number r of keys equal to it that are
// kept. On entry h holds the histogram of the first digit of those m keys; h and tmp
// (THREADS/64 + 2 words) are scratch. Requires 1 <= c <= m.
template <int THREADS>
__device__ __forceinline__ void lds_threshold(const uint32_t *keys, int m, uint32_t *h, uint32_t *tmp, uint32_t c,
                                              uint32_t &T, uint32_t &r) {
  const int tid = threadIdx.x;
  uint32_t d0, k1, d1, k2, d2;
  find_digit<(1 << SEL_BITS0), THREADS>(h, c, tmp, d0, k1);
  for (int i = tid; i < SEL_BINS; i += THREADS) h[i] = 0u;
  __syncthreads();
  for (int n = tid; n < m; n += THREADS) {
    const uint32_t key = keys[small_slot(n)];
    if ((key >> (SEL_BITS1 + SEL_BITS2)) == d0) atomicAdd(&h[(key >> SEL_BITS2) & ((1u << SEL_BITS1) - 1)], 1u);
  }
  __syncthreads();
  find_digit<(1 << SEL_BITS1), THREADS>(h, k1, tmp, d1, k2);
  for (int i = tid; i < SEL_BINS; i += THREADS) h[i] = 0u;
  __syncthreads();
  const uint32_t pre01 = (d0 << SEL_BITS1) | d1;
  for (int n = tid; n < m; n += THREADS) {
    const uint32_t key = keys[small_slot(n)];
    if ((key >> SEL_BITS2) == pre01) atomicAdd(&h[key & ((1u << SEL_BITS2) - 1)], 1u);
  }
  __syncthreads();
  find_digit<(1 << SEL_BITS2), THREADS>(h, k2, tmp, d2, r);
  T = (pre01 << SEL_BITS2) | d2;
}

// Ordered compaction of the same keys: every thread owns a run of at most MAXPER consecutive
// entries (m <= MAXPER * THREADS), read once into registers; entry n is kept iff key > T, or
// key == T and fewer than r equal keys precede it, and emit(pos, n) is called with its position
// in the output list, pos = (#greater before n) + min(#equal before n, r).
template <int THREADS, int MAXPER, class Emit>
__device__ __forceinline__ void lds_compact_run(const uint32_t *keys, int m, uint32_t T, uint32_t r, uint32_t c,
                                                uint32_t *tmp, Emit emit) {
  const int tid = threadIdx.x;
  const int per = (m + THREADS - 1) / THREADS;
  const int nlo = min(tid * per, m), nhi = min(nlo + per, m);
  uint32_t kk[MAXPER];
  uint32_t cg = 0, ce = 0;
#pragma unroll
  for (int i = 0; i < MAXPER; ++i) {
    const int n = nlo + i;
    kk[i] = keys[small_slot(min(n, m - 1))];
    cg += (n < nhi && kk[i] > T) ? 1u : 0u;
    ce += (n < nhi && kk[i] == T) ? 1u : 0u;
  }
  uint32_t total;
  const uint32_t excl = block_excl_scan<THREADS>(cg | (ce << 16), tmp, total);   // m <= 32768: both sums fit 16 bits
  uint32_t g = excl & 0xffffu, q = excl >> 16;
#pragma unroll
  for (int i = 0; i < MAXPER; ++i) {
    const int n = nlo + i;
    const bool is_gt = n < nhi && kk[i] > T, is_eq = n < nhi && kk[i] == T;
    if (is_gt || (is_eq && q < r)) {
      const uint32_t pos = g + min(q, r);
      if (pos < c) emit(pos, n);   // always true for a consistent threshold; keeps a bad state in bounds
    }
    g += is_gt ? 1u : 0u;
    q += is_eq ? 1u : 0u;
  }
}

// the same with the run length (a uniform value) rounded up to 4, 8, 16 or MAXPER
template <int THREADS, int MAXPER, class Emit>
__device__ __forceinline__ void lds_compact(const uint32_t *keys, int m, uint32_t T, uint32_t r, uint32_t c,
                                            uint32_t *tmp, Emit emit) {
  const int per = (m + THREADS - 1) / THREADS;
  if (MAXPER > 4 && per <= 4) lds_compact_run<THREADS, 4>(keys, m, T, r, c, tmp, emit);
  else if (MAXPER > 8 && per <= 8) lds_compact_run<THREADS, 8>(keys, m, T, r, c, tmp, emit);
  else if (MAXPER > 16 && per <= 16) lds_compact_run<THREADS, 16>(keys, m, T, r, c, tmp, emit);
  else lds_compact_run<THREADS, MAXPER>(keys, m, T, r, c, tmp, emit);
}

// tail padding (-1 from position c on) and counts for every target head of draft head j
template <int THREADS>
__device__ __forceinline__ void write_tail(const SelectArgs &A, int bt, int j, uint32_t c) {
  for (int ti = A.targets.off[j]; ti < A.targets.off[j + 1]; ++ti) {
    const int tgt = A.targets.tgt[ti];
    int32_t *dst = A.indices + ((size_t)bt * A.Hq + tgt) * A.k;
    for (uint32_t p = c + threadIdx.x; p < (uint32_t)A.k; p += THREADS) dst[p] = -1;
    if (A.counts && threadIdx.x == 0) A.counts[(size_t)bt * A.Hq + tgt] = (int32_t)c;
  }
}

// ------------------------------------------------- whole selection in one workgroup per row
// For rows of up to SEL_SMALL_N tokens the keys of a row fit in LDS (128 KB of the 160 KB), so
// one 1024-thread workgroup per (batch, draft head) does everything in a single launch:
// aggregate (same fp32 order), three digit histograms over the LDS-resident keys, ordered
// compaction and the copies to the target heads. No global histograms, nothing to clear.
// FROM_SRC: the scores to rank are already there (A.src, row pitch A.srcN: the block sums of
// block-granular selection) and only have to be loaded.
template <bool VEC4, bool FROM_SRC>
__global__ void __launch_bounds__(SMALL_THREADS) select_small_kernel(const SelectArgs A) {
  __shared__ uint32_t keys[SEL_SMALL_N + SEL_SMALL_N / 32];
  __shared__ uint32_t h[SEL_BINS];
  __shared__ uint32_t tmp[SMALL_THREADS / 64 + 2];
  const int row = blockIdx.x;
  const int bt = row / A.Hd, j = row % A.Hd;
  const int nb = FROM_SRC ? src_len(A, bt) : row_len(A, bt);
  const uint32_t c = (uint32_t)min(A.kh[j], nb);
  const int t0 = A.targets.off[j], t1 = A.targets.off[j + 1];
  const int tid = threadIdx.x;
  write_tail<SMALL_THREADS>(A, bt, j, c);
  const bool want_agg = !FROM_SRC && A.agg != nullptr;
  if ((c == 0 || t0 == t1) && !want_agg) return;

  for (int i = tid; i < SEL_BINS; i += SMALL_THREADS) h[i] = 0u;
  __syncthreads();
  const AggRow R = agg_row(A, row);
  float *out = want_agg ? A.agg + (size_t)row * A.N : nullptr;
  if (FROM_SRC) {
    const float *src = A.src + (size_t)row * A.srcN;
    for (int n = tid; n < nb; n += SMALL_THREADS) {
      const uint32_t key = key_of(src[n]);
      keys[small_slot(n)] = key;
      atomicAdd(&h[key >> (32 - SEL_BITS0)], 1u);
    }
  } else if (VEC4) {
    for (int n = tid * 4; n < A.N; n += SMALL_THREADS * 4) {
      const f32x4 acc = agg_quad(R, n);
      f32x4 o = acc;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t key = key_of(acc[e]);
        keys[small_slot(n + e)] = key;
        if (n + e < nb) atomicAdd(&h[key >> (32 - SEL_BITS0)], 1u);
        else o[e] = 0.f;
      }
      if (want_agg) *reinterpret_cast<f32x4 *>(out + n) = o;
    }
  } else {
    for (int n = tid; n < A.N; n += SMALL_THREADS) {
      const float acc = agg_one(R, n);
      if (want_agg) out[n] = n < nb ? acc : 0.f;
      const uint32_t key = key_of(acc);
      keys[small_slot(n)] = key;
      if (n < nb) atomicAdd(&h[key >> (32 - SEL_BITS0)], 1u);
    }
  }
  __syncthreads();
  if (c == 0 || t0 == t1) return;

  uint32_t T, r;
  lds_threshold<SMALL_THREADS>(keys, nb, h, tmp, c, T, r);
  lds_compact<SMALL_THREADS, SEL_SMALL_N / SMALL_THREADS>(keys, nb, T, r, c, tmp, [&](uint32_t pos, int n) {
    for (int ti = t0; ti < t1; ++ti) A.indices[((size_t)bt * A.Hq + A.targets.tgt[ti]) * A.k + pos] = n;
  });
}

// ------------------------------------------------------- long rows: the whole selection in one launch
// A row is cut into parts of P = PER * 1024 tokens; one 1024-thread workgroup per (part, row)
// aggregates its part once (same fp32 order), keeps the keys in LDS and never reads a score or an
// aggregate again. The three digit histograms are row-wide quantities, so at each level every part
// publishes its own histogram and adds up the histograms of all parts of its row; the digit search
// is then done redundantly by every part. While adding, a part also keeps the sum over the parts
// BEFORE it, which after the digit search gives the number of keys greater than / equal to the
// threshold in earlier parts, i.e. where its own kept tokens start in the output list: no second
// exchange is needed for the compaction.
//
// Exchange protocol (per level). The published area is zeroed by a small kernel launched before
// this one. Thread t of a part publishes the counts of bins 2t and 2t+1 in one 64-bit word whose
// top bit says "written" (a device-scope store of 8 aligned bytes: the word arrives whole), and
// reads the words of the other parts for the same two bins until their top bits are set: the
// payload is its own flag, so one memory round trip per level is all the parts wait for each
// other. The wait is bounded: after the poll limit the workgroup decides, part by part, which
// histograms have arrived completely and recomputes the others from the scores itself, so every
// workgroup exits whatever the others do (a row's parts have neighbouring workgroup ids and start
// together, so in practice the words are there on the first or second look).
constexpr int FUSED_THREADS = 1024;
constexpr unsigned long long FUSED_VALID = 1ull << 63;
// LDS slot of a part's local token l: four pad words after every 32 tokens. Quads (l % 4 == 0)
// stay contiguous and 16-byte aligned, so every pass moves four keys per LDS instruction, and both
// ways of walking the part are free of bank conflicts: consecutive lanes on consecutive quads, and
// lane t on the quads of its own run of 32 tokens (36 words apart from its neighbour's).
__device__ __forceinline__ int fused_slot(int l) { return l + ((l >> 5) << 2); }

// sum over the block of two values per thread; red needs 2 * FUSED_THREADS / 64 words
__device__ __forceinline__ void block_sum2(uint32_t a, uint32_t b, uint32_t *red, uint32_t &sa, uint32_t &sb) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    a += (uint32_t)__shfl_xor((int)a, off, 64);
    b += (uint32_t)__shfl_xor((int)b, off, 64);
  }
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) {
    red[2 * wave] = a;
    red[2 * wave + 1] = b;
  }
  __syncthreads();
  sa = sb = 0;
#pragma unroll
  for (int w = 0; w < FUSED_THREADS / 64; ++w) {
    sa += red[2 * w];
    sb += red[2 * w + 1];
  }
  __syncthreads();
}

// bin of `key` at `level` under the prefix fixed so far, or -1 when the key is no candidate
__device__ __forceinline__ int fused_bin(uint32_t key, int level, uint32_t d0, uint32_t pre01) {
  if (level == 0) return (int)(key >> (32 - SEL_BITS0));
  if (level == 1) return (key >> (SEL_BITS1 + SEL_BITS2)) == d0 ? (int)((key >> SEL_BITS2) & ((1u << SEL_BITS1) - 1)) : -1;
  return (key >> SEL_BITS2) == pre01 ? (int)(key & ((1u << SEL_BITS2) - 1)) : -1;
}

template <bool VEC4, int PER>
__global__ void __launch_bounds__(FUSED_THREADS) select_fused_kernel(const SelectArgs A) {
  constexpr int T = FUSED_THREADS;
  constexpr int P = PER * T;                       // tokens per part
  __shared__ __attribute__((aligned(16))) uint32_t keys[P + P / 8];   // later: the staged token ids of the part
  __shared__ uint32_t h[SEL_BINS];
  __shared__ uint32_t tmp[T / 64 + 2];
  __shared__ uint32_t red[2 * T / 64];
  __shared__ uint32_t lds_flag[2];                 // [0]: some thread ran out of polls, [1]: scratch of the slow path
  const int row = blockIdx.y, part = blockIdx.x;
  const int tid = threadIdx.x;
  const int bt = row / A.Hd, j = row % A.Hd;
  const int nb = row_len(A, bt);
  const uint32_t c = (uint32_t)min(A.kh[j], nb);
  const int t0 = A.targets.off[j], t1 = A.targets.off[j + 1];
  if (part == 0) write_tail<T>(A, bt, j, c);
  const bool want_agg = A.agg != nullptr;
  const bool ranked = c > 0 && t0 != t1;           // the same for every part of the row
  if (!ranked && !want_agg) return;
  const int n0 = part * P;
  const int nend = min(n0 + P, A.N);
  const int m = max(0, min(nend, nb) - n0);        // ranked tokens of this part
  const int Qv = (nb + P - 1) / P;                 // parts of the row that hold ranked tokens
  if (m == 0 && !want_agg) return;                 // the other parts do not expect this one

  for (int i = tid; i < SEL_BINS; i += T) h[i] = 0u;
  if (tid == 0) lds_flag[0] = 0u;
  __syncthreads();
  const AggRow R = agg_row(A, row);
  float *out = want_agg ? A.agg + (size_t)row * A.N : nullptr;
  if (VEC4) {
    // one quad per thread and step (more in flight did not stream faster: 16 waves per CU keep
    // enough loads outstanding, and the registers are better spent elsewhere)
#pragma unroll 1
    for (int i = 0; i < PER / 4; ++i) {
      const int l = (i * T + tid) * 4;             // local token index
      if (l < m) {
        const f32x4 acc = agg_quad(R, n0 + l);     // N % 4 == 0: the quad lies inside the row
        f32x4 o = acc;
        u32x4 kv;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          kv[e] = key_of(acc[e]);
          if (l + e < m) atomicAdd(&h[kv[e] >> (32 - SEL_BITS0)], 1u);
          else o[e] = 0.f;                         // the aggregate is 0 past the valid length
        }
        *reinterpret_cast<u32x4 *>(&keys[fused_slot(l)]) = kv;
        if (want_agg) *reinterpret_cast<f32x4 *>(out + n0 + l) = o;
      } else if (want_agg && n0 + l < nend) {
        *reinterpret_cast<f32x4 *>(out + n0 + l) = f32x4{0.f, 0.f, 0.f, 0.f};
      }
    }
  } else {
    for (int l = tid; l < nend - n0; l += T) {
      float acc = 0.f;
      if (l < m) {
        acc = agg_one(R, n0 + l);
        const uint32_t key = key_of(acc);
        keys[fused_slot(l)] = key;
        atomicAdd(&h[key >> (32 - SEL_BITS0)], 1u);
      }
      if (want_agg) out[n0 + l] = acc;
    }
  }
  __syncthreads();
  if (!ranked || m == 0) return;

  // Three levels, one loop (the code below exists once): build this part's histogram of the level
  // (level 0 was built while streaming), exchange it, find the row-wide digit.
  uint32_t pre_gt = 0, pre_eq = 0;       // keys of earlier parts greater than / equal to the threshold
  uint32_t d0 = 0, pre01 = 0, krem = c, d2 = 0;
  uint32_t cand = 0;                     // bit 4i + e: token e of this thread's quad tid + i * T shares the first digit
#pragma unroll 1
  for (int level = 0; level < 3; ++level) {
    if (level > 0) {
      for (int i = tid; i < SEL_BINS; i += T) h[i] = 0u;
      __syncthreads();
      if (level == 1) {
        // all of the thread's PER keys (quads tid, tid + T, ...), four quads in flight at a time;
        // cand remembers the candidates so that the last level only looks at those again
#pragma unroll 1
        for (int i0 = 0; i0 < PER / 4; i0 += 2) {
          u32x4 kq[2];
#pragma unroll
          for (int i = 0; i < 2; ++i)
            kq[i] = *reinterpret_cast<const u32x4 *>(&keys[fused_slot(min((tid + (i0 + i) * T) * 4, P - 4))]);
#pragma unroll
          for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int bin = fused_bin(kq[i][e], 1, d0, 0u);
              if ((tid + (i0 + i) * T) * 4 + e < m && bin >= 0) {
                atomicAdd(&h[bin], 1u);
                cand |= 1u << (4 * (i0 + i) + e);
              }
            }
        }
      } else {
        for (uint32_t rest = cand; rest; rest &= rest - 1) {
          const int bit = __builtin_ctz(rest);
          const int bin = fused_bin(keys[fused_slot((tid + (bit >> 2) * T) * 4 + (bit & 3))], 2, d0, pre01);
          if (bin >= 0) atomicAdd(&h[bin], 1u);
        }
      }
      __syncthreads();
    }
    const uint32_t own0 = h[2 * tid], own1 = h[2 * tid + 1];
    uint32_t all0 = own0, all1 = own1, bef0 = 0, bef1 = 0;
    if (Qv > 1) {
      unsigned long long *pub = A.pub + (size_t)(row * 3 + level) * A.parts * T;      // [parts][T]
      __hip_atomic_store(&pub[(size_t)part * T + tid], FUSED_VALID | own0 | ((unsigned long long)own1 << 32),
                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      bool complete = false;
      for (int spin = 0; !complete && spin <= A.fused_spin_limit; ++spin) {
        if (spin) __builtin_amdgcn_s_sleep(4);
        all0 = own0; all1 = own1; bef0 = bef1 = 0;
        complete = true;
        // loads are unconditional so that they overlap (this part's own word contributes nothing)
#pragma unroll 4
        for (int q = 0; q < Qv; ++q) {
          const unsigned long long w = __hip_atomic_load(&pub[(size_t)q * T + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          const bool use = q != part;
          if (use && !(w & FUSED_VALID)) complete = false;
          const uint32_t w0 = use ? ((uint32_t)w & 0xffffffu) : 0u, w1 = use ? ((uint32_t)(w >> 32) & 0xffffffu) : 0u;
          all0 += w0;
          all1 += w1;
          bef0 += q < part ? w0 : 0u;
          bef1 += q < part ? w1 : 0u;
        }
      }
      if (!complete) lds_flag[0] = 1u;
      __syncthreads();
      if (lds_flag[0]) {
        // Some thread ran out of polls (the flag stays set: later levels come this way too). Part by
        // part, the histogram is used if all of its 1024 words have arrived and is recomputed from
        // the scores otherwise: the same decision in every thread.
        all0 = own0; all1 = own1; bef0 = bef1 = 0;
#pragma unroll 1
        for (int q = 0; q < Qv; ++q) {
          if (q == part) continue;
          if (tid == 0) lds_flag[1] = 1u;
          __syncthreads();
          const unsigned long long w = __hip_atomic_load(&pub[(size_t)q * T + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          if (!(w & FUSED_VALID)) lds_flag[1] = 0u;
          __syncthreads();
          uint32_t w0 = (uint32_t)w & 0xffffffu, w1 = (uint32_t)(w >> 32) & 0xffffffu;
          if (lds_flag[1] == 0u) {        // uniform
            for (int i = tid; i < SEL_BINS; i += T) h[i] = 0u;
            __syncthreads();
            const int q0 = q * P, q1 = min(q0 + P, nb);
            if (VEC4) {
#pragma unroll 1
              for (int n = q0 + tid * 4; n < q1; n += T * 4) {
                const f32x4 acc = agg_quad(R, n);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  const int bin = fused_bin(key_of(acc[e]), level, d0, pre01);
                  if (n + e < q1 && bin >= 0) atomicAdd(&h[bin], 1u);
                }
              }
            } else {
#pragma unroll 1
              for (int n = q0 + tid; n < q1; n += T) {
                const int bin = fused_bin(key_of(agg_one(R, n)), level, d0, pre01);
                if (bin >= 0) atomicAdd(&h[bin], 1u);
              }
            }
            __syncthreads();
            w0 = h[2 * tid];
            w1 = h[2 * tid + 1];
          }
          __syncthreads();                // h and the flag are free again
          all0 += w0;
          all1 += w1;
          bef0 += q < part ? w0 : 0u;
          bef1 += q < part ? w1 : 0u;
        }
      }
    }
    __syncthreads();
    h[2 * tid] = all0;
    h[2 * tid + 1] = all1;
    __syncthreads();
    uint32_t digit, knext;
    find_digit<SEL_BINS, T>(h, krem, tmp, digit, knext);
    // keys of earlier parts in higher bins are greater than the threshold whatever follows; those
    // in the digit's own bin are the "equal" ones of the last level
    const uint32_t b0 = 2 * tid, b1 = 2 * tid + 1;
    const uint32_t above = (b0 > digit ? bef0 : 0u) + (b1 > digit ? bef1 : 0u);
    const uint32_t at = (b0 == digit ? bef0 : 0u) + (b1 == digit ? bef1 : 0u);
    uint32_t sa, sb;
    block_sum2(above, at, red, sa, sb);
    pre_gt += sa;
    pre_eq = sb;
    if (level == 0) d0 = digit;
    else if (level == 1) pre01 = (d0 << SEL_BITS1) | digit;
    else d2 = digit;
    krem = knext;
  }
  const uint32_t r = krem;               // keys equal to the threshold that are kept
  const uint32_t Tk = (pre01 << SEL_BITS2) | d2;

  // ordered compaction of the part: thread tid owns the PER consecutive tokens from tid * PER on;
  // what it needs to remember of them are two bits per token (greater / equal)
  static_assert(PER <= 32, "one mask bit per owned token");
  uint32_t gt_mask = 0, eq_mask = 0;
#pragma unroll 1
  for (int i0 = 0; i0 < PER; i0 += 8) {
    u32x4 kq[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) kq[i] = *reinterpret_cast<const u32x4 *>(&keys[fused_slot(tid * PER + i0 + 4 * i)]);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const bool in = tid * PER + i0 + i < m;
      const uint32_t key = kq[i >> 2][i & 3];
      gt_mask |= (in && key > Tk) ? 1u << (i0 + i) : 0u;
      eq_mask |= (in && key == Tk) ? 1u << (i0 + i) : 0u;
    }
  }
  const uint32_t cg = __builtin_popcount(gt_mask), ce = __builtin_popcount(eq_mask);
  uint32_t total;
  const uint32_t excl = block_excl_scan<T>(cg | (ce << 16), tmp, total);   // its barriers free the key buffer
  const uint32_t part_gt = total & 0xffffu, part_eq = total >> 16;
  const uint32_t first = pre_gt + min(pre_eq, r);
  const uint32_t last = min((pre_gt + part_gt) + min(pre_eq + part_eq, r), c);
  uint32_t g = pre_gt + (excl & 0xffffu), q = pre_eq + (excl >> 16);
  int32_t *staged = reinterpret_cast<int32_t *>(keys);
  for (uint32_t rest = gt_mask | eq_mask; rest; rest &= rest - 1) {
    const int i = __builtin_ctz(rest);
    const bool is_gt = (gt_mask >> i) & 1u;
    if (is_gt || q < r) {
      const uint32_t pos = g + min(q, r);
      // always inside [first, last) for a consistent threshold; the test keeps a bad state in bounds
      if (pos >= first && pos - first < (uint32_t)P) staged[pos - first] = n0 + tid * PER + i;
    }
    g += is_gt ? 1u : 0u;
    q += is_gt ? 0u : 1u;
  }
  __syncthreads();
  if (last > first) {
    const uint32_t cnt = min(last - first, (uint32_t)P);
    for (int ti = t0; ti < t1; ++ti) {
      int32_t *dst = A.indices + ((size_t)bt * A.Hq + A.targets.tgt[ti]) * A.k + first;
      for (uint32_t p = tid; p < cnt; p += T) dst[p] = staged[p];
    }
  }
}

// --------------------------------- many long rows of ready-made scores: one workgroup per row
// A call with one score per token (Tq = 1: the per-query-row masks of prefill rank every row of a
// block's scores on its own; a draft layer's summed weights) and far more rows than CUs. Cutting
// such rows into parts that wait for each other leaves every CU idle during the exchanges; here a
// row belongs to ONE workgroup, which keeps nothing but a digit histogram in LDS and reads the
// row once per digit level and once more to compact it. The re-reads come out of the caches (a
// row is 256-512 KB; what the resident workgroups hold together fits the last-level cache), and
// several small workgroups per CU are in different phases at any time, so the digit searches and
// scans of one hide behind the streaming of the others. Nothing is exchanged, cleared or stored
// besides the lists. bf16 scores have keys whose low 16 bits are all equal, so their third level
// is known without a pass.
template <bool BF16>
__device__ __forceinline__ uint32_t rowpass_key(const u32x4 &w, int e) {
  if (BF16) {
    const uint32_t pair = w[e >> 1];
    return key_of_bits((e & 1) ? (pair & 0xffff0000u) : (pair << 16));
  }
  return key_of_bits(w[e & 3]);
}

template <int THREADS, bool BF16>
__global__ void __launch_bounds__(THREADS) select_rowpass_kernel(const SelectArgs A) {
  constexpr int VPT = BF16 ? 8 : 4;       // tokens per 16-byte word
  constexpr int UNR = 4;                  // words in flight per thread
  constexpr int RUN = UNR * VPT;          // consecutive tokens a thread owns per compaction step
  static_assert(RUN <= 32 && THREADS * RUN < 65536, "mask bits per thread; packed block scan");
  __shared__ uint32_t h[SEL_BINS];
  __shared__ uint32_t tmp[THREADS / 64 + 2];
  const int row = blockIdx.x, tid = threadIdx.x;
  const int bt = row / A.Hd, j = row % A.Hd;
  const int nb = row_len(A, bt);
  const uint32_t c = (uint32_t)min(A.kh[j], nb);
  const int t0 = A.targets.off[j], t1 = A.targets.off[j + 1];
  write_tail<THREADS>(A, bt, j, c);
  if (c == 0 || t0 == t1) return;
  // N % VPT == 0 and a 16-byte aligned base (the host's condition for this path): whole words
  const u32x4 *src = reinterpret_cast<const u32x4 *>(
      static_cast<const unsigned char *>(A.scores) + (size_t)row * A.N * (BF16 ? 2 : 4));
  const int nv = (nb + VPT - 1) / VPT;    // words that hold ranked tokens

  // bf16 rows: the second digit has only 32 values that occur (5 bits of the score, the rest
  // follows the sign), so its histogram can be built in the FIRST pass for a window of first
  // digits, if the window is put where the first digit will turn out to be: a 1/16 sample of the
  // row (128-byte runs) says where. If the first digit falls outside the window the second pass
  // is made as for any row; the result never depends on the sample.
  constexpr int WIN = 8;
  constexpr int STAGE = THREADS * 8;      // list entries staged per round of the compaction
  __shared__ int32_t staged[STAGE];
  __shared__ uint32_t hw[BF16 ? WIN * 32 : 1];
  uint32_t wlo = 0;                       // first digit the window starts at
  bool win = false;
  if (BF16 && nv >= 4096) {
    win = true;
    for (int i = tid; i < SEL_BINS; i += THREADS) h[i] = 0u;
    __syncthreads();
    const int runs = (nv + 127) / 128;    // sampled run i: the 8 words from 128 i on
    uint32_t mine = 0;
    for (int s0 = tid; s0 < runs * 8; s0 += THREADS) {
      const int wi = (s0 >> 3) * 128 + (s0 & 7);
      if (wi < nv) {
        const u32x4 w = src[wi];
#pragma unroll
        for (int e = 0; e < VPT; ++e)
          if (wi * VPT + e < nb) {
            atomicAdd(&h[rowpass_key<BF16>(w, e) >> (32 - SEL_BITS0)], 1u);
            ++mine;
          }
      }
    }
    __syncthreads();
    uint32_t ns;
    block_excl_scan<THREADS>(mine, tmp, ns);
    const uint32_t want = (uint32_t)min((uint64_t)ns, max((uint64_t)1, (uint64_t)c * ns / (uint32_t)nb));
    uint32_t dest, unused;
    find_digit<SEL_BINS, THREADS>(h, want, tmp, dest, unused);
    wlo = dest >= WIN / 2 ? dest - WIN / 2 + 1 : 0u;
    for (int i = tid; i < WIN * 32; i += THREADS) hw[i] = 0u;
  }

  uint32_t d0 = 0, pre01 = 0, krem = c, d2 = 0;
#pragma unroll 1
  for (int level = 0; level < (BF16 ? 2 : 3); ++level) {
    for (int i = tid; i < SEL_BINS; i += THREADS) h[i] = 0u;
    __syncthreads();
    if (BF16 && level == 1 && win && d0 - wlo < (uint32_t)WIN) {
      // the window held the first digit: its 32 counts are the second digit's histogram
      const uint32_t low = (d0 >> (SEL_BITS0 - 1)) ? 0u : (1u << (SEL_BITS1 - 5)) - 1;   // the bits below follow the sign
      if (tid < 32) h[((uint32_t)tid << (SEL_BITS1 - 5)) | low] = hw[(d0 - wlo) * 32 + tid];
    } else {
#pragma unroll 1
      for (int i0 = tid; i0 < nv; i0 += THREADS * UNR) {
        u32x4 w[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) w[u] = src[min(i0 + u * THREADS, nv - 1)];
        if (BF16 && level == 0) {
          // The kernel is bound by its vector instructions (about 18 per token and pass in the
          // general form below), so the common case gets a form of its own: every word of the
          // wave inside the row and no sign bit among its scores (attention weights have none).
          // Then the first digit is 1024 + (the stored 16 bits >> 5) and the window's sub-bin
          // their low 5 bits: five instructions per token.
          uint32_t any = 0;
#pragma unroll
          for (int u = 0; u < UNR; ++u) any |= w[u][0] | w[u][1] | w[u][2] | w[u][3];
          const bool lane_ok = (i0 + (UNR - 1) * THREADS + 1) * VPT <= nb && (any & 0x80008000u) == 0u;
          if (__builtin_amdgcn_ballot_w64(!lane_ok) == 0) {
            const uint32_t wlo10 = wlo - (1u << (SEL_BITS0 - 1));    // modulo 2^32: the comparison below stays exact
            uint32_t *hpos = h + (1u << (SEL_BITS0 - 1));
#pragma unroll
            for (int u = 0; u < UNR; ++u)
#pragma unroll
              for (int e = 0; e < VPT; ++e) {
                const uint32_t pair = w[u][(e >> 1) & 3];
                const uint32_t r16 = (e & 1) ? pair >> 16 : pair & 0xffffu;
                const uint32_t b = r16 >> 5;
                atomicAdd(&hpos[b], 1u);
                const uint32_t wd = b - wlo10;
                if (win && wd < (uint32_t)WIN) atomicAdd(&hw[wd * 32 + (r16 & 31u)], 1u);
              }
            continue;
          }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
          const int wi = i0 + u * THREADS;
          const int valid = wi < nv ? nb - wi * VPT : 0;   // ranked tokens from this word on: >= VPT but at the row's end
#pragma unroll
          for (int e = 0; e < VPT; ++e) {
            const uint32_t key = rowpass_key<BF16>(w[u], e);
            const int bin = fused_bin(key, level, d0, pre01);
            if (e < valid && bin >= 0) {
              atomicAdd(&h[bin], 1u);
              if (BF16 && level == 0 && win && (uint32_t)bin - wlo < (uint32_t)WIN)
                atomicAdd(&hw[((uint32_t)bin - wlo) * 32 + ((key >> (32 - SEL_BITS0 - 5)) & 31u)], 1u);
            }
          }
        }
      }
    }
    __syncthreads();
    uint32_t digit, knext;
    find_digit<SEL_BINS, THREADS>(h, krem, tmp, digit, knext);
    if (level == 0) d0 = digit;
    else if (level == 1) pre01 = (d0 << SEL_BITS1) | digit;
    else d2 = digit;
    krem = knext;
  }
  // widened bf16: the 16 low key bits repeat the complement of the sign, so every key that shares
  // the first two digits is the same key
  if (BF16) d2 = (d0 >> (SEL_BITS0 - 1)) ? 0u : (1u << SEL_BITS2) - 1;
  const uint32_t r = krem;
  const uint32_t Tk = (pre01 << SEL_BITS2) | d2;

  // ordered compaction: per step, thread tid owns the RUN consecutive tokens from step + tid * RUN
  uint32_t gbase = 0, qbase = 0;          // keys greater than / equal to the threshold before this step
#pragma unroll 1
  for (int step = 0; step < nb; step += THREADS * RUN) {
    const int nlo = step + tid * RUN;
    u32x4 w[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) w[u] = src[min(nlo / VPT + u, nv - 1)];
    uint32_t gt_mask = 0, eq_mask = 0;
    // the common case again (see the first pass): a positive threshold, every run of the wave inside
    // the row, no sign bit: the stored 16 bits are compared with the threshold's
    bool plain = false;
    if (BF16 && (Tk >> 31)) {
      uint32_t any = 0;
#pragma unroll
      for (int u = 0; u < UNR; ++u) any |= w[u][0] | w[u][1] | w[u][2] | w[u][3];
      plain = __builtin_amdgcn_ballot_w64(!(nlo + RUN <= nb && (any & 0x80008000u) == 0u)) == 0;
    }
    if (plain) {
      const uint32_t T16 = (Tk >> 16) & 0x7fffu;
#pragma unroll
      for (int u = 0; u < UNR; ++u)
#pragma unroll
        for (int e = 0; e < VPT; ++e) {
          const uint32_t pair = w[u][(e >> 1) & 3];
          const uint32_t r16 = (e & 1) ? pair >> 16 : pair & 0xffffu;
          gt_mask |= (r16 > T16) ? 1u << (u * VPT + e) : 0u;
          eq_mask |= (r16 == T16) ? 1u << (u * VPT + e) : 0u;
        }
    } else {
#pragma unroll
      for (int u = 0; u < UNR; ++u)
#pragma unroll
        for (int e = 0; e < VPT; ++e) {
          const uint32_t key = rowpass_key<BF16>(w[u], e);
          gt_mask |= (key > Tk) ? 1u << (u * VPT + e) : 0u;
          eq_mask |= (key == Tk) ? 1u << (u * VPT + e) : 0u;
        }
    }
    if (!plain) {   // tokens past the row's valid length (only in its last run) are dropped from both masks
      const int left = nb - nlo;
      const uint32_t in = left >= RUN ? 0xffffffffu : (left > 0 ? (1u << left) - 1u : 0u);
      gt_mask &= in;
      eq_mask &= in;
    }
    uint32_t total;
    const uint32_t excl = block_excl_scan<THREADS>(__builtin_popcount(gt_mask) | (__builtin_popcount(eq_mask) << 16), tmp, total);
    // The step's kept tokens, places [first, last) of the list, are staged in LDS and copied out
    // coalesced, STAGE at a time: stored straight from their threads (a few 4-byte stores each,
    // scattered over the wave) they cost more than reading the row did.
    const uint32_t first = gbase + min(qbase, r);
    gbase += total & 0xffffu;
    qbase += total >> 16;
    const uint32_t last = min(gbase + min(qbase, r), c);
#pragma unroll 1
    for (uint32_t base = first; base < last; base += STAGE) {
      uint32_t g = first - min(qbase - (total >> 16), r) + (excl & 0xffffu);   // greater keys before this thread's run
      uint32_t q = qbase - (total >> 16) + (excl >> 16);                        // equal keys before it
      for (uint32_t rest = gt_mask | eq_mask; rest; rest &= rest - 1) {
        const int i = __builtin_ctz(rest);
        const bool is_gt = (gt_mask >> i) & 1u;
        if (is_gt || q < r) {
          const uint32_t pos = g + min(q, r);
          if (pos >= base && pos - base < (uint32_t)STAGE) staged[pos - base] = nlo + i;
        }
        g += is_gt ? 1u : 0u;
        q += is_gt ? 0u : 1u;
      }
      __syncthreads();
      const uint32_t cnt = min(last - base, (uint32_t)STAGE);
      for (int ti = t0; ti < t1; ++ti) {
        int32_t *dst = A.indices + ((size_t)bt * A.Hq + A.targets.tgt[ti]) * A.k + base;
        for (uint32_t p = tid; p < cnt; p += THREADS) dst[p] = staged[p];
      }
      __syncthreads();
    }
    if (gbase + min(qbase, r) >= c) break;   // the list is complete (uniform)
  }
}

// ------------------------------------------- at least a row per CU: one workgroup per row, ONE pass
// With a workgroup per row nothing has to be exchanged, but the row (128K tokens and more) does
// not fit into LDS, and every further pass over it costs its bytes again. What does fit is the
// narrow band of keys around the threshold, if the band is known before the pass. So:
//  1. Sample: runs of 128 bytes of a score row (32 fp32 or 64 bf16 tokens: whole cache lines, so
//     the sample costs 1/S of the row's traffic), one run in every S (S = 16, more for rows
//     beyond 256K so that at most 16384 keys are sampled), are aggregated and ranked out of LDS to
//     22 key bits: U, just above the
//     sample's key of rank c/S - z sqrt(c/S) - 2, and L, at or below its key of rank
//     c/S + z sqrt(c/S) + 3 (z = 5). Whatever the sample says, the result below is exact: the
//     sample only decides whether this pass suffices.
//  2. The pass: every token is aggregated once (same fp32 order). Keys >= U are certainly kept:
//     their bit is set in a bitmap of the row (LDS, one bit per token) and they are counted (G).
//     Keys in [L, U) go to the band store, unordered (an LDS counter hands out the slots), M of them.
//  3. If G < c <= G + M and the band fitted, the c-th largest key of the row is the (c - G)-th
//     largest of the band: three digit levels over the band in LDS give the threshold T and the
//     number r of keys equal to T that are kept; band entries above T get their bits, and of those
//     equal to T the r lowest tokens (a two-level search over the token ids when there are more).
//  4. The list is the bitmap read in order: each thread owns a run of words, one block scan gives
//     its first position.
// If the check of step 3 fails (about 1e-6 per row for the sampling error alone; rows with heavy
// ties or a structure the strided sample misses), the row is ranked by the plain passes over the
// scores instead (rank_by_passes): correct for every input, several times the traffic.
constexpr int BAND_THREADS = 1024;

// sum over the block of one value per thread; red needs THREADS / 64 words
template <int THREADS>
__device__ __forceinline__ uint32_t block_sum1(uint32_t a, uint32_t *red) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) a += (uint32_t)__shfl_xor((int)a, off, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = a;
  __syncthreads();
  uint32_t s = 0;
#pragma unroll
  for (int w = 0; w < THREADS / 64; ++w) s += red[w];
  __syncthreads();
  return s;
}

// The plain way for one workgroup to rank a row it cannot hold: a pass over the scores per digit
// level (the Tq rows are aggregated again each time, in the same order, so the keys repeat bit
// for bit), then a pass that compacts in token order. h: SEL_BINS words, tmp: THREADS/64 + 2.
template <int THREADS>
__device__ __forceinline__ void rank_by_passes(const SelectArgs &A, const AggRow &R, int bt, int nb, uint32_t c,
                                               int t0, int t1, uint32_t *h, uint32_t *tmp) {
  constexpr int NPOS = 2;
  const int tid = threadIdx.x;
  const int nq = (nb + 3) >> 2;           // quads that hold ranked tokens
  uint32_t d0 = 0, pre01 = 0, krem = c, d2 = 0;
#pragma unroll 1
  for (int level = 0; level < 3; ++level) {
    for (int i = tid; i < SEL_BINS; i += THREADS) h[i] = 0u;
    __syncthreads();
#pragma unroll 1
    for (int q0 = tid; q0 < nq; q0 += THREADS * NPOS) {
      int pos[NPOS];
      f32x4 acc[NPOS];
#pragma unroll
      for (int x = 0; x < NPOS; ++x) pos[x] = 4 * min(q0 + x * THREADS, nq - 1);
      agg_multi<f32x4, NPOS>(R, pos, acc);
#pragma unroll
      for (int x = 0; x < NPOS; ++x)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int n = 4 * (q0 + x * THREADS) + e;
          const int bin = fused_bin(key_of(acc[x][e]), level, d0, pre01);
          if (n < nb && bin >= 0) atomicAdd(&h[bin], 1u);
        }
    }
    __syncthreads();
    uint32_t digit, knext;
    find_digit<SEL_BINS, THREADS>(h, krem, tmp, digit, knext);
    if (level == 0) d0 = digit;
    else if (level == 1) pre01 = (d0 << SEL_BITS1) | digit;
    else d2 = digit;
    krem = knext;
  }
  const uint32_t r = krem, Tk = (pre01 << SEL_BITS2) | d2;
  // ordered compaction: per step, thread tid owns the NPOS consecutive quads from (step + tid * NPOS)
  uint32_t gbase = 0, qbase = 0;
#pragma unroll 1
  for (int step = 0; step < nq; step += THREADS * NPOS) {
    const int qlo = step + tid * NPOS;
    int pos[NPOS];
    f32x4 acc[NPOS];
#pragma unroll
    for (int x = 0; x < NPOS; ++x) pos[x] = 4 * min(qlo + x, nq - 1);
    agg_multi<f32x4, NPOS>(R, pos, acc);
    uint32_t gt_mask = 0, eq_mask = 0;
#pragma unroll
    for (int x = 0; x < NPOS; ++x)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t key = key_of(acc[x][e]);
        const bool in = 4 * (qlo + x) + e < nb;
        gt_mask |= (in && key > Tk) ? 1u << (4 * x + e) : 0u;
        eq_mask |= (in && key == Tk) ? 1u << (4 * x + e) : 0u;
      }
    uint32_t total;
    const uint32_t excl = block_excl_scan<THREADS>(__builtin_popcount(gt_mask) | (__builtin_popcount(eq_mask) << 16), tmp, total);
    uint32_t g = gbase + (excl & 0xffffu), q = qbase + (excl >> 16);
    for (uint32_t rest = gt_mask | eq_mask; rest; rest &= rest - 1) {
      const int i = __builtin_ctz(rest);
      const bool is_gt = (gt_mask >> i) & 1u;
      if (is_gt || q < r) {
        const uint32_t p = g + min(q, r);
        if (p < c)
          for (int ti = t0; ti < t1; ++ti) A.indices[((size_t)bt * A.Hq + A.targets.tgt[ti]) * A.k + p] = 4 * qlo + i;
      }
      g += is_gt ? 1u : 0u;
      q += is_gt ? 0u : 1u;
    }
    gbase += total & 0xffffu;
    qbase += total >> 16;
    if (gbase + min(qbase, r) >= c) break;   // the list is complete (uniform)
  }
}

// the c-th largest (1 <= c <= m) of keys[0 .. m), all of which lie in [lo, hi], and how many keys
// equal to it are kept. A digit that lo and hi share needs no histogram.
template <int THREADS>
__device__ __forceinline__ void band_threshold(const uint32_t *keys, int m, uint32_t c, uint32_t lo, uint32_t hi,
                                               uint32_t *h, uint32_t *tmp, uint32_t &Tk, uint32_t &r) {
  const int tid = threadIdx.x;
  uint32_t d0 = 0, pre01 = 0, krem = c, d2 = 0;
#pragma unroll 1
  for (int level = 0; level < 3; ++level) {
    if (level == 0 && (lo >> (32 - SEL_BITS0)) == (hi >> (32 - SEL_BITS0))) {
      d0 = lo >> (32 - SEL_BITS0);
      continue;
    }
    if (level == 1 && (lo >> SEL_BITS2) == (hi >> SEL_BITS2)) {
      pre01 = lo >> SEL_BITS2;
      continue;
    }
    for (int i = tid; i < SEL_BINS; i += THREADS) h[i] = 0u;
    __syncthreads();
    for (int i = tid; i < m; i += THREADS) {
      const int bin = fused_bin(keys[i], level, d0, pre01);
      if (bin >= 0) atomicAdd(&h[bin], 1u);
    }
    __syncthreads();
    uint32_t digit, knext;
    find_digit<SEL_BINS, THREADS>(h, krem, tmp, digit, knext);
    if (level == 0) d0 = digit;
    else if (level == 1) pre01 = (d0 << SEL_BITS1) | digit;
    else d2 = digit;
    krem = knext;
  }
  Tk = (pre01 << SEL_BITS2) | d2;
  r = krem;
}

// the pass of select_band_kernel with NPOS quads in flight per thread
template <int NPOS>
__device__ __forceinline__ uint32_t band_pass(const SelectArgs &A, const AggRow &R, float *out, int nb, bool spec, bool haveU,
                                              uint32_t U, bool haveL, uint32_t L, uint32_t *bits, uint32_t *skey,
                                              uint32_t *sidx, uint32_t *ctr) {
  constexpr int T = BAND_THREADS;
  const int tid = threadIdx.x, lane = tid & 63;
  const int nq = (nb + 3) >> 2;
  const int words = (nb + 31) >> 5;
  const int nq_all = spec ? ((nq + 7) & ~7) : 0;       // whole bitmap words
  const int nq_out = out ? A.N >> 2 : 0;               // the aggregate is stored for the whole row
  // keys >= U are certainly kept (none without an upper edge); the others from L on are the band
  const uint32_t L_eff = haveL ? L : 0u;
  const uint32_t up_on = haveU ? 0xfu : 0u;
  uint32_t G = 0;
#pragma unroll 1
  for (int q0 = tid; q0 < max(nq_all, nq_out); q0 += T * NPOS) {
    int pos[NPOS];
    f32x4 acc[NPOS];
    bool any = false;
#pragma unroll
    for (int x = 0; x < NPOS; ++x) {
      pos[x] = 4 * min(q0 + x * T, max(nq - 1, 0));
      any |= q0 + x * T < nq;
    }
    if (__builtin_amdgcn_ballot_w64(any)) {
      agg_multi_lim<f32x4, NPOS, (NPOS >= 8 ? 1 : (NPOS >= 4 ? 3 : 8))>(R, pos, acc);
    } else {                                           // a wave past the ranked length (it only stores zeros)
#pragma unroll
      for (int x = 0; x < NPOS; ++x) acc[x] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    uint32_t keys[NPOS][4];
    uint32_t band = 0;                                 // bit 4x + e: that token belongs to the band
#pragma unroll
    for (int x = 0; x < NPOS; ++x) {
      const int q = q0 + x * T;
      // tokens this quad holds inside the ranked length: 4 everywhere but at the row's end
      const int valid = q < nq ? min(4, nb - 4 * q) : 0;
      uint32_t up = 0, bd = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t key = key_of(acc[x][e]);
        keys[x][e] = key;
        up |= (key >= U) ? 1u << e : 0u;
        bd |= (key >= L_eff) ? 1u << e : 0u;
      }
      const uint32_t vmask = spec ? (1u << valid) - 1u : 0u;
      const uint32_t nib = up & up_on & vmask;
      band |= (bd & ~nib & vmask) << (4 * x);
      if (out && q < nq_out) {
        f32x4 o = acc[x];
        if (valid < 4) {
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = e < valid ? o[e] : 0.f;
        }
        *reinterpret_cast<f32x4 *>(out + 4 * (size_t)q) = o;
      }
      if (q < nq_all) {
        // the nibbles of eight neighbouring quads make one bitmap word, stored whole by the first
        // lane of the eight: three shifts by 1, 2, 4 lanes inside a row of 16 lanes, OR-ed
        G += __builtin_popcount(nib);
        int v = (int)(nib << (4 * (lane & 7)));
        v |= __builtin_amdgcn_update_dpp(0, v, 0x101, 0xf, 0xf, true);   // row_shl:1
        v |= __builtin_amdgcn_update_dpp(0, v, 0x102, 0xf, 0xf, true);   // row_shl:2
        v |= __builtin_amdgcn_update_dpp(0, v, 0x104, 0xf, 0xf, true);   // row_shl:4
        if ((lane & 7) == 0 && (q >> 3) < words) bits[q >> 3] = (uint32_t)v;
      }
    }
    if (band) {                                        // one slot request per thread and step
      uint32_t slot = atomicAdd(ctr, (uint32_t)__builtin_popcount(band));
#pragma unroll
      for (int x = 0; x < NPOS; ++x)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if ((band >> (4 * x + e)) & 1u) {
            if (slot < (uint32_t)BAND_CAP) {
              skey[slot] = keys[x][e];
              sidx[slot] = (uint32_t)(4 * (q0 + x * T) + e);
            }
            ++slot;
          }
    }
  }
  return G;
}

__global__ void __launch_bounds__(BAND_THREADS) select_band_kernel(const SelectArgs A) {
  constexpr int T = BAND_THREADS;
  __shared__ uint32_t bits[BAND_MAX_N / 32];           // bit n: token n is kept
  __shared__ __attribute__((aligned(16))) uint32_t store[2 * BAND_CAP];   // sample keys; band keys and tokens; staged list
  __shared__ uint32_t h[2][SEL_BINS];
  __shared__ uint32_t tmp[T / 64 + 2];
  __shared__ uint32_t red[T / 64];
  __shared__ uint32_t ctr[2];
  uint32_t *skey = store, *sidx = store + BAND_CAP;
  const int row = blockIdx.x, tid = threadIdx.x;
  const int bt = row / A.Hd, j = row % A.Hd;
  const int nb = row_len(A, bt);
  const uint32_t c = (uint32_t)min(A.kh[j], nb);
  const int t0 = A.targets.off[j], t1 = A.targets.off[j + 1];
  write_tail<T>(A, bt, j, c);
  const bool want_agg = A.agg != nullptr;
  const bool ranked = c > 0 && t0 != t1;
  if (!ranked && !want_agg) return;
  const AggRow R = agg_row(A, row);
  float *out = want_agg ? A.agg + (size_t)row * A.N : nullptr;

  // ---- 1. the band [L, U) from a strided sample
  bool haveU = false, haveL = false, spec = ranked;
  uint32_t U = 0, L = 0;
  if (ranked && nb > BAND_CAP) {
    const int run = R.bf16 ? 64 : 32;                  // tokens per sampled run: 128 bytes of a score row
    const BandPlan bp = band_plan(nb, c, run);
    const int ns = bp.ns, rq = run >> 2;
    haveU = bp.s_hi >= 1;
    haveL = true;
    spec = bp.fits;
    if (spec) {
      for (int i = tid; i < SEL_BINS; i += T) h[0][i] = 0u;
      __syncthreads();
      for (int s0 = tid; 4 * s0 < ns; s0 += 2 * T) {   // sampled quad s: quad s % rq of run s / rq; two in flight
        int pos[2];
        f32x4 acc[2];
#pragma unroll
        for (int x = 0; x < 2; ++x) {
          const int s = min(s0 + x * T, (ns - 1) >> 2);
          pos[x] = (s / rq) * bp.S * run + (s % rq) * 4;
        }
        agg_multi<f32x4, 2>(R, pos, acc);
#pragma unroll
        for (int x = 0; x < 2; ++x)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const uint32_t key = key_of(acc[x][e]);
            const int i = 4 * (s0 + x * T) + e;
            if (i < ns) {
              skey[i] = key;
              atomicAdd(&h[0][key >> (32 - SEL_BITS0)], 1u);
            }
          }
      }
      __syncthreads();
      uint32_t dh = 0, kh1 = 1, dl, kl1, dh1 = 0, dl1;
      if (haveU) find_digit<SEL_BINS, T>(h[0], (uint32_t)bp.s_hi, tmp, dh, kh1);
      find_digit<SEL_BINS, T>(h[0], (uint32_t)bp.s_lo, tmp, dl, kl1);
      for (int i = tid; i < SEL_BINS; i += T) h[0][i] = h[1][i] = 0u;
      __syncthreads();
      for (int i = tid; i < ns; i += T) {
        const uint32_t key = skey[i], top = key >> (32 - SEL_BITS0), mid = (key >> SEL_BITS2) & ((1u << SEL_BITS1) - 1);
        if (haveU && top == dh) atomicAdd(&h[0][mid], 1u);
        if (top == dl) atomicAdd(&h[1][mid], 1u);
      }
      __syncthreads();
      uint32_t unused;
      if (haveU) find_digit<SEL_BINS, T>(h[0], kh1, tmp, dh1, unused);
      find_digit<SEL_BINS, T>(h[1], kl1, tmp, dl1, unused);
      const uint32_t u22 = ((dh << SEL_BITS1) | dh1) + 1u;
      if (haveU && u22 < (1u << (SEL_BITS0 + SEL_BITS1))) U = u22 << SEL_BITS2;
      else haveU = false;                              // nothing can lie above the sample's top bin
      L = ((dl << SEL_BITS1) | dl1) << SEL_BITS2;
    }
  }
  // rows of up to BAND_CAP tokens: the whole row is the band (haveU = haveL = false, spec = true)

  // ---- 2. the pass; about 16 row loads in flight per thread whatever Tq is
  if (tid == 0) ctr[0] = 0u;
  __syncthreads();
  uint32_t G = 0;
  if (spec || want_agg) {
    if (A.Tq == 1) G = band_pass<8>(A, R, out, nb, spec, haveU, U, haveL, L, bits, skey, sidx, ctr);
    else if (A.Tq <= 3) G = band_pass<4>(A, R, out, nb, spec, haveU, U, haveL, L, bits, skey, sidx, ctr);
    else G = band_pass<2>(A, R, out, nb, spec, haveU, U, haveL, L, bits, skey, sidx, ctr);
  }
  __syncthreads();
  if (!ranked) return;
  const uint32_t M = ctr[0];
  G = block_sum1<T>(G, red);
  if (!spec || G >= c || G + M < c || M > (uint32_t)BAND_CAP) {
    rank_by_passes<T>(A, R, bt, nb, c, t0, t1, h[0], tmp);
    return;
  }

  // ---- 3. the threshold inside the band, bits of the band's kept tokens
  uint32_t Tk, r;
  band_threshold<T>(skey, (int)M, c - G, haveL ? L : 0u, haveU ? U - 1u : 0xffffffffu, h[0], tmp, Tk, r);
  uint32_t E = 0;
  for (int i = tid; i < (int)M; i += T) {
    const uint32_t key = skey[i];
    if (key > Tk) atomicOr(&bits[sidx[i] >> 5], 1u << (sidx[i] & 31));
    E += key == Tk ? 1u : 0u;
  }
  E = block_sum1<T>(E, red);
  uint32_t cut = 0;                                    // equal keys are kept from this reversed token id on
  if (E > r) {
    // the r lowest tokens among the E equal ones: rank the reversed ids, 11 + 8 bits
    constexpr uint32_t REV = BAND_MAX_N - 1;
    for (int i = tid; i < SEL_BINS; i += T) h[0][i] = 0u;
    __syncthreads();
    for (int i = tid; i < (int)M; i += T)
      if (skey[i] == Tk) atomicAdd(&h[0][(REV - sidx[i]) >> 8], 1u);
    __syncthreads();
    uint32_t da, ra, db, rb;
    find_digit<SEL_BINS, T>(h[0], r, tmp, da, ra);
    for (int i = tid; i < SEL_BINS; i += T) h[0][i] = 0u;
    __syncthreads();
    for (int i = tid; i < (int)M; i += T)
      if (skey[i] == Tk && ((REV - sidx[i]) >> 8) == da) atomicAdd(&h[0][(REV - sidx[i]) & 255u], 1u);
    __syncthreads();
    find_digit<SEL_BINS, T>(h[0], ra, tmp, db, rb);
    cut = (da << 8) | db;
  }
  for (int i = tid; i < (int)M; i += T)
    if (skey[i] == Tk && (BAND_MAX_N - 1 - sidx[i]) >= cut) atomicOr(&bits[sidx[i] >> 5], 1u << (sidx[i] & 31));
  __syncthreads();

  // ---- 4. the list: set bits in token order, staged in LDS (the band store is free now) and
  // copied out coalesced, once per target head, 2 * BAND_CAP entries per round
  const int words = (nb + 31) >> 5;
  const int per = (words + T - 1) / T;                 // words per thread, consecutive
  const int w0 = min(tid * per, words), w1 = min(w0 + per, words);
  uint32_t mine = 0;
  for (int w = w0; w < w1; ++w) mine += __builtin_popcount(bits[w]);
  uint32_t total;
  const uint32_t first = block_excl_scan<T>(mine, tmp, total);
  const uint32_t kept = min(total, c);                 // total == c for a consistent state
  int32_t *staged = reinterpret_cast<int32_t *>(store);
#pragma unroll 1
  for (uint32_t base = 0; base < kept; base += 2 * BAND_CAP) {
    uint32_t p = first;
    if (p < base + 2 * BAND_CAP && p + mine > base)
      for (int w = w0; w < w1; ++w)
        for (uint32_t rest = bits[w]; rest; rest &= rest - 1) {
          if (p >= base && p - base < 2u * BAND_CAP) staged[p - base] = 32 * w + __builtin_ctz(rest);
          ++p;
        }
    __syncthreads();
    const uint32_t cnt = min(kept - base, 2u * BAND_CAP);
    for (int ti = t0; ti < t1; ++ti) {
      int32_t *dst = A.indices + ((size_t)bt * A.Hq + A.targets.tgt[ti]) * A.k + base;
      for (uint32_t i = tid; i < cnt; i += T) dst[i] = staged[i];
    }
    __syncthreads();
  }
}

// ---------------------------------------------- small budgets on long rows: chunk-local top-k
// Every token of a row's top-c (ordered by key descending, then token ascending) has fewer
// than c tokens of the whole row before it in that order, hence fewer than c tokens of its own
// chunk: it belongs to the top-c of its chunk under the same rule. So each chunk keeps only
// its own best min(c, chunk length) tokens (the pool), and the row is ranked from the pool.
//
// Local kernel, (chunk, row) grid, 256 threads per 8192-token chunk or 1024 per 32768-token
// chunk (fewer, larger chunks keep the pool small on very long rows): aggregates the chunk (same
// fp32 order), keeps the 32 keys of each thread in registers, finds the chunk's threshold with three LDS digit
// histograms, and writes the kept (key, token) pairs to the chunk's pool segment in token
// order. Thread t owns tokens n0 + (i*THREADS + t)*4 .. +3 for i = 0..7, so token order is (i, t).
template <int IT>
struct LocalKeys {
  uint32_t k[IT][4];
};

template <int THREADS>
__global__ void __launch_bounds__(THREADS) select_local_kernel(const SelectArgs A) {
  constexpr int CHUNK = THREADS * 32;          // 32 keys per thread
  constexpr int IT = 8;
  __shared__ uint32_t h[SEL_BINS];
  __shared__ uint32_t tmp[THREADS / 64 + 2];
  const int row = blockIdx.y, chunk = blockIdx.x;
  const int bt = row / A.Hd, j = row % A.Hd;
  const int nb = row_len(A, bt);
  const int n0 = chunk * CHUNK;
  const int nvalid = max(0, min(n0 + CHUNK, nb) - n0);     // ranked tokens of this chunk
  uint32_t c = (uint32_t)min(A.kh[j], nvalid);
  const bool want_agg = A.agg != nullptr;
  if (A.targets.off[j] == A.targets.off[j + 1]) c = 0;        // no target head reads this draft head
  if (c == 0 && !want_agg) return;
  for (int i = threadIdx.x; i < SEL_BINS; i += THREADS) h[i] = 0u;
  __syncthreads();
  const AggRow R = agg_row(A, row);
  float *out = want_agg ? A.agg + (size_t)row * A.N : nullptr;
  LocalKeys<IT> K;
#pragma clang loop unroll(full)
  for (int i = 0; i < IT; ++i) {
    const int n = n0 + (i * THREADS + threadIdx.x) * 4;
    if (n < A.N) {                                             // N % 4 == 0 on this path
      const f32x4 acc = agg_quad(R, n);
      f32x4 o = acc;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        K.k[i][e] = key_of(acc[e]);
        if (n + e < nb) atomicAdd(&h[K.k[i][e] >> (32 - SEL_BITS0)], 1u);
        else o[e] = 0.f;
      }
      if (want_agg) *reinterpret_cast<f32x4 *>(out + n) = o;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) K.k[i][e] = 0u;
    }
  }
  __syncthreads();
  if (c == 0) return;
  // threshold of the chunk: three digits over the register-resident keys
  uint32_t d0, k1, d1, k2, d2, r;
  find_digit<(1 << SEL_BITS0), THREADS>(h, c, tmp, d0, k1);
  for (int i = threadIdx.x; i < SEL_BINS; i += THREADS) h[i] = 0u;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < IT; ++i)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int n = n0 + (i * THREADS + threadIdx.x) * 4 + e;
      const uint32_t key = K.k[i][e];
      if (n < nb && (key >> (SEL_BITS1 + SEL_BITS2)) == d0) atomicAdd(&h[(key >> SEL_BITS2) & ((1u << SEL_BITS1) - 1)], 1u);
    }
  __syncthreads();
  find_digit<(1 << SEL_BITS1), THREADS>(h, k1, tmp, d1, k2);
  for (int i = threadIdx.x; i < SEL_BINS; i += THREADS) h[i] = 0u;
  __syncthreads();
  const uint32_t pre01 = (d0 << SEL_BITS1) | d1;
#pragma unroll
  for (int i = 0; i < IT; ++i)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int n = n0 + (i * THREADS + threadIdx.x) * 4 + e;
      const uint32_t key = K.k[i][e];
      if (n < nb && (key >> SEL_BITS2) == pre01) atomicAdd(&h[key & ((1u << SEL_BITS2) - 1)], 1u);
    }
  __syncthreads();
  find_digit<(1 << SEL_BITS2), THREADS>(h, k2, tmp, d2, r);
  const uint32_t T = (pre01 << SEL_BITS2) | d2;

  // Ordered compaction into the chunk's pool segment, one block scan per sweep of 1024 tokens.
  // Every chunk before this one is full and keeps min(budget, CHUNK) pairs, so the row's
  // pool is contiguous and this chunk's place in it is known without communication.
  const size_t seg = (size_t)row * A.pool_nchunks * A.pool_pitch + (size_t)chunk * min(A.kh[j], CHUNK);
  uint32_t *pk = A.pool_key + seg;
  int32_t *pi = A.pool_idx + seg;
  uint32_t g0 = 0, q0 = 0;                                     // greater / equal in the sweeps before
#pragma unroll
  for (int i = 0; i < IT; ++i) {
    const int n = n0 + (i * THREADS + threadIdx.x) * 4;
    uint32_t cg = 0, ce = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const bool in = n + e < nb;
      cg += (in && K.k[i][e] > T) ? 1u : 0u;
      ce += (in && K.k[i][e] == T) ? 1u : 0u;
    }
    uint32_t total;
    const uint32_t excl = block_excl_scan<THREADS>(cg | (ce << 16), tmp, total);
    uint32_t g = g0 + (excl & 0xffffu), q = q0 + (excl >> 16);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const bool in = n + e < nb;
      const bool is_gt = in && K.k[i][e] > T, is_eq = in && K.k[i][e] == T;
      if (is_gt || (is_eq && q < r)) {
        const uint32_t pos = g + min(q, r);
        if (pos < c) {                 // always true for a consistent threshold
          pk[pos] = K.k[i][e];
          pi[pos] = n + e;
        }
      }
      g += is_gt ? 1u : 0u;
      q += is_eq ? 1u : 0u;
    }
    g0 += total & 0xffffu;
    q0 += total >> 16;
  }
}

// Pool kernel, one 1024-thread workgroup per row: the chunks' kept pairs, concatenated in
// chunk order (= token order), are loaded into LDS and ranked like a short row; the kept
// tokens go to every target head of the draft head.
constexpr int POOL_MAX = SEL_POOL_MAX;   // pooled pairs per row: keys and tokens fit in LDS
__global__ void __launch_bounds__(SMALL_THREADS) select_pool_kernel(const SelectArgs A) {
  __shared__ uint32_t keys[POOL_MAX + POOL_MAX / 32];
  __shared__ int32_t toks[POOL_MAX + POOL_MAX / 32];
  __shared__ uint32_t h[SEL_BINS];
  __shared__ uint32_t red[2 * SMALL_THREADS / 64];
  __shared__ uint32_t tmp[SMALL_THREADS / 64 + 2];
  const int row = blockIdx.x;
  const int bt = row / A.Hd, j = row % A.Hd;
  const int nb = row_len(A, bt);
  const uint32_t c = (uint32_t)min(A.kh[j], nb);
  const int t0 = A.targets.off[j], t1 = A.targets.off[j + 1];
  const int tid = threadIdx.x;
  write_tail<SMALL_THREADS>(A, bt, j, c);
  if (c == 0 || t0 == t1) return;
  for (int i = tid; i < SEL_BINS; i += SMALL_THREADS) h[i] = 0u;
  // pooled pairs of the row: the full chunks keep min(budget, chunk length) each, the last one
  // min(budget, its length)
  const uint32_t kfull = (uint32_t)min(A.kh[j], A.pool_chunk);
  const uint32_t m = min((uint32_t)(nb / A.pool_chunk) * kfull + min((uint32_t)A.kh[j], (uint32_t)(nb % A.pool_chunk)),
                         (uint32_t)POOL_MAX);
  const uint32_t *pk = A.pool_key + (size_t)row * A.pool_nchunks * A.pool_pitch;
  const int32_t *pi = A.pool_idx + (size_t)row * A.pool_nchunks * A.pool_pitch;
  // The pairs were written by other workgroups: their loads miss the caches, so eight
  // independent ones are issued per thread before any is used (uniform trip count, clamped
  // addresses, the surplus ignored).
  uint32_t kmin = 0xffffffffu, kmax = 0u;
  for (uint32_t e0 = 0; e0 < m; e0 += SMALL_THREADS * 8) {
    uint32_t key[8];
    int32_t tok[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const uint32_t e = min(e0 + u * SMALL_THREADS + tid, m - 1);
      key[u] = pk[e];
      tok[u] = pi[e];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const uint32_t e = e0 + u * SMALL_THREADS + tid;
      if (e < m) {
        keys[small_slot((int)e)] = key[u];
        toks[small_slot((int)e)] = tok[u];
        kmin = min(kmin, key[u]);
        kmax = max(kmax, key[u]);
      }
    }
  }
  // The pooled keys are all large, so their leading bits agree and the first digit would put
  // them into a handful of bins (LDS atomics on one address serialise). Ranking the keys
  // shifted left by the length of their common prefix is the same ranking and spreads them.
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, off, 64));
    kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, off, 64));
  }
  if ((tid & 63) == 0) {
    red[(tid >> 6) * 2] = kmin;
    red[(tid >> 6) * 2 + 1] = kmax;
  }
  __syncthreads();
#pragma unroll
  for (int w = 0; w < SMALL_THREADS / 64; ++w) {
    kmin = min(kmin, red[w * 2]);
    kmax = max(kmax, red[w * 2 + 1]);
  }
  uint32_t T, r;
  if (kmin == kmax) {
    T = kmin;            // all pooled keys are equal: the first c in token order are kept
    r = c;
  } else {
    const int shift = __clz((int)(kmin ^ kmax));               // 0..31
    for (uint32_t e = tid; e < m; e += SMALL_THREADS) {
      const uint32_t key = keys[small_slot((int)e)] << shift;
      keys[small_slot((int)e)] = key;
      atomicAdd(&h[key >> (32 - SEL_BITS0)], 1u);
    }
    __syncthreads();
    lds_threshold<SMALL_THREADS>(keys, (int)m, h, tmp, c, T, r);
  }
  lds_compact<SMALL_THREADS, POOL_MAX / SMALL_THREADS>(keys, (int)m, T, r, c, tmp, [&](uint32_t pos, int n) {
    const int32_t tok = toks[small_slot(n)];
    for (int ti = t0; ti < t1; ++ti) A.indices[((size_t)bt * A.Hq + A.targets.tgt[ti]) * A.k + pos] = tok;
  });
}

}  // namespace

static inline bool vec_ok(const SelectArgs &a) {   // aggregation: scores and agg rows
  return (a.N % 4) == 0 && (reinterpret_cast<uintptr_t>(a.scores) % 16) == 0 &&
         (reinterpret_cast<uintptr_t>(a.agg) % 16) == 0;
}

static inline bool src_vec_ok(const SelectArgs &a) {   // ranking passes: rows of src
  return (a.srcN % 4) == 0 && (reinterpret_cast<uintptr_t>(a.src) % 16) == 0;
}

hipError_t launch_select_small(const SelectArgs &a, hipStream_t s) {
  if ((size_t)a.B * a.Hd == 0) return hipSuccess;
  const dim3 grid(a.B * a.Hd), block(SMALL_THREADS);
  const bool v = (a.N % 4) == 0 && (reinterpret_cast<uintptr_t>(a.scores) % 16) == 0 &&
                 (a.agg == nullptr || (reinterpret_cast<uintptr_t>(a.agg) % 16) == 0);
  if (v)
    STS_LAUNCH((select_small_kernel<true, false>), grid, block, 0, s, a);
  else
    STS_LAUNCH((select_small_kernel<false, false>), grid, block, 0, s, a);
  return sts_take_launch_status();
}

// ranks the rows of a.src (up to SEL_SMALL_N entries each) out of LDS
hipError_t launch_select_rank(const SelectArgs &a, hipStream_t s) {
  if ((size_t)a.B * a.Hd == 0) return hipSuccess;
  STS_LAUNCH((select_small_kernel<false, true>), dim3(a.B * a.Hd), dim3(SMALL_THREADS), 0, s, a);
  return sts_take_launch_status();
}

bool select_aggblock_ok(const SelectArgs &a) {
  const bool pow2 = (a.page & (a.page - 1)) == 0;
  return pow2 && a.page >= 4 && a.page <= 256 && (a.N % a.page) == 0 &&
         (reinterpret_cast<uintptr_t>(a.scores) % 16) == 0 &&
         (a.agg == nullptr || (reinterpret_cast<uintptr_t>(a.agg) % 16) == 0);
}

hipError_t launch_select_aggblock(const SelectArgs &a, hipStream_t s) {
  if ((size_t)a.B * a.Hd == 0 || a.N == 0) return hipSuccess;
  const dim3 grid((a.N + SEL_CHUNK - 1) / SEL_CHUNK, a.B * a.Hd), block(SEL_THREADS);
  STS_LAUNCH(select_aggblock_kernel, grid, block, 0, s, a);
  return sts_take_launch_status();
}

hipError_t launch_select_fused(const SelectArgs &a, hipStream_t s) {
  if ((size_t)a.B * a.Hd == 0 || a.parts == 0) return hipSuccess;
  const dim3 grid(a.parts, a.B * a.Hd), block(FUSED_THREADS);
  const bool v = (a.N % 4) == 0 && (reinterpret_cast<uintptr_t>(a.scores) % 16) == 0 &&
                 (a.agg == nullptr || (reinterpret_cast<uintptr_t>(a.agg) % 16) == 0);
#define STS_FUSED(PER)                                                                     \
  do {                                                                                     \
    if (v) STS_LAUNCH((select_fused_kernel<true, PER>), grid, block, 0, s, a);             \
    else STS_LAUNCH((select_fused_kernel<false, PER>), grid, block, 0, s, a);              \
  } while (0)
  switch (a.part_tokens) {
    case 8192: STS_FUSED(8); break;
    case 16384: STS_FUSED(16); break;
    case 32768: STS_FUSED(32); break;
    default: return hipErrorInvalidValue;
  }
#undef STS_FUSED
  return sts_take_launch_status();
}

// one workgroup per row, Tq == 1, unpaged, no aggregate output; the caller has checked the shape
bool select_rowpass_ok(const SelectArgs &a) {
  return a.Tq == 1 && a.kind == STS_SCORES_PROBS && a.page == 1 && a.agg == nullptr && a.N > 0 &&
         (a.N % (a.scores_bf16 ? 8 : 4)) == 0 && (reinterpret_cast<uintptr_t>(a.scores) % 16) == 0;
}

hipError_t launch_select_rowpass(const SelectArgs &a, hipStream_t s) {
  if ((size_t)a.B * a.Hd == 0) return hipSuccess;
  if (!select_rowpass_ok(a)) return hipErrorInvalidValue;
  const dim3 grid(a.B * a.Hd);
  if (a.rowpass_threads == 1024) {
    if (a.scores_bf16) STS_LAUNCH((select_rowpass_kernel<1024, true>), grid, dim3(1024), 0, s, a);
    else STS_LAUNCH((select_rowpass_kernel<1024, false>), grid, dim3(1024), 0, s, a);
  } else {
    if (a.scores_bf16) STS_LAUNCH((select_rowpass_kernel<256, true>), grid, dim3(256), 0, s, a);
    else STS_LAUNCH((select_rowpass_kernel<256, false>), grid, dim3(256), 0, s, a);
  }
  return sts_take_launch_status();
}

// one workgroup per row and one pass (select_band_kernel): token granularity, quads, a bitmap of the row in LDS
bool select_band_ok(const SelectArgs &a) {
  return a.page == 1 && a.N > 0 && a.N <= BAND_MAX_N && (a.N % 4) == 0 && (reinterpret_cast<uintptr_t>(a.scores) % 16) == 0 &&
         (a.agg == nullptr || (reinterpret_cast<uintptr_t>(a.agg) % 16) == 0);
}

hipError_t launch_select_band(const SelectArgs &a, hipStream_t s) {
  if ((size_t)a.B * a.Hd == 0) return hipSuccess;
  if (!select_band_ok(a)) return hipErrorInvalidValue;
  STS_LAUNCH(select_band_kernel, dim3(a.B * a.Hd), dim3(BAND_THREADS), 0, s, a);
  return sts_take_launch_status();
}

// zeroes the area the parts of the fused selection publish their histograms in (one 64-bit word per
// row, level, part and thread), 16 bytes per thread
hipError_t launch_select_clear_pub(const SelectArgs &a, hipStream_t s) {
  const size_t n16 = (size_t)a.B * a.Hd * 3 * (size_t)a.parts * FUSED_THREADS / 2;
  if (n16 == 0) return hipSuccess;
  STS_LAUNCH(select_clear16_kernel, dim3((unsigned)((n16 + SEL_THREADS - 1) / SEL_THREADS)), dim3(SEL_THREADS), 0, s,
             reinterpret_cast<u32x4 *>(a.pub), n16);
  return sts_take_launch_status();
}

hipError_t launch_select_local(const SelectArgs &a, hipStream_t s) {
  if ((size_t)a.B * a.Hd == 0 || a.pool_nchunks == 0) return hipSuccess;
  const dim3 grid(a.pool_nchunks, a.B * a.Hd);
  if (a.pool_chunk == 256 * 32)
    STS_LAUNCH(select_local_kernel<256>, grid, dim3(256), 0, s, a);
  else   // 1024 * 32
    STS_LAUNCH(select_local_kernel<1024>, grid, dim3(1024), 0, s, a);
  return sts_take_launch_status();
}

hipError_t launch_select_pool(const SelectArgs &a, hipStream_t s) {
  if ((size_t)a.B * a.Hd == 0) return hipSuccess;
  STS_LAUNCH(select_pool_kernel, dim3(a.B * a.Hd), dim3(SMALL_THREADS), 0, s, a);
  return sts_take_launch_status();
}

hipError_t launch_select_block(const SelectArgs &a, hipStream_t s) {
  if ((size_t)a.B * a.Hd == 0 || a.srcN == 0) return hipSuccess;
  const bool pow2 = (a.page & (a.page - 1)) == 0;
  if (pow2 && a.page >= 4 && a.page <= 256 && (a.N % a.page) == 0 &&
      (reinterpret_cast<uintptr_t>(a.agg) % 16) == 0) {
    const dim3 grid((a.N + SEL_CHUNK - 1) / SEL_CHUNK, a.B * a.Hd), block(SEL_THREADS);
    STS_LAUNCH(select_block_vec_kernel, grid, block, 0, s, a);
  } else {
    const dim3 grid((a.srcN + SEL_THREADS - 1) / SEL_THREADS, a.B * a.Hd), block(SEL_THREADS);
    STS_LAUNCH(select_block_kernel, grid, block, 0, s, a);
  }
  return sts_take_launch_status();
}

hipError_t launch_select_clear(const SelectArgs &a, hipStream_t s) {
  const size_t n = (size_t)a.clear_words;
  if (n == 0) return hipSuccess;
  STS_LAUNCH(select_clear_kernel, dim3((unsigned)((n + SEL_THREADS - 1) / SEL_THREADS)),
                     dim3(SEL_THREADS), 0, s, a.hist, n);
  return sts_take_launch_status();
}

hipError_t launch_select_agg(const SelectArgs &a, hipStream_t s) {
  const int chunks = (a.N + SEL_CHUNK - 1) / SEL_CHUNK;
  if ((size_t)a.B * a.Hd == 0 || chunks == 0) return hipSuccess;
  const dim3 grid(chunks, a.B * a.Hd), block(SEL_THREADS);
  if (vec_ok(a))
    STS_LAUNCH(select_agg_kernel<true>, grid, block, 0, s, a);
  else
    STS_LAUNCH(select_agg_kernel<false>, grid, block, 0, s, a);
  return sts_take_launch_status();
}

hipError_t launch_select_hist(const SelectArgs &a, int pass, hipStream_t s) {
  if ((size_t)a.B * a.Hd == 0 || a.nchunks == 0) return hipSuccess;
  const dim3 grid((a.nchunks + a.hist_cpw - 1) / a.hist_cpw, a.B * a.Hd), block(SEL_THREADS);
  const bool v = src_vec_ok(a);
  if (pass == 1) {
    if (v) STS_LAUNCH((select_hist_kernel<1, true>), grid, block, 0, s, a);
    else STS_LAUNCH((select_hist_kernel<1, false>), grid, block, 0, s, a);
  } else {
    if (v) STS_LAUNCH((select_hist_kernel<2, true>), grid, block, 0, s, a);
    else STS_LAUNCH((select_hist_kernel<2, false>), grid, block, 0, s, a);
  }
  return sts_take_launch_status();
}

hipError_t launch_select_write(const SelectArgs &a, hipStream_t s) {
  if ((size_t)a.B * a.Hd == 0) return hipSuccess;
  const dim3 grid(a.nchunks > 0 ? a.nchunks : 1, a.B * a.Hd), block(SEL_THREADS);
  if (src_vec_ok(a))
    STS_LAUNCH(select_write_kernel<true>, grid, block, 0, s, a);
  else
    STS_LAUNCH(select_write_kernel<false>, grid, block, 0, s, a);
  return sts_take_launch_status();
}
