// Two-dimensional masks of prefill (paper Section 4.2: during prefill every query token has an
// index set of its own). For a block of up to 16 query rows the attention kernel gathers the
// UNION of the rows' sets once and is told, per gathered token, which rows keep it. This kernel
// builds that form from per-row lists: for every (batch, target head) the ascending union of the
// lists of its draft head's rows, and a 16-bit word per union entry, bit i set iff row i keeps
// the token.
//
// One 1024-thread workgroup per (draft head, batch); the union is the same for every target head
// that reads the draft head and is written to each of them. The token range is walked in chunks
// of 32768 tokens whose row bits sit in LDS (two tokens per word): every list entry that falls
// into the chunk ORs its row's bit into its token's half word (one entry of every row per thread
// in flight: the lists come out of L2, and a thread that waited for each entry in turn spent
// most of its time waiting); then every thread takes 32 consecutive tokens, one block scan gives the
// kept tokens their places, and they are written in token order.
#include "common.h"

namespace {

constexpr int UN_THREADS = 1024;
constexpr int UN_CHUNK = 32768;            // tokens per LDS pass
constexpr int UN_MAX_SEG = 64;             // chunks up to which the lists are read by segments (2M tokens)
constexpr int UN_STAGE = 10240;            // entries staged at a time: 4 + 2 bytes each inside the 64 KB bit buffer

__device__ __forceinline__ uint32_t un_wave_incl_scan(uint32_t v) {
  int x = (int)v;
  x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, false);   // row_shr:1
  x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, false);   // row_shr:2
  x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xf, 0xf, false);   // row_shr:4
  x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xf, 0xf, false);   // row_shr:8
  x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
  x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
  return (uint32_t)x;
}

__global__ void __launch_bounds__(UN_THREADS) union_rows_kernel(const UnionArgs A) {
  __shared__ uint32_t bits[UN_CHUNK / 2];          // row bits of the chunk's tokens, two tokens per word
  __shared__ uint32_t wave_tot[UN_THREADS / 64];
  __shared__ int tgt[STS_MAX_HEADS];               // target heads that read this draft head
  __shared__ int ntgt_s;
  const int j = blockIdx.x, bt = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) {
    int n = 0;
    for (int t = 0; t < A.Hq; ++t)
      if (A.map[t] == j) tgt[n++] = t;
    ntgt_s = n;
  }
  __syncthreads();
  const int ntgt = ntgt_s;
  if (ntgt == 0) return;
  __shared__ int cnts[16];                         // entries of each row's list
  if (tid < 16) cnts[tid] = tid < A.Tq ? (A.row_cnt ? min(max(A.row_cnt[((size_t)bt * A.Hd + j) * A.Tq + tid], 0), A.k) : A.k) : 0;
  __syncthreads();
  const int32_t *lists = A.row_idx + ((size_t)bt * A.Hd + j) * A.Tq * (size_t)A.k;      // [Tq][k]
  const size_t out_row = (size_t)bt * A.Hq;        // outputs of target t: (out_row + t) * pitch
  // Lists as the selection writes them are ascending, so the entries of a chunk are one segment
  // of each list, and reading only that segment per chunk reads every list once instead of once
  // per chunk (at 128K tokens the re-reads were three quarters of this kernel's traffic). The
  // segment ends come from a binary search per (row, chunk end), all at once. Nothing is taken on
  // trust: the segments cover every list completely, and an entry that names a token outside
  // the chunk of the segment it was read in (a list that is not ascending) sets a flag, after which
  // the whole union is built again the plain way, every chunk reading every entry.
  const int nchunks = (A.N + UN_CHUNK - 1) / UN_CHUNK;
  __shared__ int seg[16][UN_MAX_SEG + 1];          // seg[i][c]: first entry of row i at or past chunk c's start
  __shared__ int out_of_place;
  bool by_segments = nchunks > 1 && nchunks <= UN_MAX_SEG;
  if (by_segments) {
    if (tid == 0) out_of_place = 0;
    for (int x = tid; x < 16 * (nchunks + 1); x += UN_THREADS) {
      const int i = x / (nchunks + 1), c = x % (nchunks + 1);
      int lo = 0, hi = cnts[i];                    // lower bound of c * UN_CHUNK in row i
      if (c == 0) hi = 0;
      else if (c == nchunks) lo = hi;
      const int32_t *row = lists + (size_t)i * A.k;
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (row[mid] < c * UN_CHUNK) lo = mid + 1;
        else hi = mid;
      }
      seg[i][c] = lo;
    }
    __syncthreads();
  }
  uint32_t written = 0;                            // union entries before the current chunk
  for (int base = 0; base < A.N; base += UN_CHUNK) {
    for (int i = tid; i < UN_CHUNK / 2; i += UN_THREADS) bits[i] = 0u;
    __syncthreads();
    const int ch = base / UN_CHUNK;
    // one entry of every row per thread and step: up to 16 loads in flight
    int span = A.k;                                // entries per row to look at: the longest segment
    if (by_segments) {
      span = 0;
      for (int i = 0; i < A.Tq; ++i) span = max(span, seg[i][ch + 1] - seg[i][ch]);
    }
    for (int e = tid; e < span; e += UN_THREADS) {
      int n[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int lo = by_segments ? seg[i][ch] : 0, hi = by_segments ? seg[i][ch + 1] : cnts[i];
        n[i] = (i < A.Tq && lo + e < hi) ? lists[(size_t)i * A.k + lo + e] : -1;
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int off = n[i] - base;
        // entries outside the cache (the -1 padding, anything else out of range) name no token
        if (n[i] >= 0 && n[i] < A.N) {
          if (off >= 0 && off < UN_CHUNK) atomicOr(&bits[off >> 1], (1u << i) << (16 * (off & 1)));
          else if (by_segments) out_of_place = 1;
        }
      }
    }
    __syncthreads();
    if (by_segments && out_of_place) {               // uniform: start again, every chunk reading every entry
      by_segments = false;
      written = 0;
      base = -UN_CHUNK;
      continue;
    }
    // thread tid owns tokens base + 32 tid .. + 31 (16 words)
    uint32_t w[16];
    uint32_t kept = 0;
#pragma unroll
    for (int x = 0; x < 16; ++x) {
      w[x] = bits[tid * 16 + x];
      kept += ((w[x] & 0xffffu) ? 1u : 0u) + ((w[x] >> 16) ? 1u : 0u);
    }
    const uint32_t incl = un_wave_incl_scan(kept);
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t before = 0, total = 0;
#pragma unroll
    for (int x = 0; x < UN_THREADS / 64; ++x) {
      const uint32_t v = wave_tot[x];
      if (x < wave) before += v;
      total += v;
    }
    // The chunk's entries, in token order, are staged in the (now free) bit buffer, UN_STAGE at a
    // time, and copied out coalesced to every target head: scattered 4- and 2-byte stores straight
    // from the owning threads were the slowest part of this kernel.
    const uint32_t rel0 = before + incl - kept;       // this thread's first place within the chunk
    int32_t *stg_idx = reinterpret_cast<int32_t *>(bits);
    uint16_t *stg_mask = reinterpret_cast<uint16_t *>(bits + UN_STAGE);
    for (uint32_t r0 = 0; r0 < total; r0 += UN_STAGE) {
      uint32_t rel = rel0;
      if (rel < r0 + UN_STAGE && rel + kept > r0) {
#pragma unroll
        for (int x = 0; x < 16; ++x)
#pragma unroll
          for (int hlf = 0; hlf < 2; ++hlf) {
            const uint32_t m = hlf ? (w[x] >> 16) : (w[x] & 0xffffu);
            if (m) {
              if (rel >= r0 && rel - r0 < (uint32_t)UN_STAGE) {
                stg_idx[rel - r0] = base + tid * 32 + 2 * x + hlf;
                stg_mask[rel - r0] = (uint16_t)m;
              }
              ++rel;
            }
          }
      }
      __syncthreads();
      const uint32_t first = written + r0;             // place of the staged entries in the list
      // a pitch below the union's size truncates the list
      const uint32_t n = first < (uint32_t)A.pitch ? min(min(total - r0, (uint32_t)UN_STAGE), (uint32_t)A.pitch - first) : 0u;
      for (int ti = 0; ti < ntgt; ++ti) {
        const size_t o = (out_row + tgt[ti]) * (size_t)A.pitch + first;
        for (uint32_t p = tid; p < n; p += UN_THREADS) {
          A.indices[o + p] = stg_idx[p];
          A.row_mask[o + p] = stg_mask[p];
        }
      }
      __syncthreads();
    }
    written += total;
    __syncthreads();                                  // bits and wave_tot are rewritten next round
  }
  const uint32_t c = min(written, (uint32_t)A.pitch);
  for (int ti = 0; ti < ntgt; ++ti) {
    const size_t o = (out_row + tgt[ti]) * (size_t)A.pitch;
    for (uint32_t p = c + tid; p < (uint32_t)A.pitch; p += UN_THREADS) {
      A.indices[o + p] = -1;
      A.row_mask[o + p] = 0;
    }
    if (tid == 0 && A.counts) A.counts[out_row + tgt[ti]] = (int32_t)c;
  }
}

}  // namespace

hipError_t launch_union_rows(const UnionArgs &a, hipStream_t s) {
  if ((size_t)a.B * a.Hq == 0) return hipSuccess;
  STS_LAUNCH(union_rows_kernel, dim3(a.Hd, a.B), dim3(UN_THREADS), 0, s, a);
  return sts_take_launch_status();
}
