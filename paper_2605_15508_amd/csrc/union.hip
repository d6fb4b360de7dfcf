// Two-dimensional masks of prefill (paper Section 4.2: during prefill every query token has an
// index set of its own). For a block of up to 16 query rows the attention kernel gathers the
// UNION of the rows' sets once and is told, per gathered token, which rows keep it. This kernel
// builds that form from per-row lists: for every (batch, target head) the ascending union of the
// lists of its draft head's rows, and a 16-bit word per union entry, bit i set iff row i keeps
// the token.
//
// One 1024-thread workgroup per (target head, batch). The token range is walked in chunks of
// 32768 tokens whose row bits sit in LDS (two tokens per word): every list entry that falls into
// the chunk ORs its row's bit into its token's half word; then every thread takes 32 consecutive
// tokens, one block scan gives the kept tokens their places, and they are written in token order.
#include "common.h"

namespace {

constexpr int UN_THREADS = 1024;
constexpr int UN_CHUNK = 32768;            // tokens per LDS pass

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
  const int t = blockIdx.x, bt = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = A.map[t];
  const int32_t *lists = A.row_idx + ((size_t)bt * A.Hd + j) * A.Tq * (size_t)A.k;      // [Tq][k]
  const int32_t *lcnt = A.row_cnt ? A.row_cnt + ((size_t)bt * A.Hd + j) * A.Tq : nullptr;
  int32_t *out_idx = A.indices + ((size_t)bt * A.Hq + t) * (size_t)A.pitch;
  uint16_t *out_mask = A.row_mask + ((size_t)bt * A.Hq + t) * (size_t)A.pitch;
  uint32_t written = 0;                            // union entries before the current chunk
  for (int base = 0; base < A.N; base += UN_CHUNK) {
    for (int i = tid; i < UN_CHUNK / 2; i += UN_THREADS) bits[i] = 0u;
    __syncthreads();
    for (int i = 0; i < A.Tq; ++i) {
      const int c = lcnt ? min(max(lcnt[i], 0), A.k) : A.k;
      const int32_t *row = lists + (size_t)i * A.k;
      for (int e = tid; e < c; e += UN_THREADS) {
        const int n = row[e];
        const int off = n - base;
        // entries outside the cache (the -1 padding, anything else out of range) name no token
        if (n >= 0 && n < A.N && off >= 0 && off < UN_CHUNK) atomicOr(&bits[off >> 1], (1u << i) << (16 * (off & 1)));
      }
    }
    __syncthreads();
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
    uint32_t pos = written + before + incl - kept;
#pragma unroll
    for (int x = 0; x < 16; ++x)
#pragma unroll
      for (int hlf = 0; hlf < 2; ++hlf) {
        const uint32_t m = hlf ? (w[x] >> 16) : (w[x] & 0xffffu);
        if (m) {
          if (pos < (uint32_t)A.pitch) {             // a pitch below the union's size truncates the list
            out_idx[pos] = base + tid * 32 + 2 * x + hlf;
            out_mask[pos] = (uint16_t)m;
          }
          ++pos;
        }
      }
    written += total;
    __syncthreads();                                  // bits and wave_tot are rewritten next round
  }
  const uint32_t c = min(written, (uint32_t)A.pitch);
  for (uint32_t p = c + tid; p < (uint32_t)A.pitch; p += UN_THREADS) {
    out_idx[p] = -1;
    out_mask[p] = 0;
  }
  if (tid == 0 && A.counts) A.counts[(size_t)bt * A.Hq + t] = (int32_t)c;
}

}  // namespace

hipError_t launch_union_rows(const UnionArgs &a, hipStream_t s) {
  if ((size_t)a.B * a.Hq == 0) return hipSuccess;
  STS_LAUNCH(union_rows_kernel, dim3(a.Hq, a.B), dim3(UN_THREADS), 0, s, a);
  return sts_take_launch_status();
}
