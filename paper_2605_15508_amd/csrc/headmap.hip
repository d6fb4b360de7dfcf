// Head-mapping construction (paper Algorithm 1, Section 4.1) on the GPU.
//
// The per-row top-k index sets of both traces come from the selection pipeline (ascending
// lists). This file counts, for every (target head, draft head), the indices the two lists
// share, summed over all rows, and then takes for each target head the first draft head with
// the largest count. All integer work.
#include "common.h"

namespace {

__global__ void __launch_bounds__(256) headmap_clear_kernel(unsigned long long *p, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0ull;
}

// grid (S*R, Ht): one workgroup per (row pair, target head); loops over the draft heads.
// Both lists are ascending, so membership is a binary search in the target list.
__global__ void __launch_bounds__(256) headmap_overlap_kernel(const int32_t *idx_d, const int32_t *idx_t,
                                                              int S, int R, int Hd, int Ht, int k, int c,
                                                              unsigned long long *overlap) {
  __shared__ uint32_t wave_cnt[4];
  const int sr = blockIdx.x, ht = blockIdx.y;
  const int s = sr / R, r = sr - s * R;
  const int32_t *lt = idx_t + (((size_t)s * Ht + ht) * R + r) * k;
  for (int hd = 0; hd < Hd; ++hd) {
    const int32_t *ld = idx_d + (((size_t)s * Hd + hd) * R + r) * k;
    uint32_t cnt = 0;
    for (int i = threadIdx.x; i < c; i += 256) {
      const int32_t x = ld[i];
      int lo = 0, hi = c;                       // first position with lt[pos] >= x
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (lt[mid] < x) lo = mid + 1; else hi = mid;
      }
      cnt += (lo < c && lt[lo] == x) ? 1u : 0u;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) cnt += __shfl_xor(cnt, off, 64);
    if ((threadIdx.x & 63) == 0) wave_cnt[threadIdx.x >> 6] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) {
      const uint32_t tot = wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
      if (tot) atomicAdd(&overlap[(size_t)ht * Hd + hd], (unsigned long long)tot);
    }
    __syncthreads();
  }
}

// one thread per target head: strict improvement over a running maximum that starts below
// zero, so the first best draft head wins and zero overlap maps to draft head 0
__global__ void __launch_bounds__(256) headmap_argmax_kernel(const unsigned long long *overlap, int Hd, int Ht,
                                                             int32_t *map) {
  const int ht = blockIdx.x * 256 + threadIdx.x;
  if (ht >= Ht) return;
  long long best = -1;
  int arg = 0;
  for (int hd = 0; hd < Hd; ++hd) {
    const long long v = (long long)overlap[(size_t)ht * Hd + hd];
    if (v > best) {
      best = v;
      arg = hd;
    }
  }
  map[ht] = arg;
}

}  // namespace

hipError_t launch_headmap_clear(unsigned long long *overlap, int n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  STS_LAUNCH(headmap_clear_kernel, dim3((n + 255) / 256), dim3(256), 0, s, overlap, n);
  return sts_take_launch_status();
}

hipError_t launch_headmap_overlap(const int32_t *idx_d, const int32_t *idx_t, int S, int R, int Hd, int Ht,
                                  int k, int c, unsigned long long *overlap, hipStream_t s) {
  if ((size_t)S * R == 0 || Ht == 0 || c == 0) return hipSuccess;
  STS_LAUNCH(headmap_overlap_kernel, dim3(S * R, Ht), dim3(256), 0, s, idx_d, idx_t, S, R, Hd, Ht, k, c,
                     overlap);
  return sts_take_launch_status();
}

hipError_t launch_headmap_argmax(const unsigned long long *overlap, int Hd, int Ht, int32_t *map, hipStream_t s) {
  if (Ht == 0) return hipSuccess;
  STS_LAUNCH(headmap_argmax_kernel, dim3((Ht + 255) / 256), dim3(256), 0, s, overlap, Hd, Ht, map);
  return sts_take_launch_status();
}
