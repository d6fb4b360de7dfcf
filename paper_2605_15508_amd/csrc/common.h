// Shared declarations of the STS HIP library (gfx950 only). Internal: the public surface is
// include/sts.h.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <tuple>
#include <type_traits>
#include <utility>

#include "../../include/sts.h"

// Every kernel goes out through STS_LAUNCH. With the library's timing aid switched on, the host
// code sets this pair of events before a launch and the dispatch itself stamps them with the
// kernel's own begin and end times (no extra packets around it); otherwise it is an ordinary
// launch. The status is the launch call's own return value (an error that some earlier, unrelated
// HIP call of the process left behind is neither reported as ours nor cleared); a launcher hands
// it back with sts_take_launch_status().
struct StsLaunchEvents { hipEvent_t start, stop; };
extern thread_local StsLaunchEvents g_sts_launch_events;
extern thread_local hipError_t g_sts_launch_rc;

template <class Tuple, size_t... I>
inline void sts_arg_pointers(Tuple &vals, void **ptrs, std::index_sequence<I...>) {
  ((ptrs[I] = static_cast<void *>(&std::get<I>(vals))), ...);
}

template <class... P, class... A>
inline void sts_launch(void (*kernel)(P...), dim3 grid, dim3 block, unsigned shmem, hipStream_t stream, const A &...args) {
  std::tuple<std::remove_cv_t<P>...> vals(args...);      // copies of the kernel's own parameter types
  void *ptrs[sizeof...(P)];
  sts_arg_pointers(vals, ptrs, std::index_sequence_for<P...>{});
  const hipError_t rc =
      g_sts_launch_events.start
          ? hipExtLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, ptrs, shmem, stream,
                               g_sts_launch_events.start, g_sts_launch_events.stop, 0)
          : hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, ptrs, shmem, stream);
  if (g_sts_launch_rc == hipSuccess) g_sts_launch_rc = rc;
}
#define STS_LAUNCH(kernel, grid, block, shmem, stream, ...) sts_launch(kernel, grid, block, shmem, stream, __VA_ARGS__)

// status of the launches since the last call of this function (the first failure, if any)
inline hipError_t sts_take_launch_status() {
  const hipError_t rc = g_sts_launch_rc;
  g_sts_launch_rc = hipSuccess;
  return rc;
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int STS_MAX_HEADS = 256;   // Hq, Hd upper bound (tables travel as kernel arguments)
constexpr int STS_MAX_GROUP = 16;    // query heads per KV head
constexpr int STS_TILE_KEYS = 32;    // keys per wave tile
constexpr int STS_WG_WAVES = 4;      // waves per attention workgroup

// A work unit of the attention kernels: the query heads of one KV group that share one index
// row (sparse) or all heads of the group (dense). Packed: bits 0-7 KV head, 8-23 mask of the
// member heads within the group, 24-28 number of member heads.
struct AttnUnitTable {
  uint32_t unit[STS_MAX_HEADS];
};

struct AttnArgs {
  const uint16_t *q, *k, *v;
  const int32_t *indices, *counts, *seq_lens;
  const uint16_t *row_mask;               // [B,Hq,kmax] laid out like indices: bit i = query row i keeps the entry; or NULL
  int64_t stride_b, stride_h, stride_n;   // elements
  int64_t idx_stride_b, cnt_stride_b;     // elements between batches of indices / counts
  int32_t B, Tq, Hq, Hkv, G, N, kmax;
  int32_t num_units, num_splits;
  int32_t page, page_shift;               // tokens per index entry / page (power of two <= 32)
  const int32_t *block_table;             // [B, table_stride] logical block -> physical page, or NULL
  int32_t table_stride, num_pages;
  int64_t stride_page;                    // elements between pages of the pool
  const uint16_t *k_new, *v_new;          // [B,Tq,Hkv,d] the block's own keys/values, or NULL
  int32_t causal;
  int32_t direct;                         // single split: the split kernel writes the result itself
  float scale_log2;                       // scale * log2(e)
  float scale;
  float *part_o;                          // [B*U*S][NQ*16][D]
  float *part_ml;                         // [B*U*S][NQ*16][2]  (max in log2 domain, sum)
  void *logits_out;
  int32_t logits_bf16;
  float *agg_out;                         // [B,Hq,N] summed attention weights of the query block (dense only), or NULL
  int32_t ps_heads, ps_sets, ps_splits;   // second pass: heads per workgroup, such sets per KV head, key-range splits
  int32_t ps_tp;                          // second pass: rows per head, Tq rounded up to a power of two
  void *out;
  float *lse_out;
  int32_t out_dtype;
  AttnUnitTable units;
};

struct AttnPlan {
  int32_t nq;          // query tiles of 16 rows per unit (1, 2 or 4)
  int32_t num_units;   // per batch element
  int32_t num_splits;
  size_t part_o_bytes, part_ml_bytes, lse_bytes;
  AttnUnitTable units;
};

// select ------------------------------------------------------------------------------------

constexpr int SEL_BITS0 = 11, SEL_BITS1 = 11, SEL_BITS2 = 10;
constexpr int SEL_BINS = 2048;          // bins of the widest digit
constexpr int SEL_CHUNK = 8192;         // tokens per workgroup in the scan kernels
constexpr int SEL_THREADS = 256;
constexpr int SEL_SMALL_N = 32768;      // LDS capacity of the one-workgroup-per-row selection (tokens)
constexpr int SEL_FLAG_PITCH = 32;      // words between the published counts of two chunks: one 128-byte line each
constexpr int SEL_FUSED_N = 8192;
constexpr int SEL_FUSED_MAX_PARTS = 8;   // parts per row of the one-launch selection: every part reads every other
                                         // part's histograms, which grows with the square (256K tokens; a test knob
                                         // allows up to 256)
constexpr int SEL_POOL_MAX = 16384;     // chunk-local winners per row that the pool kernel ranks out of LDS       // rows up to this many tokens always take it

// One workgroup per row, one pass (select_band_kernel): what the strided sample of a row of nb
// ranked tokens with budget c looks like, and whether the band it is expected to give fits the
// workgroup's store. The kernel decides per row with this; the host asks the same question for
// a full-length row when it chooses the path.
constexpr int BAND_CAP = 8192;          // band entries (key and token) a workgroup holds; it samples up to twice as many keys
constexpr int BAND_MAX_N = 524288;      // tokens per row: one bit each in LDS
constexpr int BAND_Z = 5;               // half-width of the band in standard deviations of the sample count
struct BandPlan {
  int S;                // one run of `run` tokens is sampled in every S runs
  int runs, ns;         // sampled runs and tokens (the last run may be cut by the row's end)
  long long s_hi, s_lo; // sample ranks that give the band's upper and lower edge (s_hi < 1: no upper edge)
  bool fits;
};
__host__ __device__ inline BandPlan band_plan(int nb, uint32_t c, int run) {
  BandPlan p;
  const int row_runs = (nb + run - 1) / run;
  p.S = 16;
  while (((row_runs + p.S - 1) / p.S) * run > 2 * BAND_CAP) p.S <<= 1;
  p.runs = (row_runs + p.S - 1) / p.S;              // sampled run i starts at token i * S * run
  const int last = nb - (p.runs - 1) * p.S * run;
  p.ns = (p.runs - 1) * run + (last < run ? last : run);
  const uint32_t cs = c / (uint32_t)p.S;
  uint32_t sq = (uint32_t)sqrtf((float)cs);
  while ((uint64_t)sq * sq > cs) --sq;
  while ((uint64_t)(sq + 1) * (sq + 1) <= cs) ++sq;
  ++sq;                                   // > sqrt(cs): one standard deviation of the sample count, rounded up
  p.s_hi = (long long)cs - (long long)BAND_Z * sq - 2;
  p.s_lo = (long long)cs + (long long)BAND_Z * sq + 3;
  const long long expect = (long long)p.S * (p.s_lo - (p.s_hi >= 1 ? p.s_hi : 0));
  p.fits = nb > 0 && p.s_lo <= p.ns && expect <= BAND_CAP - BAND_CAP / 8;
  return p;
}

struct SelectTargets {
  // targets of draft head j: tgt[off[j] .. off[j+1])
  uint16_t off[STS_MAX_HEADS + 1];
  uint8_t tgt[STS_MAX_HEADS];
};

struct SelectArgs {
  const void *scores;         // fp32 or bf16 (scores_bf16)
  const float *lse;
  int32_t scores_bf16;
  const int32_t *seq_lens;
  int32_t *indices, *counts;
  float *agg;                 // [B,Hd,N] (agg_out or workspace)
  float *blk;                 // [B,Hd,NB] per-block sums (page > 1), else unused
  const float *src;           // what is ranked: agg (page == 1) or blk
  int32_t srcN;               // row length of src: N or NB
  int32_t page;               // tokens per block (>= 1)
  uint32_t *hist;             // [rows][3][SEL_BINS]
  uint32_t *state;            // [rows][8]: digits 0/1 and remaining k after each, [6] budget
  uint32_t *chunk_cnt;        // [rows][nchunks][SEL_FLAG_PITCH], word 0: published flag | equal count << 14 | greater count
  uint32_t *pool_key;         // [rows][pool_nchunks * pool_pitch] chunk-local winners (small budgets), token
                              // order, contiguous per row: chunk c starts at c * min(budget of the row, pool_chunk)
  int32_t *pool_idx;          // their token ids
  int32_t pool_chunk;         // tokens per chunk of the local kernel: 8192 or 32768
  int32_t pool_nchunks;       // ceil(N / pool_chunk)
  int32_t pool_pitch;         // min(k, pool_chunk)
  uint64_t clear_words;       // words to zero from `hist` on: histograms, state and chunk flags
  int32_t hist_cpw;           // consecutive chunks per workgroup of the refinement histograms (1, 2 or 4)
  int32_t spin_limit;         // polls of an unpublished earlier chunk before it is recounted locally
  unsigned long long *pub;    // fused selection: [rows][3][parts][1024] words the parts publish (top bit: written;
                              // two bin counts in the halves), zero before the launch
  int32_t part_tokens, parts; // fused selection: tokens per part (8192..32768) and parts per row
  int32_t fused_spin_limit;   // polls of another part's flag before its histogram is recomputed locally
  int32_t rowpass_threads;    // one workgroup per row (select_rowpass_kernel): 256 or 1024 threads
  int32_t agg_is_input;       // `agg` is the caller's score tensor itself (one fp32 probability row per head): never stored to
  int32_t B, Hd, Tq, N, Hq, k, kind, reduce, nchunks;   // k: row pitch of indices = largest budget
  SelectTargets targets;
  int32_t kh[STS_MAX_HEADS];  // budget of draft head j (<= k)
};

// union of per-row index lists (union.hip)
struct UnionArgs {
  const int32_t *row_idx;     // [B,Hd,Tq,k]
  const int32_t *row_cnt;     // [B,Hd,Tq] or nullptr (= k)
  int32_t *indices;           // [B,Hq,pitch]
  uint16_t *row_mask;         // [B,Hq,pitch]
  int32_t *counts;            // [B,Hq] or nullptr
  int32_t B, Hd, Hq, Tq, N, k, pitch;
  uint8_t map[STS_MAX_HEADS]; // target head -> draft head
};
hipError_t launch_union_rows(const UnionArgs &a, hipStream_t s);

// device address of the current device's copy of the static scratch array (scratch.hip)
sts_status sts_static_scratch(void **out);

// launches (defined in the .hip files); each returns the status of its own launch call
hipError_t launch_attn_split(const AttnArgs &a, int d, int nq, bool sparse, hipStream_t s);
hipError_t launch_attn_combine(const AttnArgs &a, int d, int nq, hipStream_t s);
hipError_t launch_attn_probsum(const AttnArgs &a, int d, int nq, hipStream_t s);
int attn_probsum_wgs_per_cu(int d, int nq);
hipError_t launch_select_clear(const SelectArgs &a, hipStream_t s);
hipError_t launch_select_agg(const SelectArgs &a, hipStream_t s);
hipError_t launch_select_block(const SelectArgs &a, hipStream_t s);
hipError_t launch_select_small(const SelectArgs &a, hipStream_t s);
hipError_t launch_select_rank(const SelectArgs &a, hipStream_t s);
bool select_aggblock_ok(const SelectArgs &a);
hipError_t launch_select_aggblock(const SelectArgs &a, hipStream_t s);
hipError_t launch_select_fused(const SelectArgs &a, hipStream_t s);
hipError_t launch_select_clear_pub(const SelectArgs &a, hipStream_t s);
bool select_band_ok(const SelectArgs &a);
hipError_t launch_select_band(const SelectArgs &a, hipStream_t s);
bool select_rowpass_ok(const SelectArgs &a);
hipError_t launch_select_rowpass(const SelectArgs &a, hipStream_t s);
hipError_t launch_select_local(const SelectArgs &a, hipStream_t s);
hipError_t launch_select_pool(const SelectArgs &a, hipStream_t s);
hipError_t launch_select_hist(const SelectArgs &a, int pass, hipStream_t s);
hipError_t launch_select_write(const SelectArgs &a, hipStream_t s);
hipError_t launch_headmap_clear(unsigned long long *overlap, int n, hipStream_t s);
hipError_t launch_headmap_overlap(const int32_t *idx_d, const int32_t *idx_t, int S, int R, int Hd, int Ht,
                                  int k, int c, unsigned long long *overlap, hipStream_t s);
hipError_t launch_headmap_argmax(const unsigned long long *overlap, int Hd, int Ht, int32_t *map, hipStream_t s);
