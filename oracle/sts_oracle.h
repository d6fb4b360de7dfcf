/*
 * sts_oracle.h -- CPU oracle for the STS hot path. TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct implementation of what the GPU library computes:
 * draft-score aggregation, per-head top-k index selection, head remapping, and softmax
 * attention restricted to an index set (with dense attention as the identity index set),
 * plus the offline head-mapping procedure (Algorithm 1 of the paper).
 *
 * Nothing here is shared with the HIP path: no headers, helpers, tables or constants.
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * Every pointer is a HOST pointer. Layouts are row-major, contiguous unless a stride is
 * given. bf16 tensors are passed as their raw 16-bit patterns (uint16_t).
 * Floating point: accumulations are fp64 except oracle_aggregate, whose fp32 left-to-right
 * addition order is part of the selection contract (index sets must be bit-exact).
 *
 * Pins (tests/test_oracle_*.py): O(N^2) counting definition of top-k with ties, closed
 * forms (zero logits => mean of V, one dominant key), mask-restricted full softmax,
 * budget == N equals dense, split/merge invariance, torch.topk value multisets,
 * torch scaled_dot_product_attention, hand-worked Algorithm 1 examples.
 * The paper prints no numeric worked example for any step, so absolute values are pinned
 * by these definitions only.
 *
 * All functions return 0 on success, negative on invalid arguments.
 */
#ifndef STS_ORACLE_H
#define STS_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORACLE_SCORES_PROBS = 0, ORACLE_SCORES_LOGITS_LSE = 1 };
enum { ORACLE_REDUCE_SUM = 0, ORACLE_REDUCE_MAX = 1 };

/* Section 4.3 (one mask per speculative batch): reduce the draft attention weights of the
 * Tq query rows of the speculative block into one score per (batch, draft head, token).
 *   scores [B,Hd,Tq,N] fp32 : probabilities (kind PROBS) or scaled logits (LOGITS_LSE)
 *   lse    [B,Hd,Tq]   fp32 : natural-log normalisers, only read for LOGITS_LSE
 *   A      [B,Hd,N]    fp32 : out
 * SUM adds the Tq rows left to right in fp32 (one rounding per add); MAX takes the maximum.
 * LOGITS_LSE first forms p = expf(s - lse) in fp32. */
int oracle_aggregate(const float *scores, const float *lse, int B, int Hd, int Tq, int N,
                     int kind, int reduce, float *A);

/* Section 4.2 (top-k on each draft head's attention weights): for every (b, j) order the
 * tokens n in [0, N_b) by (A descending, n ascending), keep the first c = min(k, N_b) and
 * emit them in ascending n. -0 equals +0. NaN is rejected (returns -2).
 *   A [B,Hd,N] ; seq_lens [B] or NULL (N_b = N)
 *   sel [B,Hd,k] out, tail padded with -1 ; cnt [B,Hd] out */
int oracle_select(const float *A, int B, int Hd, int N, const int32_t *seq_lens, int k,
                  int32_t *sel, int32_t *cnt);

/* Section 4.2 (top-k over blocks instead of individual tokens) / Section 6.3 (page size p_s):
 * score of block m = A[m*p] + A[m*p+1] + ... over the tokens of the block that lie below the
 * valid length, added left to right in fp32 (the paper does not name the operator; summing
 * keeps "attention mass captured" as the criterion). NB = ceil(N / page) blocks per row.
 *   A [B,Hd,N] ; seq_lens [B] or NULL ; blk [B,Hd,NB] out (blocks past the length get 0) */
int oracle_block_scores(const float *A, int B, int Hd, int N, const int32_t *seq_lens, int page,
                        float *blk);

/* Section 4.2 (remap masks through the offline mapping dictionary):
 *   indices[b,t,:] = sel[b, head_map[t], :], counts[b,t] = cnt[b, head_map[t]]. */
int oracle_remap(const int32_t *sel, const int32_t *cnt, int B, int Hd, int Hq, int k,
                 const int32_t *head_map, int32_t *indices, int32_t *counts);

/* Section 4.2 / Section 2.3 (attend only to the key-value pairs named by the indices, the
 * full cache is kept): for each batch b, query head t, query row i
 *   s_c = scale * sum_e Q[b,i,t,e] K[b,g(t),I_c,e],  p_c = exp(s_c - max s), l = sum p_c
 *   out[b,i,t,:] = sum_c p_c V[b,g(t),I_c,:] / l ,   lse[b,t,i] = max s + ln l
 * with g(t) = t / (Hq/Hkv). indices == NULL means the dense case I = 0..N_b-1.
 *   q [B,Tq,Hq,d] bf16 bits ; k,v bf16 bits with element strides (stride_b,stride_h,stride_n)
 *   indices [B,Hq,kmax] ; counts [B,Hq] or NULL (= kmax) ; seq_lens [B] or NULL (dense only)
 *   out [B,Tq,Hq,d] fp32 ; lse_out [B,Hq,Tq] or NULL ; logits_out [B,Hq,Tq,N] or NULL
 *   (dense only: the scaled logits s_c, the paper's QK^T dump of Section 5).
 * A row with no valid key gives out = 0 and lse = -inf. An index outside [0,N) returns -3.
 * k_new, v_new [B,Tq,Hkv,d] (bf16 bits) or NULL: the keys/values of the speculative block's
 * own Tq tokens, which are not in the cache yet (Section 2.1: the target verifies all
 * candidates in one parallel step, so candidate i also attends to candidates before it).
 * They are appended after the cached keys of every query row: row i sees new tokens 0..i when
 * causal != 0, all Tq otherwise.
 * head_begin/head_end restrict the computed query heads to [head_begin, head_end) and
 * batch_begin/batch_end the batches (other outputs untouched) so callers can sample. */
int oracle_attn(const uint16_t *q, const uint16_t *k, const uint16_t *v, int B, int Tq, int Hq,
                int Hkv, int d, int N, int64_t stride_b, int64_t stride_h, int64_t stride_n,
                const int32_t *indices, const int32_t *counts, int kmax,
                const int32_t *seq_lens, float scale, float *out, float *lse_out,
                float *logits_out, int batch_begin, int batch_end, int head_begin,
                int head_end, const uint16_t *k_new, const uint16_t *v_new, int causal);

/* Algorithm 1 (head mapping construction). Traces are attention-weight rows:
 *   a_d [S,Hd,R,N], a_t [S,Ht,R,N] fp32 (S samples, R query rows each).
 * For each target head the draft head maximising the number of shared top-k indices, the
 * overlap being summed over all rows and samples; the first draft head reaching the
 * maximum wins (strict improvement test). Top-k uses the same tie rule as oracle_select.
 *   map [Ht] out ; overlap [Ht,Hd] out (int64), may be NULL */
int oracle_head_mapping(const float *a_d, const float *a_t, int S, int Hd, int Ht, int R,
                        int N, int k, int32_t *map, int64_t *overlap);

/* Number of OpenMP threads the oracle will use (for reporting). */
int oracle_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif
