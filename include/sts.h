/*
 * sts.h -- C ABI of the MI355X (gfx950) library for the hot path of STS, Speculative Token
 * Sparsity: draft attention scores -> per-target-head top-k index sets -> verification
 * attention over the gathered rows of a full, never-pruned KV cache.
 *
 * Conventions
 *  - C11, no C++ types cross the ABI. Pointers marked [dev] are DEVICE pointers owned by the
 *    caller (e.g. torch allocations); pointers marked [host] are HOST pointers read during
 *    the call and not retained.
 *  - The entry points never allocate, free or synchronise: each call validates its arguments
 *    on the host and enqueues kernels on `stream` (a hipStream_t passed as void*, NULL = the
 *    default stream). Scratch memory comes from the caller as `workspace`; query its size
 *    with the *_workspace_bytes functions (the size depends only on the integer shape
 *    fields, `sparse`/flags and pointer NULL-ness, never on device data).
 *  - Inputs are never written. Outputs and workspace must not alias inputs or each other.
 *    Calls that share a workspace or an output buffer must be ordered by the caller (same
 *    stream, or events between streams): the library holds no state and takes no locks.
 *  - Return value: STS_OK (0) or a negative sts_status. On error nothing has been enqueued
 *    (except STS_EHIP, a failed launch, after which earlier kernels of the call may have
 *    been enqueued and the outputs are undefined). STS_EHIP reports the launch calls' own
 *    return values: an error left behind by an unrelated HIP call of the process is neither
 *    reported nor cleared. No exceptions, no errno, no logging.
 *  - Results are deterministic run to run: the split count depends only on the shape and the
 *    partial results are combined in a fixed order; selection uses integer arithmetic only.
 *  - bf16 tensors are raw 16-bit patterns. All accumulation is fp32.
 *  - No environment variable is read on the call path; tuning and test knobs are set with
 *    sts_set_knob (below).
 */
#ifndef STS_H
#define STS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  STS_OK = 0,
  STS_EINVAL = -1,       /* NULL where data is required, negative size, bad enum, bad head map */
  STS_EUNSUPPORTED = -2, /* shape outside what the kernels cover (see each call) */
  STS_EWORKSPACE = -3,   /* workspace NULL or smaller than *_workspace_bytes */
  STS_EHIP = -4          /* the HIP runtime reported an error at launch */
} sts_status;

typedef enum { STS_SCORES_PROBS = 0, STS_SCORES_LOGITS_LSE = 1 } sts_score_kind;
typedef enum { STS_REDUCE_SUM = 0, STS_REDUCE_MAX = 1 } sts_reduce;
typedef enum { STS_BF16 = 0, STS_F32 = 1 } sts_dtype;

/* ----------------------------------------------------------------------------------------
 * sts_select -- online mask generation (paper Section 4.2: top-k over each draft head's
 * attention weights, remapped to the target heads through the offline head-mapping
 * dictionary of Section 4.1; Section 4.3: one mask per speculative batch).
 *
 * For every batch b and draft head j the draft attention weights of the Tq query rows of
 * the speculative block are reduced to one score per cached token,
 *     A[b,j,n] = ((P[b,j,0,n] + P[b,j,1,n]) + P[b,j,2,n]) + ...   (fp32, left to right)
 * (or their maximum), the c = min(k, N_b) tokens with the largest A are kept, ties going to
 * the lower token index, and written in ascending token order to every target head t with
 * head_map[t] == j. With kind == STS_SCORES_LOGITS_LSE the input holds scaled logits s and
 * P = exp(s - lse[b,j,i]) is formed on the fly. -0 and +0 compare equal. NaN scores are a
 * caller error (they are ordered above +inf, deterministically, but that order is not part
 * of the contract).
 *
 * Block granularity (paper Section 4.2: top-k over blocks instead of tokens; Section 6.3:
 * page size p_s). With page_size = p > 1 the aggregated scores of the tokens of block m,
 * A[m*p] + A[m*p+1] + ... (fp32, left to right, tokens below N_b only), rank the
 * ceil(N_b / p) blocks; k then counts blocks and `indices` holds ascending block ids.
 * agg_out stays per token.
 *
 * Score precision (paper Section 5: the draft's attention kernel dumps the query-key products
 * to global memory; the paper does not say in which type). The scores are fp32, or, with
 * scores_bf16, bf16: every value is widened exactly and everything after that is the same
 * fp32 arithmetic, so the result equals that of the call on the widened tensor. lse stays fp32.
 *
 * Per-head budgets (paper Section 6.4: how much can be pruned differs strongly between
 * layers, so budgets are set per layer; the same holds per head). The budget of a layer is
 * simply the k of that layer's call. With k_head != NULL draft head j keeps
 * c = min(k_head[j], N_b) entries instead; k stays the row pitch of `indices` and the upper
 * bound of every k_head[j]. Rows are padded with -1 from c on, counts hold c, so the lists
 * feed sts_sparse_attn unchanged (kmax = k, counts given).
 *
 * The Hq target heads need not belong to one layer: every target head of any layer that maps
 * to these draft heads can be listed (up to 256), the scores are then aggregated and ranked
 * once per draft head, and each layer's sts_sparse_attn reads its heads' slice of `indices`
 * in place (idx_stride_b / cnt_stride_b there).
 *
 * A ready-made aggregate (one fp32 probability row per draft head: Tq = 1, kind PROBS, e.g.
 * sts_dense_attn's weights_sum_out) is ranked where it lies when agg_out is NULL: no copy into
 * the workspace is made, and the tensor is only read.
 *
 * Supported: 1 <= Tq <= 64, 1 <= Hq <= 256, 1 <= Hd <= 256, N < 2^31 - 2^16,
 * page_size <= 4096. Rows of size zero are handled (nothing is read; counts are 0).
 */
typedef struct {
  int32_t B, Hd, Tq, N, Hq;
  int32_t k;                /* token budget per head, >= 1; k >= N_b selects everything */
  const void *scores;       /* [dev] [B,Hd,Tq,N] contiguous, fp32 (or bf16, see scores_bf16):
                               probabilities or scaled logits */
  const float *lse;         /* [dev] [B,Hd,Tq] natural-log normalisers; LOGITS_LSE only, else NULL */
  const int32_t *head_map;  /* [host] [Hq] target head -> draft head, values in [0,Hd) */
  const int32_t *seq_lens;  /* [dev] [B] valid lengths N_b <= N, or NULL (N_b = N) */
  int32_t *indices;         /* [dev] out [B,Hq,k] ascending token ids; positions >= c hold -1 */
  int32_t *counts;          /* [dev] out [B,Hq] c = min(k, N_b); may be NULL */
  float *agg_out;           /* [dev] out [B,Hd,N] the aggregated scores A, 0 at n >= N_b; may be NULL */
  int32_t kind;             /* sts_score_kind */
  int32_t reduce;           /* sts_reduce */
  int32_t page_size;        /* 0 or 1: token granularity. p > 1: block granularity (see above) */
  const int32_t *k_head;    /* [host] optional [Hd]: budget of draft head j, 1 <= k_head[j] <= k
                               (see above); NULL = k for every head */
  int32_t scores_bf16;      /* 0: scores are fp32. Non-zero: scores are bf16 bit patterns, widened
                               exactly to fp32 before any arithmetic (half the bytes to read) */
  void *workspace;          /* [dev] 256-byte aligned scratch */
  size_t workspace_bytes;
} sts_select_params;

/* ----------------------------------------------------------------------------------------
 * sts_sparse_attn -- sparse verification attention (paper Section 4.2: the target's
 * attention layers attend only to the key-value pairs named by the provided indices;
 * Section 2.3: the full cache is kept; Section 5: per-head KV sets, split-K).
 * sts_dense_attn -- the same kernel family over all N_b cached tokens (the dense baseline
 * of Section 6.1, and the draft-side attention that also dumps QK^T, Section 5).
 *
 * For each batch b, query head t (KV head g = t / (Hq/Hkv)) and query row i:
 *     s_c = scale * <Q[b,i,t,:], K[b,g,I_c,:]>,   p_c = exp(s_c - max_c s_c),
 *     out[b,i,t,:] = sum_c p_c V[b,g,I_c,:] / sum_c p_c,   lse[b,t,i] = max_c s_c + ln sum_c p_c
 * where I = indices[b,t,0:counts[b,t]] (sparse) or 0..N_b-1 (dense). The N cached tokens
 * are the prefix before the speculative block, so every query row sees all of them; the
 * block's own causal part is merged by the caller using lse_out. A row with no key gives
 * out = 0 and lse = -inf. Index values must lie in [0,N); they are clamped into range for
 * memory safety, never checked. A repeated index is counted once per occurrence.
 *
 * Block granularity and paged caches (paper Section 5: sparsity at block granularity over
 * KV blocks scattered in memory; Section 6.3: page size p_s). With page_size = p in
 * {2,4,8,16,32} an index entry m stands for the tokens m*p .. min((m+1)*p, N)-1, in order,
 * and counts/kmax count entries. With block_table != NULL the cache is a pool of pages of
 * p tokens shared by the batch: token n of batch b lives in page block_table[b, n / p] at
 * slot n % p, i.e. at element offset page*kv_stride_page + g*kv_stride_h + (n % p)*kv_stride_n
 * of k and v (kv_stride_b is ignored). N stays the logical length bound; table entries are
 * clamped into [0, num_pages) for memory safety. Both options apply to sparse and dense.
 *
 * The speculative block's own tokens (paper Section 2.1: the target checks all candidates in
 * one parallel step, so candidate i also attends to the candidates before it). Their keys and
 * values are not in the cache yet; pass them as k_new / v_new and they are appended after the
 * cached keys of every query row (causally when `causal` is set) in the final merge of the call, so
 * out and lse_out cover the whole verification attention. Without them the caller merges that
 * part itself using lse_out.
 *
 * An index set per query row (paper Section 4.2: during prefill the sparsity pattern is
 * two-dimensional, every query token of a head has a mask of its own). With row_mask the call
 * gathers each entry of `indices` once for the whole block of up to 16 query rows and row i
 * attends only to the entries whose word has bit i set: `indices` holds the union of the rows'
 * sets (sts_union_rows builds both from per-row lists). A row that keeps nothing gives out = 0 and
 * lse = -inf. Contiguous or strided caches, any page_size; not with block_table.
 *
 * Summed attention weights (paper Section 4.3: one mask per speculative batch, from the draft's
 * attention over the whole query block; Section 5: the draft layer hands its scores to the
 * selection). With weights_sum_out the dense call makes a second pass over K once the row
 * normalisers are known and writes A[b,t,n] = sum_i exp(s[i,n] - lse[i]) -- bit for bit what
 * logits_out + lse_out fed to sts_select (kind LOGITS_LSE, reduce SUM) aggregate to -- so the
 * Tq times larger logits never reach memory. Feed it to sts_select as kind PROBS with Tq = 1.
 * Contiguous caches only (no block_table, kv_stride_n <= 2^26), without k_new.
 *
 * Supported: d in {64,128}; Hq % Hkv == 0; Hq/Hkv <= 16; 1 <= Tq <= 16; Hq <= 256;
 * kv strides with kv_stride_n*2 bytes a multiple of 16 and bases 16-byte aligned.
 */
typedef struct {
  int32_t B, Tq, Hq, Hkv, d, N;
  const void *q;            /* [dev] bf16 [B,Tq,Hq,d] contiguous */
  const void *k, *v;        /* [dev] bf16 [B,Hkv,N,d], element strides below, unit stride on d */
  int64_t kv_stride_b, kv_stride_h, kv_stride_n;   /* in elements, shared by k and v */
  const int32_t *indices;   /* [dev] [B,Hq,kmax] (sparse); must be NULL for dense */
  const int32_t *counts;    /* [dev] [B,Hq] valid entries per row, or NULL (= kmax) */
  int32_t kmax;
  const int32_t *head_map;  /* [host] optional hint [Hq]: heads of one KV group with equal
                               values have identical index rows and are processed together
                               over one gathered tile. NULL = every head on its own. */
  const int32_t *seq_lens;  /* [dev] [B] (dense only) or NULL */
  float scale;              /* usually 1/sqrt(d) */
  void *out;                /* [dev] [B,Tq,Hq,d] of out_dtype */
  int32_t out_dtype;        /* sts_dtype */
  float *lse_out;           /* [dev] optional [B,Hq,Tq], natural log */
  void *logits_out;         /* [dev] dense only, optional [B,Hq,Tq,N] scaled logits s_c, fp32 or
                               (logits_bf16) rounded to nearest-even bf16 */
  int32_t page_size;        /* 0 or 1: entries are tokens; else tokens per entry / per page */
  const int32_t *block_table; /* [dev] [B, table_stride] logical block -> physical page, or NULL */
  int32_t table_stride;     /* entries per batch row of block_table, >= ceil(N / page_size) */
  int32_t num_pages;        /* pages in the pool (paged only) */
  int64_t kv_stride_page;   /* elements between consecutive pages of the pool (paged only) */
  const void *k_new, *v_new; /* [dev] optional bf16 [B,Tq,Hkv,d] contiguous: see below; both or neither */
  int32_t causal;           /* with k_new: non-zero = query row i sees new tokens 0..i, zero = all Tq */
  int32_t logits_bf16;      /* type of logits_out: 0 fp32, non-zero bf16 (feeds sts_select's scores_bf16) */
  int64_t idx_stride_b;     /* elements between the batches of `indices`; 0 = Hq*kmax (contiguous). Lets a
                               call read its heads out of a wider list, e.g. the layer slice
                               [:, l*Hq:(l+1)*Hq, :] of one sts_select over the target heads of several
                               layers that share draft heads (the aggregation is then paid once) */
  int64_t cnt_stride_b;     /* same for `counts`; 0 = Hq */
  float *weights_sum_out;   /* [dev] dense only, optional [B,Hq,N] fp32: the attention weights summed over
                               the Tq query rows, sum_i exp(s[i,n] - lse[i]), rows added in order; 0 at
                               n >= N_b (see below) */
  const uint16_t *row_mask; /* [dev] sparse only, optional, laid out like `indices` ([B,Hq,kmax], the same
                               batch stride): bit i of an entry's word set iff query row i keeps the entry
                               (see above); NULL = every row keeps every entry */
  void *workspace;          /* [dev] 256-byte aligned scratch */
  size_t workspace_bytes;
} sts_attn_params;

/* ----------------------------------------------------------------------------------------
 * sts_head_map -- offline head-mapping construction (paper Algorithm 1, Section 4.1).
 *
 * Traces are attention-weight rows of both models over the same inputs: a_d [S,Hd,R,N] and
 * a_t [S,Ht,R,N] (S samples, R query rows per sample, N keys). For every target head the
 * draft head whose top-k index sets share the most indices with the target head's, the
 * overlap being summed over all S*R rows; a later draft head must beat the running maximum
 * strictly, so the first draft head reaching the maximum wins, and a target head with no
 * overlap at all maps to draft head 0. Top-k uses sts_select's order (ties to the lower
 * index). One map per k. Not on the serving path: it runs once, offline.
 *
 * Supported: N < 2^31 - 2^16, 1 <= Hd, Ht; S*R*max(Hd,Ht) rows are processed in slices.
 */
typedef struct {
  int32_t S, R, Hd, Ht, N;
  int32_t k;                /* top-k size, >= 1 (k >= N keeps every index) */
  const float *a_d;         /* [dev] [S,Hd,R,N] fp32 contiguous */
  const float *a_t;         /* [dev] [S,Ht,R,N] fp32 contiguous */
  int32_t *map;             /* [dev] out [Ht] target head -> draft head */
  unsigned long long *overlap; /* [dev] out [Ht,Hd] summed intersection sizes; may be NULL */
  void *workspace;          /* [dev] 256-byte aligned scratch */
  size_t workspace_bytes;
} sts_headmap_params;

/* ----------------------------------------------------------------------------------------
 * sts_union_rows -- two-dimensional masks for a block of query rows (paper Section 4.2: during
 * prefill each query token has its own mask). Per-row index lists, one per (batch, draft head,
 * query row) -- e.g. sts_select on the score tensor viewed as [B, Hd*Tq, 1, N] with the identity
 * head map, whose output is [B, Hd, Tq, k] -- become, for every target head t, the ascending union
 * of the lists of the rows of draft head head_map[t], and one 16-bit word per union entry whose
 * bit i is set iff row i keeps the token: the form sts_sparse_attn reads with row_mask, gathering
 * every token once for the whole block.
 * A row's valid entries are its first row_counts[b,j,i] ones (any order; values outside [0,N),
 * such as the -1 padding, name no token). The outputs have `pitch` entries per (batch, target
 * head): a union longer than that is truncated to its first `pitch` tokens (counts then equal
 * pitch; pitch >= min(Tq*k, N) never truncates); the tail is padded with -1 / 0.
 * Supported: 1 <= Tq <= 16, Hq, Hd <= 256. No workspace.
 */
typedef struct {
  int32_t B, Hd, Hq, Tq, N;
  int32_t k;                   /* pitch of the per-row lists */
  const int32_t *row_indices;  /* [dev] [B,Hd,Tq,k] */
  const int32_t *row_counts;   /* [dev] [B,Hd,Tq] valid entries per row, or NULL (= k) */
  const int32_t *head_map;     /* [host] [Hq] target head -> draft head */
  int32_t pitch;               /* entries per (batch, target head) of the outputs */
  int32_t *indices;            /* [dev] out [B,Hq,pitch] ascending union, -1 padded */
  uint16_t *row_mask;          /* [dev] out [B,Hq,pitch] */
  int32_t *counts;             /* [dev] out [B,Hq] union sizes; may be NULL */
} sts_union_params;

sts_status sts_union_rows(const sts_union_params *p, void *stream);

size_t sts_headmap_workspace_bytes(const sts_headmap_params *p);
sts_status sts_head_map(const sts_headmap_params *p, void *stream);

size_t sts_select_workspace_bytes(const sts_select_params *p);
size_t sts_attn_workspace_bytes(const sts_attn_params *p, int sparse);

sts_status sts_select(const sts_select_params *p, void *stream);
sts_status sts_sparse_attn(const sts_attn_params *p, void *stream);
sts_status sts_dense_attn(const sts_attn_params *p, void *stream);

/* ----------------------------------------------------------------------------------------
 * sts_sparse_attn_static -- sts_sparse_attn for callers that cannot allocate device memory or
 * carry a workspace around: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc. Same arguments, same kernels, same results as sts_sparse_attn (bit for bit),
 * except that p->workspace and p->workspace_bytes are ignored: the per-split partial results go
 * to an array of STS_STATIC_SCRATCH_BYTES that the library's code object holds in device memory
 * (each GPU the library runs on holds its own copy until the process ends). The call allocates
 * and frees nothing and keeps the timing aid below switched off for its launches.
 *  - A shape whose partials need more than STS_STATIC_SCRATCH_BYTES (what
 *    sts_attn_workspace_bytes(p, 1) returns) is refused with STS_EWORKSPACE, nothing enqueued.
 *  - The current device must be the device of `stream`. The first call on a device asks the
 *    runtime for that device's copy of the array; STS_EHIP if that fails.
 *  - Every call on a GPU shares that GPU's array, which keeps the last call's contents. Nothing
 *    in it has to start at zero (every workgroup writes its partial before the combine step
 *    reads it), but two calls that overlap on one GPU (different streams with no event between
 *    them) race on it: order them, or use sts_sparse_attn with a workspace per stream.
 */
#define STS_STATIC_SCRATCH_BYTES ((size_t)8 << 20)
sts_status sts_sparse_attn_static(const sts_attn_params *p, void *stream);

const char *sts_strerror(int status);   /* any int: values that are no sts_status give "unknown status" */
int sts_version(void);

/* ----------------------------------------------------------------------------------------
 * Measurement aid (not on the hot path): when enabled, every kernel launch of the calls
 * above carries a pair of HIP events that its dispatch on the call's stream stamps with the
 * kernel's own begin and end times. sts_prof_read synchronises those
 * events and returns, per kernel kind, the number of launches and their summed duration
 * since the last sts_prof_reset. Enabling allocates events lazily; at most STS_PROF_MAX
 * launches are kept per reset, later ones are not recorded. Keep it switched off while a
 * stream is being captured into a graph (the stamped launch is not a capturable node).
 */
typedef enum {
  STS_K_SELECT_CLEAR = 0,  /* zero histograms */
  STS_K_SELECT_AGG = 1,    /* aggregation + first-digit histogram */
  STS_K_SELECT_HIST = 2,   /* refinement histograms */
  STS_K_SELECT_ROWPASS = 3,/* many long rows of ready-made scores: one workgroup per row, several passes */
  STS_K_SELECT_WRITE = 4,  /* per-chunk counts, ordered compaction + head remap */
  STS_K_ATTN_SPARSE = 5,   /* split sparse gather flash-decode */
  STS_K_ATTN_DENSE = 6,    /* split dense flash-decode */
  STS_K_ATTN_COMBINE = 7,  /* split combine */
  STS_K_SELECT_BLOCK = 8,  /* per-block score sums + first-digit histogram (page_size > 1) */
  STS_K_HEADMAP = 9,       /* Algorithm 1: overlap counting and argmax */
  STS_K_SELECT_SMALL = 10, /* whole selection in one workgroup per row (rows up to 32768 tokens) */
  STS_K_SELECT_LOCAL = 11, /* small budgets: aggregation + top-k inside each 8192-token chunk */
  STS_K_SELECT_POOL = 12,  /* small budgets: ranking of the chunks' winners, one workgroup per row */
  STS_K_ATTN_PROBSUM = 13, /* dense second pass over K: attention weights summed over the query block */
  STS_K_SELECT_FUSED = 14, /* long rows: aggregation, threshold and compaction in one launch */
  STS_K_UNION_ROWS = 15,   /* union of per-row index lists + row bits */
  STS_K_SELECT_BAND = 16,  /* at least a row per compute unit: one workgroup per row, one pass */
  STS_K_COUNT_ = 17
} sts_kernel_kind;
#define STS_PROF_MAX 4096

void sts_prof_enable(int on);
void sts_prof_reset(void);
sts_status sts_prof_read(int kernel_kind, int32_t *launches, double *total_ms);

/* Tuning and test knobs (process-wide; not part of the method). Before a knob is first set or
 * read, its environment variable, read once per process, gives the initial value; NaN (the
 * default) leaves the library's own rule in force. Set them between calls, never while a call
 * of another thread is in flight.
 *  - STS_KNOB_ATTN_WGS_PER_CU (env STS_ATTN_WGS_PER_CU): target workgroups per compute unit when
 *    the context is split. It changes the split count, hence sts_attn_workspace_bytes and the
 *    rounding of the output: a workspace sized before the change may be refused afterwards
 *    (STS_EWORKSPACE; never written out of bounds).
 *  - STS_KNOB_SELECT_SPIN_LIMIT (env STS_SELECT_SPIN_LIMIT): polls of another workgroup's
 *    published counts before they are recomputed locally. No effect on results.
 *  - STS_KNOB_PROBSUM_WGS_PER_CU (env STS_PROBSUM_WGS_PER_CU): workgroups per compute unit of the
 *    pass that writes weights_sum_out. No effect on results.
 *  - STS_KNOB_SELECT_PATH (env STS_SELECT_PATH): 0 the library's rule, 1 histogram pipeline only,
 *    2 pipeline or chunk-local top-k + pool, 3 the one-launch selection for rows of up to 256
 *    parts (the rule stops at 8), 4 one workgroup per row in several passes wherever the shape
 *    allows it (Tq = 1, probabilities, token granularity, no agg_out, N a multiple of 4, or of 8
 *    for bf16), 5 one workgroup per row in one pass wherever the shape allows it (token
 *    granularity, N a multiple of 4 up to 524288). It changes sts_select_workspace_bytes, never
 *    the results.
 *  - STS_KNOB_SELECT_ROW_THREADS (env STS_SELECT_ROW_THREADS): 256 or 1024, the workgroup size of
 *    the several-pass one-workgroup-per-row selection (the rule: 256 from 4 rows per compute
 *    unit on, else 1024). No effect on results.
 */
typedef enum {
  STS_KNOB_ATTN_WGS_PER_CU = 0,
  STS_KNOB_SELECT_SPIN_LIMIT = 1,
  STS_KNOB_PROBSUM_WGS_PER_CU = 2,
  STS_KNOB_SELECT_PATH = 3,
  STS_KNOB_SELECT_ROW_THREADS = 4,
  STS_KNOB_COUNT_ = 5
} sts_knob;
void sts_set_knob(int knob, double value);
double sts_get_knob(int knob);

/* Launch geometry chosen for a shape (for reports): number of context splits and of
 * (head-set) work units per batch element. Returns STS_OK or the validation error. */
sts_status sts_attn_plan(const sts_attn_params *p, int sparse, int32_t *num_splits,
                         int32_t *units_per_batch, int32_t *query_tiles);

#ifdef __cplusplus
}
#endif
#endif
