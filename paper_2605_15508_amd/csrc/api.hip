// Host side of the C ABI declared in include/sts.h: argument validation, launch planning,
// workspace carving, kernel enqueue, and the optional per-kernel event timing.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "common.h"

thread_local StsLaunchEvents g_sts_launch_events = {nullptr, nullptr};
thread_local hipError_t g_sts_launch_rc = hipSuccess;

namespace {

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// ------------------------------------------------------------------------- profiling aid
struct ProfEvent {
  hipEvent_t start, stop;
  int kind;
};
std::mutex g_prof_mu;
bool g_prof_on = false;
std::vector<ProfEvent> g_prof_pool;   // created lazily, reused after reset
size_t g_prof_used = 0;

template <class F>
hipError_t run_kernel(int kind, hipStream_t s, F &&launch) {
  if (!g_prof_on) return launch();
  std::lock_guard<std::mutex> lk(g_prof_mu);
  if (g_prof_used >= STS_PROF_MAX) return launch();
  if (g_prof_used == g_prof_pool.size()) {
    ProfEvent e;
    if (hipEventCreate(&e.start) != hipSuccess) return launch();
    if (hipEventCreate(&e.stop) != hipSuccess) {
      (void)hipEventDestroy(e.start);
      return launch();
    }
    g_prof_pool.push_back(e);
  }
  ProfEvent &e = g_prof_pool[g_prof_used];
  e.kind = kind;
  // the dispatch stamps the two events with the kernel's own begin and end (every launcher
  // enqueues exactly one kernel per call)
  g_sts_launch_events = StsLaunchEvents{e.start, e.stop};
  const hipError_t rc = launch();
  g_sts_launch_events = StsLaunchEvents{nullptr, nullptr};
  if (rc == hipSuccess) ++g_prof_used;
  return rc;
}

// ------------------------------------------------------------------------- tuning knobs
// Values set with sts_set_knob; before the first set or get of a knob its environment variable
// (read once per process) gives the initial value. NaN = not set: the library's own rule applies.
const char *const KNOB_ENV[STS_KNOB_COUNT_] = {"STS_ATTN_WGS_PER_CU", "STS_SELECT_SPIN_LIMIT",
                                               "STS_PROBSUM_WGS_PER_CU", "STS_SELECT_PATH",
                                               "STS_SELECT_ROW_THREADS"};
std::mutex g_knob_mu;
double g_knob[STS_KNOB_COUNT_];
bool g_knob_init = false;

void knobs_init_locked() {
  if (g_knob_init) return;
  for (int i = 0; i < STS_KNOB_COUNT_; ++i) {
    const char *e = getenv(KNOB_ENV[i]);
    g_knob[i] = (e && *e) ? atof(e) : NAN;
  }
  g_knob_init = true;
}

double knob(int which) {
  std::lock_guard<std::mutex> lk(g_knob_mu);
  knobs_init_locked();
  return g_knob[which];
}

int cu_count() {
  static const int cus = [] {   // once per process (thread-safe initialisation)
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      return n;
    return 256;
  }();
  return cus;
}

// ------------------------------------------------------------------------ attention plan
sts_status validate_attn(const sts_attn_params *p, int sparse) {
  if (!p) return STS_EINVAL;
  if (p->B < 0 || p->Tq < 1 || p->Hq < 1 || p->Hkv < 1 || p->N < 0) return STS_EINVAL;
  if (p->Hq % p->Hkv != 0) return STS_EINVAL;
  if (p->d != 64 && p->d != 128) return STS_EUNSUPPORTED;
  if (p->Tq > 16 || p->Hq > STS_MAX_HEADS || p->Hq / p->Hkv > STS_MAX_GROUP) return STS_EUNSUPPORTED;
  if (p->out_dtype != STS_BF16 && p->out_dtype != STS_F32) return STS_EINVAL;
  if (!isfinite(p->scale)) return STS_EINVAL;
  if (p->row_mask && (!sparse || p->block_table)) return sparse ? STS_EUNSUPPORTED : STS_EINVAL;
  if (sparse) {
    if (p->kmax < 0) return STS_EINVAL;
    if (p->logits_out || p->seq_lens) return STS_EINVAL;
    if (p->head_map)
      for (int t = 0; t < p->Hq; ++t)
        if (p->head_map[t] < 0) return STS_EINVAL;
  } else {
    if (p->indices || p->counts) return STS_EINVAL;
  }
  if (p->kv_stride_n < p->d || (p->kv_stride_n * 2) % 16 != 0 || (p->kv_stride_h * 2) % 16 != 0 ||
      (p->kv_stride_b * 2) % 16 != 0)
    return STS_EUNSUPPORTED;
  const int page = p->page_size <= 1 ? 1 : p->page_size;
  if (page != 1 && page != 2 && page != 4 && page != 8 && page != 16 && page != 32) return STS_EUNSUPPORTED;
  if (p->block_table) {
    if (p->num_pages < 1 || p->kv_stride_page < 1 || (p->kv_stride_page * 2) % 16 != 0) return STS_EINVAL;
    if ((int64_t)p->table_stride * page < p->N) return STS_EINVAL;
  }
  if (sparse && (int64_t)p->kmax * page > 0x7fffffffll - 65536) return STS_EUNSUPPORTED;
  if (p->idx_stride_b < 0 || p->cnt_stride_b < 0) return STS_EINVAL;
  if (sparse && p->idx_stride_b && p->idx_stride_b < (int64_t)p->Hq * p->kmax) return STS_EINVAL;
  if (sparse && p->cnt_stride_b && p->cnt_stride_b < p->Hq) return STS_EINVAL;
  if ((p->k_new == nullptr) != (p->v_new == nullptr)) return STS_EINVAL;
  if (p->k_new && (reinterpret_cast<uintptr_t>(p->k_new) % 16 != 0 || reinterpret_cast<uintptr_t>(p->v_new) % 16 != 0))
    return STS_EUNSUPPORTED;
  return STS_OK;
}

int page_of(const sts_attn_params *p) { return p->page_size <= 1 ? 1 : p->page_size; }

// Group query heads into units and pick the split count. Uses only host data.
sts_status plan_attn(const sts_attn_params *p, int sparse, AttnPlan &pl) {
  const sts_status v = validate_attn(p, sparse);
  if (v != STS_OK) return v;
  const int G = p->Hq / p->Hkv;
  // at most 4 query tiles of 16 rows per unit; 2 for the logits dump at head size 128, whose
  // four-tile form would not fit the register file (a KV group with more rows is served by two
  // units, each reading K and V: next to the dump's own writes that costs little)
  int max_heads = ((!sparse && p->logits_out && p->d == 128) ? 32 : 64) / p->Tq;
  if (max_heads < 1) max_heads = 1;
  if (max_heads > STS_MAX_GROUP) max_heads = STS_MAX_GROUP;
  int nu = 0, max_rows = 0;
  memset(&pl.units, 0, sizeof(pl.units));
  for (int g = 0; g < p->Hkv; ++g) {
    bool done[STS_MAX_GROUP] = {false};
    for (int i = 0; i < G; ++i) {
      if (done[i]) continue;
      // members of the set led by head i, in head order
      int members[STS_MAX_GROUP], nm = 0;
      for (int j2 = i; j2 < G; ++j2) {
        if (done[j2]) continue;
        const bool same = !sparse || j2 == i ||
                          (p->head_map && p->head_map[g * G + j2] == p->head_map[g * G + i]);
        if (same) {
          members[nm++] = j2;
          done[j2] = true;
        }
      }
      for (int s0 = 0; s0 < nm; s0 += max_heads) {
        const int cnt = (nm - s0 < max_heads) ? nm - s0 : max_heads;
        uint32_t mask = 0;
        for (int m = 0; m < cnt; ++m) mask |= 1u << members[s0 + m];
        if (nu >= STS_MAX_HEADS) return STS_EUNSUPPORTED;
        pl.units.unit[nu++] = (uint32_t)g | (mask << 8) | ((uint32_t)cnt << 24);
        if (cnt * p->Tq > max_rows) max_rows = cnt * p->Tq;
      }
    }
  }
  pl.num_units = nu;
  pl.nq = max_rows <= 16 ? 1 : (max_rows <= 32 ? 2 : 4);
  const int64_t len = sparse ? (int64_t)p->kmax * page_of(p) : p->N;
  const int64_t tiles = (len + STS_TILE_KEYS - 1) / STS_TILE_KEYS;
  // Workgroups per CU the split count aims at. Two for the gather (its two dependent latencies
  // per tile want more waves) and for head size 64; one for the dense kernel at head size 128,
  // where a second workgroup per CU only costs (128K context, batch 4: 348 -> 324 us; 32K,
  // batch 1: 51 -> 44 us),
  // and for four query tiles (one workgroup fills the register file).
  // The gather with two query tiles at head size 128 (as register-bound as the dense kernel)
  // is 3% faster with one as well.
  int64_t resident = (int64_t)cu_count() * ((pl.nq == 4 || (p->d == 128 && (!sparse || pl.nq == 2))) ? 1 : 2);
  const double wgs_knob = knob(STS_KNOB_ATTN_WGS_PER_CU);   // tuning knob: target workgroups per CU
  const bool wgs_set = wgs_knob > 0.0;                       // (NaN compares false)
  if (wgs_set) resident = (int64_t)(cu_count() * wgs_knob);
  const int64_t units_total = (int64_t)p->B * nu;
  int64_t S = units_total > 0 ? resident / units_total : 1;
  // at least two tiles per wave, so that the partials and their combine stay small next to
  // the gathered bytes; a list of up to 16 tiles is not split at all (its workgroup writes
  // the result itself, one launch instead of two)
  const int64_t s_cap = tiles <= 16 ? 1 : (tiles + 2 * STS_WG_WAVES - 1) / (2 * STS_WG_WAVES);
  if (S > s_cap) S = s_cap;
  if (S > 256) S = 256;
  // With at least one unit per CU, halving every unit only adds the combine launch: one
  // workgroup per CU keeps enough loads in flight (70B-shaped layer, 256 units of 410 tiles:
  // 268 us unsplit against 278 us in two halves).
  if (S == 2 && units_total >= cu_count() && !wgs_set) S = 1;
  if (S < 1) S = 1;
  pl.num_splits = (int)S;
  const size_t parts = (size_t)units_total * (size_t)S;
  if ((size_t)units_total * (size_t)S > 0x7fffffffull) return STS_EUNSUPPORTED;
  pl.part_o_bytes = align256(parts * (size_t)pl.nq * 16 * p->d * sizeof(float));
  pl.part_ml_bytes = align256(parts * (size_t)pl.nq * 16 * 2 * sizeof(float));
  pl.lse_bytes = (!sparse && p->weights_sum_out && !p->lse_out)
                     ? align256((size_t)p->B * p->Hq * p->Tq * sizeof(float)) : 0;
  return STS_OK;
}

// ws / ws_bytes: the scratch memory of the call (the caller's workspace, or the library's static
// array for the entry point that allocates nothing, which also keeps the timing aid off: creating
// events allocates).
sts_status run_attn(const sts_attn_params *p, int sparse, hipStream_t s, void *ws, size_t ws_bytes, bool timed) {
  AttnPlan pl;
  const sts_status v = plan_attn(p, sparse, pl);
  if (v != STS_OK) return v;
  if (p->B == 0) return STS_OK;
  if (!p->q || !p->out) return STS_EINVAL;
  if (p->N > 0 && (!p->k || !p->v)) return STS_EINVAL;
  if (sparse && p->kmax > 0 && !p->indices) return STS_EINVAL;
  if (sparse && p->kmax > 0 && p->N == 0) return STS_EINVAL;
  const size_t need = pl.part_o_bytes + pl.part_ml_bytes + pl.lse_bytes;
  if (!ws || ws_bytes < need) return STS_EWORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return STS_EWORKSPACE;
  const bool want_sum = !sparse && p->weights_sum_out != nullptr;
  // (the second pass adds a 32-bit lane offset of up to 12 rows to a 64-bit tile address)
  if (want_sum && (p->block_table || p->k_new || page_of(p) != 1 ||
                   reinterpret_cast<uintptr_t>(p->weights_sum_out) % 4 != 0 ||
                   p->kv_stride_n < 0 || p->kv_stride_n > (int64_t)1 << 26))
    return STS_EUNSUPPORTED;
  if (reinterpret_cast<uintptr_t>(p->k) % 16 != 0 || reinterpret_cast<uintptr_t>(p->v) % 16 != 0 ||
      reinterpret_cast<uintptr_t>(p->q) % 16 != 0 || reinterpret_cast<uintptr_t>(p->out) % 16 != 0 ||
      reinterpret_cast<uintptr_t>(p->logits_out) % 16 != 0)
    return STS_EUNSUPPORTED;

  AttnArgs a;
  memset(&a, 0, sizeof(a));
  a.q = static_cast<const uint16_t *>(p->q);
  a.k = static_cast<const uint16_t *>(p->k);
  a.v = static_cast<const uint16_t *>(p->v);
  a.indices = sparse ? p->indices : nullptr;
  a.counts = sparse ? p->counts : nullptr;
  a.row_mask = sparse ? p->row_mask : nullptr;
  a.idx_stride_b = p->idx_stride_b ? p->idx_stride_b : (int64_t)p->Hq * p->kmax;
  a.cnt_stride_b = p->cnt_stride_b ? p->cnt_stride_b : p->Hq;
  a.seq_lens = sparse ? nullptr : p->seq_lens;
  a.stride_b = p->kv_stride_b;
  a.stride_h = p->kv_stride_h;
  a.stride_n = p->kv_stride_n;
  a.B = p->B; a.Tq = p->Tq; a.Hq = p->Hq; a.Hkv = p->Hkv; a.G = p->Hq / p->Hkv; a.N = p->N;
  a.kmax = sparse ? p->kmax : 0;
  a.page = page_of(p);
  a.page_shift = 0;
  while ((1 << a.page_shift) < a.page) ++a.page_shift;
  a.block_table = p->block_table;
  a.table_stride = p->table_stride;
  a.num_pages = p->num_pages;
  a.stride_page = p->kv_stride_page;
  a.k_new = static_cast<const uint16_t *>(p->k_new);
  a.v_new = static_cast<const uint16_t *>(p->v_new);
  a.causal = p->causal;
  a.direct = (pl.num_splits == 1) ? 1 : 0;
  a.num_units = pl.num_units;
  a.num_splits = pl.num_splits;
  a.scale = p->scale;
  a.scale_log2 = p->scale * 1.44269504088896340736f;
  a.part_o = static_cast<float *>(ws);
  a.part_ml = reinterpret_cast<float *>(static_cast<unsigned char *>(ws) + pl.part_o_bytes);
  a.logits_out = sparse ? nullptr : p->logits_out;
  a.logits_bf16 = p->logits_bf16 ? 1 : 0;
  a.out = p->out;
  a.lse_out = p->lse_out;
  if (want_sum && !a.lse_out)   // the second pass needs the row normalisers
    a.lse_out = reinterpret_cast<float *>(static_cast<unsigned char *>(ws) + pl.part_o_bytes + pl.part_ml_bytes);
  a.out_dtype = p->out_dtype;
  a.units = pl.units;

  hipError_t rc = timed ? run_kernel(sparse ? STS_K_ATTN_SPARSE : STS_K_ATTN_DENSE, s,
                                     [&] { return launch_attn_split(a, p->d, pl.nq, sparse != 0, s); })
                        : launch_attn_split(a, p->d, pl.nq, sparse != 0, s);
  if (rc != hipSuccess) return STS_EHIP;
  if (!a.direct) {
    rc = timed ? run_kernel(STS_K_ATTN_COMBINE, s, [&] { return launch_attn_combine(a, p->d, pl.nq, s); })
               : launch_attn_combine(a, p->d, pl.nq, s);
    if (rc != hipSuccess) return STS_EHIP;
  }
  if (want_sum && p->N > 0) {
    // Second pass over K. Heads of a KV group share a workgroup in sets of up to 64 rows; the key
    // range is cut so that the grid is one full residency of the chip (a second, partly filled
    // round would cost more than finer balancing gains), each wave keeping at least 4 tiles.
    a.agg_out = p->weights_sum_out;
    int tp = 1;
    while (tp < p->Tq) tp *= 2;      // a head's rows fill an aligned power-of-two run of MFMA columns
    int hs = 64 / tp;
    if (hs > a.G) hs = a.G;
    a.ps_tp = tp;
    a.ps_heads = hs;
    a.ps_sets = (a.G + hs - 1) / hs;
    const int rows = hs * tp;
    const int nq = rows <= 16 ? 1 : (rows <= 32 ? 2 : 4);
    const int64_t tiles = ((int64_t)p->N + STS_TILE_KEYS - 1) / STS_TILE_KEYS;
    const int64_t groups = (int64_t)p->B * p->Hkv * a.ps_sets;
    double per_cu = attn_probsum_wgs_per_cu(p->d, nq);
    if (const double f = knob(STS_KNOB_PROBSUM_WGS_PER_CU); f > 0.0) per_cu = f;   // tuning knob
    int64_t S = (int64_t)(cu_count() * per_cu) / groups;
    const int64_t s_cap = (tiles + 4 * STS_WG_WAVES - 1) / (4 * STS_WG_WAVES);
    if (S > s_cap) S = s_cap;
    if (S < 1) S = 1;
    if (groups * S > 0x7fffffffll) return STS_EUNSUPPORTED;
    a.ps_splits = (int)S;
    rc = run_kernel(STS_K_ATTN_PROBSUM, s, [&] { return launch_attn_probsum(a, p->d, nq, s); });
    if (rc != hipSuccess) return STS_EHIP;
  }
  return STS_OK;
}

// --------------------------------------------------------------------------- select plan
struct SelectPlan {
  bool small;          // one workgroup per row, keys in LDS, a single launch
  bool pool;           // shape allows chunk-local top-k + one ranking workgroup per row
  bool fused;          // long rows: parts of a row in LDS, one launch (plus the flag clear)
  bool band;           // at least a row per CU: one workgroup per row, one pass, no workspace
  bool rowpass;        // many long rows of ready-made scores: one workgroup per row, no workspace
  int rowpass_threads;
  int nchunks, page, srcN, pool_pitch, pool_chunk, pool_nchunks;
  int part_tokens, parts;
  size_t agg_bytes, blk_bytes, hist_bytes, state_bytes, chunk_bytes;
  size_t pool_key_bytes;
  size_t pub_bytes, pflag_bytes;
  size_t pipeline_total() const { return agg_bytes + blk_bytes + hist_bytes + state_bytes + chunk_bytes; }
  size_t pool_total() const { return pool ? 2 * pool_key_bytes : 0; }
  size_t fused_total() const { return pub_bytes + pflag_bytes; }
  // a pool-shaped call falls back to the pipeline when its pointers are not 16-byte aligned,
  // so the workspace covers both
  size_t total() const {
    if (rowpass || band) return 0;
    if (fused) return fused_total();
    return pipeline_total() > pool_total() ? pipeline_total() : pool_total();
  }
};

sts_status plan_select(const sts_select_params *p, SelectPlan &pl) {
  if (!p) return STS_EINVAL;
  if (p->B < 0 || p->Hd < 1 || p->Tq < 1 || p->N < 0 || p->Hq < 1 || p->k < 1) return STS_EINVAL;
  if (p->kind != STS_SCORES_PROBS && p->kind != STS_SCORES_LOGITS_LSE) return STS_EINVAL;
  if (p->reduce != STS_REDUCE_SUM && p->reduce != STS_REDUCE_MAX) return STS_EINVAL;
  if (p->Tq > 64 || p->Hq > STS_MAX_HEADS || p->Hd > STS_MAX_HEADS) return STS_EUNSUPPORTED;
  if ((int64_t)p->N > 0x7fffffffll - 65536) return STS_EUNSUPPORTED;
  if ((int64_t)p->B * p->Hd > 65535) return STS_EUNSUPPORTED;   // grid.y
  if (p->page_size < 0 || p->page_size > 4096) return STS_EUNSUPPORTED;
  pl.page = p->page_size <= 1 ? 1 : p->page_size;
  pl.srcN = (p->N + pl.page - 1) / pl.page;
  pl.nchunks = (pl.srcN + SEL_CHUNK - 1) / SEL_CHUNK;
  const size_t rows = (size_t)p->B * p->Hd;
  // One workgroup ranks a whole row out of LDS at one CU's pace: a clear win for short rows
  // (one launch instead of six), and for rows up to the LDS limit when there are enough rows
  // to fill the chip anyway; longer or fewer rows keep the many-workgroup pipeline.
  pl.small = pl.page == 1 && (p->N <= SEL_FUSED_N || (p->N <= SEL_SMALL_N && rows >= 256));
  pl.pool = false;
  pl.pool_pitch = 0;
  pl.pool_key_bytes = 0;
  pl.fused = false;
  pl.rowpass = false;
  pl.band = false;
  pl.rowpass_threads = 0;
  pl.part_tokens = pl.parts = 0;
  pl.pub_bytes = pl.pflag_bytes = 0;
  // test / tuning knob: 0 the library's rule, 1 histogram pipeline only, 2 pipeline or pool,
  // 3 the one-launch selection wherever its shape limits allow, 4 one workgroup per row in
  // several passes wherever its shape limits allow, 5 one workgroup per row in one pass likewise
  const double path_knob = knob(STS_KNOB_SELECT_PATH);
  const int path = path_knob == path_knob ? (int)path_knob : 0;
  // Enough rows to give at least every second CU one, and rows that do not fit one workgroup's
  // LDS: one workgroup per row, which samples the row, keeps the band of keys around the
  // threshold in LDS during a single pass and never talks to another workgroup
  // (select_band_kernel); nothing to clear, no workspace. The band of a full-length row with the
  // call's largest budget has to fit (rows for which it does not, decided in the kernel, are
  // ranked by plain passes there). Measured against the paths below, 128K-token rows, 10%: 256
  // rows of 8 fp32 scores per token 220 against 289 us, bf16 140 against 203, 512 rows of 16 bf16
  // scores 448 against 613, 256 rows of one fp32 score 67 against 147 (pipeline, in place), 128
  // rows of 5 scores 93 against 111; 64 rows: 83 against 58, hence the limit.
  // One bf16 score per token and many rows per CU (a mask per query row of prefill) is the one
  // shape that plain passes by small workgroups serve better (select_rowpass_kernel; 4096 rows of
  // 128K: 754 against 962 us; one workgroup per row out of parts that exchange: 2.1 ms).
  {
    int kmax = p->k;
    if (p->k_head) {
      kmax = 1;
      for (int j = 0; j < p->Hd; ++j) kmax = p->k_head[j] > kmax ? p->k_head[j] : kmax;
    }
    const bool aligned = reinterpret_cast<uintptr_t>(p->scores) % 16 == 0;
    const bool band_ok = pl.page == 1 && p->N > 0 && p->N <= BAND_MAX_N && (p->N % 4) == 0 && aligned &&
                         (!p->agg_out || reinterpret_cast<uintptr_t>(p->agg_out) % 16 == 0);
    const bool fits = band_ok && (p->N <= BAND_CAP ||
                                  band_plan(p->N, (uint32_t)(kmax < p->N ? kmax : p->N), p->scores_bf16 ? 64 : 32).fits);
    const bool rowpass_ok = pl.page == 1 && p->Tq == 1 && p->kind == STS_SCORES_PROBS && !p->agg_out && p->N > 0 &&
                            (p->N % (p->scores_bf16 ? 8 : 4)) == 0 && aligned;
    const int64_t cus = cu_count();
    const bool long_rows = !pl.small && p->N > SEL_FUSED_N;
    const bool take_rowpass = path == 4 ? rowpass_ok
                                        : path == 0 && rowpass_ok && long_rows && p->scores_bf16 && (int64_t)rows >= 4 * cus;
    const bool take_band = path == 5 ? band_ok : path == 0 && !take_rowpass && fits && long_rows && 2 * (int64_t)rows >= cus;
    if (take_rowpass || take_band) {
      pl.small = false;
      pl.band = take_band;
      pl.rowpass = take_rowpass;
      pl.rowpass_threads = (int64_t)rows >= 4 * cus ? 256 : 1024;
      if (const double t = knob(STS_KNOB_SELECT_ROW_THREADS); t == 256.0 || t == 1024.0) pl.rowpass_threads = (int)t;
      pl.nchunks = 0;
      pl.pool_chunk = pl.pool_nchunks = 0;
      pl.agg_bytes = pl.blk_bytes = pl.hist_bytes = pl.state_bytes = pl.chunk_bytes = 0;
      return STS_OK;
    }
  }
  if (pl.small) {
    pl.nchunks = 0;
    pl.agg_bytes = pl.blk_bytes = pl.hist_bytes = pl.state_bytes = pl.chunk_bytes = 0;
    return STS_OK;
  }
  // Small budgets on long rows: each chunk of the row keeps its own best k tokens and one
  // workgroup per row ranks that pool out of LDS (two launches, the scores are read once and
  // the aggregate is never stored). The ranking workgroup works at one CU's pace, about 1.2 us
  // per 1000 pooled pairs on top of 10 us, so the pool must be small: up to 8192 pairs it beats
  // the five-launch pipeline for every shape measured, up to 16384 only when the pipeline's
  // passes over the aggregate are long (8M scores or more in the call). Chunks are 8192 tokens,
  // or 32768 when only that keeps the pool small enough (long rows, middle budgets).
  pl.pool_chunk = pl.pool_nchunks = 0;
  if (pl.page == 1 && (p->N % 4) == 0 && path != 1) {
    for (const int chunk : {SEL_CHUNK, 4 * SEL_CHUNK}) {
      const int64_t nch = ((int64_t)p->N + chunk - 1) / chunk;
      const int64_t pitch = p->k < chunk ? p->k : chunk;
      const int64_t pooled = nch * pitch;
      // a grid of few large workgroups leaves most of the chip idle: then the pipeline is as fast
      if (chunk > SEL_CHUNK && (int64_t)rows * nch < 128) break;
      if (pooled <= SEL_POOL_MAX / 2 || (pooled <= SEL_POOL_MAX && (int64_t)rows * p->N >= (int64_t)1 << 23)) {
        pl.pool = true;
        pl.pool_chunk = chunk;
        pl.pool_nchunks = (int)nch;
        pl.pool_pitch = (int)pitch;
        pl.pool_key_bytes = align256(rows * (size_t)nch * (size_t)pitch * sizeof(uint32_t));
        break;
      }
    }
  }
  // Long rows at token granularity: one launch in which every workgroup keeps a part of a row in
  // LDS (select_fused_kernel). Parts are as large as LDS allows (32768 tokens) when that still
  // gives a workgroup per CU, else smaller, down to 8192, to spread short calls over the chip.
  // (One exception under the library's own rule: a ready-made fp32 aggregate, Tq = 1, that the
  // pipeline ranks where it lies, in a call with more workgroups than CUs. There the pipeline's
  // passes over the caller's tensor beat several rounds of workgroups that wait for each other:
  // 70B-shaped layer, 256 rows of 128K: 153 against 182 us.)
  const bool in_place = p->Tq == 1 && p->kind == STS_SCORES_PROBS && !p->scores_bf16 && !p->agg_out;
  const bool many_rounds = (int64_t)rows * (((int64_t)p->N + SEL_SMALL_N - 1) / SEL_SMALL_N) > cu_count();
  if (pl.page == 1 && p->N > SEL_FUSED_N && path != 1 && path != 2 && !(path == 0 && in_place && many_rounds)) {
    const int max_parts = path == 3 ? 256 : SEL_FUSED_MAX_PARTS;
    int P = SEL_SMALL_N;
    while (P > SEL_FUSED_N && (int64_t)rows * (((int64_t)p->N + P - 1) / P) < cu_count() &&
           ((int64_t)p->N + P / 2 - 1) / (P / 2) <= max_parts)
      P >>= 1;
    const int64_t parts = ((int64_t)p->N + P - 1) / P;
    if (parts <= max_parts) {
      pl.fused = true;
      pl.pool = false;
      pl.part_tokens = P;
      pl.parts = (int)parts;
      pl.pub_bytes = align256(rows * 3 * (size_t)parts * 1024 * sizeof(unsigned long long));
      pl.pflag_bytes = 0;
    }
  }
  pl.agg_bytes = p->agg_out ? 0 : align256(rows * (size_t)p->N * sizeof(float));
  pl.blk_bytes = pl.page > 1 ? align256(rows * (size_t)pl.srcN * sizeof(float)) : 0;
  pl.hist_bytes = align256(rows * 3 * SEL_BINS * sizeof(uint32_t));
  pl.state_bytes = align256(rows * 8 * sizeof(uint32_t));
  pl.chunk_bytes = align256(rows * (size_t)pl.nchunks * SEL_FLAG_PITCH * sizeof(uint32_t));
  return STS_OK;
}

}  // namespace

extern "C" {

size_t sts_attn_workspace_bytes(const sts_attn_params *p, int sparse) {
  AttnPlan pl;
  if (plan_attn(p, sparse, pl) != STS_OK) return 0;
  const size_t n = pl.part_o_bytes + pl.part_ml_bytes + pl.lse_bytes;
  return n ? n : 256;
}

sts_status sts_attn_plan(const sts_attn_params *p, int sparse, int32_t *num_splits,
                         int32_t *units_per_batch, int32_t *query_tiles) {
  AttnPlan pl;
  const sts_status v = plan_attn(p, sparse, pl);
  if (v != STS_OK) return v;
  if (num_splits) *num_splits = pl.num_splits;
  if (units_per_batch) *units_per_batch = pl.num_units;
  if (query_tiles) *query_tiles = pl.nq;
  return STS_OK;
}

sts_status sts_sparse_attn(const sts_attn_params *p, void *stream) {
  if (!p) return STS_EINVAL;
  return run_attn(p, 1, static_cast<hipStream_t>(stream), p->workspace, p->workspace_bytes, true);
}

sts_status sts_dense_attn(const sts_attn_params *p, void *stream) {
  if (!p) return STS_EINVAL;
  return run_attn(p, 0, static_cast<hipStream_t>(stream), p->workspace, p->workspace_bytes, true);
}

sts_status sts_sparse_attn_static(const sts_attn_params *p, void *stream) {
  if (!p) return STS_EINVAL;
  void *ws = nullptr;
  const sts_status v = sts_static_scratch(&ws);
  if (v != STS_OK) return v;
  // a shape whose partial results do not fit the array comes back as STS_EWORKSPACE
  return run_attn(p, 1, static_cast<hipStream_t>(stream), ws, STS_STATIC_SCRATCH_BYTES, false);
}

size_t sts_select_workspace_bytes(const sts_select_params *p) {
  SelectPlan pl;
  if (plan_select(p, pl) != STS_OK) return 0;
  const size_t n = pl.total();
  return n ? n : 256;
}

static sts_status enqueue_select(const sts_select_params *p, void *stream) {
  SelectPlan pl;
  const sts_status v = plan_select(p, pl);
  if (v != STS_OK) return v;
  if (!p->head_map || !p->indices) return STS_EINVAL;
  for (int t = 0; t < p->Hq; ++t)
    if (p->head_map[t] < 0 || p->head_map[t] >= p->Hd) return STS_EINVAL;
  if (p->k_head)
    for (int j = 0; j < p->Hd; ++j)
      if (p->k_head[j] < 1 || p->k_head[j] > p->k) return STS_EINVAL;
  if (p->B == 0) return STS_OK;
  if (p->N > 0 && !p->scores) return STS_EINVAL;
  if (p->kind == STS_SCORES_LOGITS_LSE && !p->lse) return STS_EINVAL;
  const size_t need = pl.total();
  if (need > 0) {
    if (!p->workspace || p->workspace_bytes < need) return STS_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(p->workspace) % 256 != 0) return STS_EWORKSPACE;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);

  SelectArgs a;
  memset(&a, 0, sizeof(a));
  a.scores = p->scores;
  a.scores_bf16 = p->scores_bf16 ? 1 : 0;
  a.lse = p->kind == STS_SCORES_LOGITS_LSE ? p->lse : nullptr;
  a.seq_lens = p->seq_lens;
  a.indices = p->indices;
  a.counts = p->counts;
  unsigned char *w = static_cast<unsigned char *>(p->workspace);
  a.agg = p->agg_out ? p->agg_out : reinterpret_cast<float *>(w);
  w += pl.agg_bytes;
  a.blk = pl.page > 1 ? reinterpret_cast<float *>(w) : nullptr;
  w += pl.blk_bytes;
  a.page = pl.page;
  a.srcN = pl.srcN;
  a.src = pl.page > 1 ? a.blk : a.agg;
  a.hist = reinterpret_cast<uint32_t *>(w);
  w += pl.hist_bytes;
  a.state = reinterpret_cast<uint32_t *>(w);
  w += pl.state_bytes;
  a.chunk_cnt = reinterpret_cast<uint32_t *>(w);
  a.B = p->B; a.Hd = p->Hd; a.Tq = p->Tq; a.N = p->N; a.Hq = p->Hq; a.k = p->k;
  a.kind = p->kind; a.reduce = p->reduce; a.nchunks = pl.nchunks;
  for (int j = 0; j < p->Hd; ++j) a.kh[j] = p->k_head ? p->k_head[j] : p->k;
  a.clear_words = (pl.hist_bytes + pl.state_bytes + pl.chunk_bytes) / sizeof(uint32_t);
  // The refinement histograms pay a digit search, a zeroed LDS histogram and a flush of up to
  // 2048 global atomics per workgroup: with more than about a thousand workgroups it is cheaper
  // to give each of them 2 or 4 consecutive chunks (1M-token rows: 22 -> 17.7 us per pass).
  {
    const size_t wgs = (size_t)p->B * p->Hd * (size_t)(pl.nchunks > 0 ? pl.nchunks : 1);
    a.hist_cpw = wgs >= 4096 ? 4 : (wgs >= 2048 ? 2 : 1);
  }
  // Test knob: STS_SELECT_SPIN_LIMIT bounds the polls of an earlier chunk's published counts
  // before the waiting workgroup recounts that chunk itself (0: one look, then recount).
  {
    const double v = knob(STS_KNOB_SELECT_SPIN_LIMIT);
    const bool set = v == v;   // not NaN
    a.spin_limit = !set ? 256 : (v < 0 ? 0 : (v > 65536 ? 65536 : (int)v));
    // the parts of the one-launch selection wait for ALL parts of their row, and recomputing a
    // missing part's histogram means re-reading its scores: a far longer patience by default
    a.fused_spin_limit = !set ? 20000 : a.spin_limit;
  }
  // inverse of the head map: the target heads fed by each draft head, in head order
  {
    int cnt[STS_MAX_HEADS + 1] = {0};
    for (int t = 0; t < p->Hq; ++t) ++cnt[p->head_map[t] + 1];
    for (int j = 0; j < p->Hd; ++j) cnt[j + 1] += cnt[j];
    for (int j = 0; j <= p->Hd; ++j) a.targets.off[j] = (uint16_t)cnt[j];
    int fill[STS_MAX_HEADS] = {0};
    for (int t = 0; t < p->Hq; ++t) {
      const int j = p->head_map[t];
      a.targets.tgt[cnt[j] + fill[j]++] = (uint8_t)t;
    }
  }

  hipError_t rc;
  if (pl.band) {
    a.agg = p->agg_out;   // optional output only
    a.src = nullptr;
    a.hist = a.state = a.chunk_cnt = nullptr;
    rc = run_kernel(STS_K_SELECT_BAND, s, [&] { return launch_select_band(a, s); });
    return rc == hipSuccess ? STS_OK : STS_EHIP;
  }
  if (pl.rowpass) {
    a.agg = nullptr;
    a.src = nullptr;
    a.hist = a.state = a.chunk_cnt = nullptr;
    a.rowpass_threads = pl.rowpass_threads;
    rc = run_kernel(STS_K_SELECT_ROWPASS, s, [&] { return launch_select_rowpass(a, s); });
    return rc == hipSuccess ? STS_OK : STS_EHIP;
  }
  if (pl.fused) {
    unsigned char *fw = static_cast<unsigned char *>(p->workspace);
    a.pub = reinterpret_cast<unsigned long long *>(fw);
    a.part_tokens = pl.part_tokens;
    a.parts = pl.parts;
    a.agg = p->agg_out;   // optional output only: the keys never leave LDS
    a.src = nullptr;
    a.hist = a.state = a.chunk_cnt = nullptr;   // the pipeline's scratch does not exist on this path
    if (pl.parts > 1) {
      rc = run_kernel(STS_K_SELECT_CLEAR, s, [&] { return launch_select_clear_pub(a, s); });
      if (rc != hipSuccess) return STS_EHIP;
    }
    rc = run_kernel(STS_K_SELECT_FUSED, s, [&] { return launch_select_fused(a, s); });
    return rc == hipSuccess ? STS_OK : STS_EHIP;
  }
  if (pl.pool && reinterpret_cast<uintptr_t>(p->scores) % 16 == 0 &&
      (!p->agg_out || reinterpret_cast<uintptr_t>(p->agg_out) % 16 == 0)) {
    unsigned char *pw = static_cast<unsigned char *>(p->workspace);
    a.pool_key = reinterpret_cast<uint32_t *>(pw);
    a.pool_idx = reinterpret_cast<int32_t *>(pw + pl.pool_key_bytes);
    a.pool_pitch = pl.pool_pitch;
    a.pool_chunk = pl.pool_chunk;
    a.pool_nchunks = pl.pool_nchunks;
    a.agg = p->agg_out;   // optional output only
    rc = run_kernel(STS_K_SELECT_LOCAL, s, [&] { return launch_select_local(a, s); });
    if (rc != hipSuccess) return STS_EHIP;
    rc = run_kernel(STS_K_SELECT_POOL, s, [&] { return launch_select_pool(a, s); });
    return rc == hipSuccess ? STS_OK : STS_EHIP;
  }
  if (pl.small) {
    a.agg = p->agg_out;   // optional output only: the keys never leave LDS
    rc = run_kernel(STS_K_SELECT_SMALL, s, [&] { return launch_select_small(a, s); });
    return rc == hipSuccess ? STS_OK : STS_EHIP;
  }
  // Block granularity: aggregation and block sums in one pass when the shape allows (the
  // per-token aggregate is then stored only on request), and up to 16384 blocks per row are
  // ranked by one workgroup per row out of LDS: two launches, nothing to clear (18 us for 8192
  // blocks, 28 us for 16384, against about 30 us for the four kernels it replaces).
  SelectArgs f = a;
  f.agg = p->agg_out;
  const bool fused_blocks = pl.page > 1 && select_aggblock_ok(f);
  if (fused_blocks && pl.srcN <= SEL_SMALL_N / 2) {
    f.hist = nullptr;
    rc = run_kernel(STS_K_SELECT_AGG, s, [&] { return launch_select_aggblock(f, s); });
    if (rc != hipSuccess) return STS_EHIP;
    rc = run_kernel(STS_K_SELECT_SMALL, s, [&] { return launch_select_rank(f, s); });
    return rc == hipSuccess ? STS_OK : STS_EHIP;
  }
  // One fp32 probability row per head (an aggregate computed elsewhere, e.g. the draft layer's
  // summed attention weights): the aggregate is the input itself, so the first pass only builds
  // the first-digit histogram and the later passes read the caller's tensor.
  if (pl.page == 1 && p->Tq == 1 && p->kind == STS_SCORES_PROBS && !p->scores_bf16 && !p->agg_out) {
    a.agg = const_cast<float *>(static_cast<const float *>(p->scores));
    a.src = a.agg;
    a.agg_is_input = 1;
  }
  if (pl.nchunks > 0) {
    rc = run_kernel(STS_K_SELECT_CLEAR, s, [&] { return launch_select_clear(a, s); });
    if (rc != hipSuccess) return STS_EHIP;
    if (fused_blocks) {
      rc = run_kernel(STS_K_SELECT_AGG, s, [&] { return launch_select_aggblock(f, s); });
      if (rc != hipSuccess) return STS_EHIP;
    } else {
      rc = run_kernel(STS_K_SELECT_AGG, s, [&] { return launch_select_agg(a, s); });
      if (rc != hipSuccess) return STS_EHIP;
      if (pl.page > 1) {
        rc = run_kernel(STS_K_SELECT_BLOCK, s, [&] { return launch_select_block(a, s); });
        if (rc != hipSuccess) return STS_EHIP;
      }
    }
    rc = run_kernel(STS_K_SELECT_HIST, s, [&] { return launch_select_hist(a, 1, s); });
    if (rc != hipSuccess) return STS_EHIP;
    rc = run_kernel(STS_K_SELECT_HIST, s, [&] { return launch_select_hist(a, 2, s); });
    if (rc != hipSuccess) return STS_EHIP;
  }
  rc = run_kernel(STS_K_SELECT_WRITE, s, [&] { return launch_select_write(a, s); });
  return rc == hipSuccess ? STS_OK : STS_EHIP;
}

sts_status sts_select(const sts_select_params *p, void *stream) { return enqueue_select(p, stream); }

// ---------------------------------------------------------------------------- head mapping
namespace {
constexpr int HM_SLICE = 32768;   // rows per selection launch (grid.y limit)

struct HeadmapPlan {
  size_t idx_d_bytes, idx_t_bytes, overlap_bytes, select_bytes;
};

sts_status plan_headmap(const sts_headmap_params *p, HeadmapPlan &pl) {
  if (!p) return STS_EINVAL;
  if (p->S < 0 || p->R < 0 || p->Hd < 1 || p->Ht < 1 || p->N < 0 || p->k < 1) return STS_EINVAL;
  if ((int64_t)p->N > 0x7fffffffll - 65536) return STS_EUNSUPPORTED;
  const size_t rows_d = (size_t)p->S * p->Hd * p->R, rows_t = (size_t)p->S * p->Ht * p->R;
  if (rows_d > 0x7fffffffull || rows_t > 0x7fffffffull || (size_t)p->S * p->R > 0x7fffffffull) return STS_EUNSUPPORTED;
  if (p->Ht > 65535) return STS_EUNSUPPORTED;
  pl.idx_d_bytes = align256(rows_d * (size_t)p->k * sizeof(int32_t));
  pl.idx_t_bytes = align256(rows_t * (size_t)p->k * sizeof(int32_t));
  pl.overlap_bytes = align256((size_t)p->Ht * p->Hd * sizeof(unsigned long long));
  // One selection slice at a time: B = rows of the slice, one draft head, one query row. The
  // selection chooses its path (and with it its scratch size) from the row count, so the scratch
  // is sized for the largest need over every slice size that will be launched: the full slices
  // and the tail slice of either trace.
  pl.select_bytes = 0;
  for (const size_t rows : {rows_d, rows_t}) {
    const size_t sizes[2] = {rows >= (size_t)HM_SLICE ? (size_t)HM_SLICE : 0, rows % (size_t)HM_SLICE};
    for (const size_t n : sizes) {
      if (n == 0) continue;
      sts_select_params sp;
      memset(&sp, 0, sizeof(sp));
      sp.B = (int32_t)n;
      sp.Hd = 1; sp.Tq = 1; sp.N = p->N; sp.Hq = 1; sp.k = p->k;
      SelectPlan spl;
      const sts_status v = plan_select(&sp, spl);
      if (v != STS_OK) return v;
      if (spl.total() > pl.select_bytes) pl.select_bytes = spl.total();
    }
  }
  return STS_OK;
}

// top-k index lists of every row of one trace, slice by slice, through the selection pipeline
sts_status select_rows(const float *trace, size_t rows, int N, int k, int32_t *idx, void *ws, size_t ws_bytes,
                       void *stream) {
  static const int32_t identity[1] = {0};
  for (size_t r0 = 0; r0 < rows; r0 += HM_SLICE) {
    sts_select_params sp;
    memset(&sp, 0, sizeof(sp));
    sp.B = (int32_t)(rows - r0 < (size_t)HM_SLICE ? rows - r0 : (size_t)HM_SLICE);
    sp.Hd = 1; sp.Tq = 1; sp.N = N; sp.Hq = 1; sp.k = k;
    sp.scores = trace + r0 * (size_t)N;
    sp.head_map = identity;
    sp.indices = idx + r0 * (size_t)k;
    sp.kind = STS_SCORES_PROBS;
    sp.reduce = STS_REDUCE_SUM;
    sp.workspace = ws;
    sp.workspace_bytes = ws_bytes;
    const sts_status v = enqueue_select(&sp, stream);
    if (v != STS_OK) return v;
  }
  return STS_OK;
}
}  // namespace

size_t sts_headmap_workspace_bytes(const sts_headmap_params *p) {
  HeadmapPlan pl;
  if (plan_headmap(p, pl) != STS_OK) return 0;
  return pl.idx_d_bytes + pl.idx_t_bytes + pl.overlap_bytes + pl.select_bytes + 256;
}

sts_status sts_head_map(const sts_headmap_params *p, void *stream) {
  HeadmapPlan pl;
  const sts_status v = plan_headmap(p, pl);
  if (v != STS_OK) return v;
  if (!p->map) return STS_EINVAL;
  const bool have_rows = (size_t)p->S * p->R > 0 && p->N > 0;
  if (have_rows && (!p->a_d || !p->a_t)) return STS_EINVAL;
  const size_t need = pl.idx_d_bytes + pl.idx_t_bytes + pl.overlap_bytes + pl.select_bytes;
  if (!p->workspace || p->workspace_bytes < need) return STS_EWORKSPACE;
  if (reinterpret_cast<uintptr_t>(p->workspace) % 256 != 0) return STS_EWORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned char *w = static_cast<unsigned char *>(p->workspace);
  int32_t *idx_d = reinterpret_cast<int32_t *>(w);
  w += pl.idx_d_bytes;
  int32_t *idx_t = reinterpret_cast<int32_t *>(w);
  w += pl.idx_t_bytes;
  // the counts accumulate in the caller's buffer when one is given
  unsigned long long *ov = p->overlap ? p->overlap : reinterpret_cast<unsigned long long *>(w);
  w += pl.overlap_bytes;
  void *sel_ws = w;

  const int c = p->k < p->N ? p->k : p->N;
  if (have_rows) {
    sts_status rc = select_rows(p->a_d, (size_t)p->S * p->Hd * p->R, p->N, p->k, idx_d, sel_ws, pl.select_bytes, stream);
    if (rc != STS_OK) return rc;
    rc = select_rows(p->a_t, (size_t)p->S * p->Ht * p->R, p->N, p->k, idx_t, sel_ws, pl.select_bytes, stream);
    if (rc != STS_OK) return rc;
  }
  hipError_t e = run_kernel(STS_K_HEADMAP, s, [&] { return launch_headmap_clear(ov, p->Ht * p->Hd, s); });
  if (e != hipSuccess) return STS_EHIP;
  if (have_rows) {
    e = run_kernel(STS_K_HEADMAP, s, [&] {
      return launch_headmap_overlap(idx_d, idx_t, p->S, p->R, p->Hd, p->Ht, p->k, c, ov, s);
    });
    if (e != hipSuccess) return STS_EHIP;
  }
  e = run_kernel(STS_K_HEADMAP, s, [&] { return launch_headmap_argmax(ov, p->Hd, p->Ht, p->map, s); });
  return e == hipSuccess ? STS_OK : STS_EHIP;
}

sts_status sts_union_rows(const sts_union_params *p, void *stream) {
  if (!p) return STS_EINVAL;
  if (p->B < 0 || p->Hd < 1 || p->Hq < 1 || p->Tq < 1 || p->N < 0 || p->k < 0 || p->pitch < 0) return STS_EINVAL;
  if (p->Tq > 16 || p->Hq > STS_MAX_HEADS || p->Hd > STS_MAX_HEADS || p->B > 65535) return STS_EUNSUPPORTED;
  if ((int64_t)p->N > 0x7fffffffll - 65536) return STS_EUNSUPPORTED;
  if (!p->head_map || !p->indices || !p->row_mask) return STS_EINVAL;
  for (int t = 0; t < p->Hq; ++t)
    if (p->head_map[t] < 0 || p->head_map[t] >= p->Hd) return STS_EINVAL;
  if (p->B == 0) return STS_OK;
  if (p->k > 0 && !p->row_indices) return STS_EINVAL;
  UnionArgs a;
  memset(&a, 0, sizeof(a));
  a.row_idx = p->row_indices;
  a.row_cnt = p->row_counts;
  a.indices = p->indices;
  a.row_mask = p->row_mask;
  a.counts = p->counts;
  a.B = p->B; a.Hd = p->Hd; a.Hq = p->Hq; a.Tq = p->Tq; a.N = p->N; a.k = p->k; a.pitch = p->pitch;
  for (int t = 0; t < p->Hq; ++t) a.map[t] = (uint8_t)p->head_map[t];
  hipStream_t s = static_cast<hipStream_t>(stream);
  const hipError_t rc = run_kernel(STS_K_UNION_ROWS, s, [&] { return launch_union_rows(a, s); });
  return rc == hipSuccess ? STS_OK : STS_EHIP;
}

const char *sts_strerror(int status) {   // an int on purpose: any value a caller holds may be asked about
  switch (status) {
    case STS_OK: return "ok";
    case STS_EINVAL: return "invalid argument";
    case STS_EUNSUPPORTED: return "unsupported shape";
    case STS_EWORKSPACE: return "workspace missing, misaligned or too small";
    case STS_EHIP: return "HIP launch error";
  }
  return "unknown status";
}

int sts_version(void) { return 204; }

void sts_set_knob(int which, double value) {
  if (which < 0 || which >= STS_KNOB_COUNT_) return;
  std::lock_guard<std::mutex> lk(g_knob_mu);
  knobs_init_locked();
  g_knob[which] = value;
}

double sts_get_knob(int which) {
  if (which < 0 || which >= STS_KNOB_COUNT_) return NAN;
  return knob(which);
}

void sts_prof_enable(int on) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  g_prof_on = on != 0;
}

void sts_prof_reset(void) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  g_prof_used = 0;
}

sts_status sts_prof_read(int kernel_kind, int32_t *launches, double *total_ms) {
  if (kernel_kind < 0 || kernel_kind >= STS_K_COUNT_) return STS_EINVAL;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  int n = 0;
  double ms = 0.0;
  for (size_t i = 0; i < g_prof_used; ++i) {
    const ProfEvent &e = g_prof_pool[i];
    if (e.kind != kernel_kind) continue;
    if (hipEventSynchronize(e.stop) != hipSuccess) return STS_EHIP;
    float t = 0.f;
    // a launcher that had nothing to enqueue (an empty grid) leaves its pair unstamped
    if (hipEventElapsedTime(&t, e.start, e.stop) != hipSuccess) {
      (void)hipGetLastError();
      continue;
    }
    ms += t;
    ++n;
  }
  if (launches) *launches = n;
  if (total_ms) *total_ms = ms;
  return STS_OK;
}

}  // extern "C"
