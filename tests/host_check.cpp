// Host-side sanitizer driver (test infrastructure, not part of libsts.so). It is linked with the
// library's host file only: the kernel launchers are replaced by stubs that check their launch
// arguments and touch no device memory, so every entry point can be driven on a machine without
// a GPU, with made-up device addresses, under AddressSanitizer and UndefinedBehaviorSanitizer:
// planning, workspace sizing and carving, argument validation, the head-map tables, error paths.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "common.h"

static long g_launches = 0;
static const unsigned char *g_ws_lo = nullptr, *g_ws_hi = nullptr;

static void fail(const char *what) {
  fprintf(stderr, "host check failed: %s\n", what);
  exit(3);
}
static void in_ws(const void *p, const char *what) {
  const unsigned char *c = static_cast<const unsigned char *>(p);
  if (p && (c < g_ws_lo || c > g_ws_hi)) fail(what);
}

// the static scratch array lives in device memory: here a made-up address stands in for it
static unsigned char *const g_static_ws = reinterpret_cast<unsigned char *>(uintptr_t(3) << 40);
sts_status sts_static_scratch(void **out) { *out = g_static_ws; return STS_OK; }

// ---- stub launchers: argument checks only
hipError_t launch_attn_split(const AttnArgs &a, int d, int nq, bool sparse, hipStream_t) {
  ++g_launches;
  if ((d != 64 && d != 128) || (nq != 1 && nq != 2 && nq != 4)) fail("split: d / nq");
  if (a.num_splits < 1 || a.num_units < 1 || a.num_units > STS_MAX_HEADS) fail("split: grid");
  if (sparse && !a.indices && a.kmax > 0) fail("split: indices");
  in_ws(a.part_o, "split: part_o");
  in_ws(a.part_ml, "split: part_ml");
  for (int u = 0; u < a.num_units; ++u) {
    const uint32_t unit = a.units.unit[u];
    const int g = unit & 0xff, n = (unit >> 24) & 0x1f;
    if (g >= a.Hkv || n < 1 || n * a.Tq > nq * 16) fail("split: unit table");
  }
  return hipSuccess;
}
hipError_t launch_attn_combine(const AttnArgs &a, int, int, hipStream_t) { ++g_launches; if (a.direct) fail("combine after a direct launch"); return hipSuccess; }
hipError_t launch_attn_probsum(const AttnArgs &a, int, int nq, hipStream_t) {
  ++g_launches;
  if (!a.agg_out || !a.lse_out || a.ps_splits < 1 || a.ps_sets < 1 || a.ps_heads < 1) fail("probsum: args");
  if (a.ps_tp < a.Tq || (a.ps_tp & (a.ps_tp - 1)) || a.ps_heads * a.ps_tp > nq * 16) fail("probsum: rows");
  return hipSuccess;
}
int attn_probsum_wgs_per_cu(int, int) { return 2; }
static void check_select(const SelectArgs &a, const char *what) {
  ++g_launches;
  if (a.B < 1 || a.Hd < 1 || a.k < 1) fail(what);
  in_ws(a.hist, what);
  in_ws(a.state, what);
  in_ws(a.chunk_cnt, what);
  in_ws(a.pool_key, what);
  in_ws(a.pool_idx, what);
  in_ws(a.blk, what);
  if (a.targets.off[a.Hd] != a.Hq) fail("select: inverse head map");
  for (int j = 0; j < a.Hd; ++j)
    for (int t = a.targets.off[j]; t < a.targets.off[j + 1]; ++t)
      if (a.targets.tgt[t] >= a.Hq) fail("select: target table");
  for (int j = 0; j < a.Hd; ++j)
    if (a.kh[j] < 1 || a.kh[j] > a.k) fail("select: budgets");
  if (a.page < 1 || a.srcN != (a.N + a.page - 1) / a.page) fail("select: block count");
  if (a.spin_limit < 0) fail("select: spin limit");
}
static void check_pipeline(const SelectArgs &a, const char *what) {
  check_select(a, what);
  if (a.nchunks != (a.srcN + SEL_CHUNK - 1) / SEL_CHUNK) fail("pipeline: chunks");
  if (a.hist_cpw != 1 && a.hist_cpw != 2 && a.hist_cpw != 4) fail("pipeline: chunks per workgroup");
  if (!a.hist || !a.state || !a.chunk_cnt) fail("pipeline: workspace parts");
  if (!a.agg_is_input) in_ws(a.agg, "pipeline: aggregate");
  // the cleared region covers the three histograms, the state words and the chunk flags of every row
  const size_t rows = (size_t)a.B * a.Hd;
  if (a.clear_words < rows * (3 * SEL_BINS + 8 + (size_t)a.nchunks * SEL_FLAG_PITCH)) fail("pipeline: cleared region");
  in_ws(reinterpret_cast<const unsigned char *>(a.hist) + a.clear_words * 4, "pipeline: cleared region end");
}
static void check_pool(const SelectArgs &a, const char *what) {
  check_select(a, what);
  if (a.pool_chunk != SEL_CHUNK && a.pool_chunk != 4 * SEL_CHUNK) fail("pool: chunk size");
  if (a.pool_nchunks != (a.N + a.pool_chunk - 1) / a.pool_chunk) fail("pool: chunks");
  if (a.pool_pitch != (a.k < a.pool_chunk ? a.k : a.pool_chunk)) fail("pool: pitch");
  if ((int64_t)a.pool_nchunks * a.pool_pitch > SEL_POOL_MAX) fail("pool: pairs per row beyond the LDS limit");
  if (a.N % 4 != 0 || a.page != 1 || !a.pool_key || !a.pool_idx) fail("pool: shape");
  in_ws(reinterpret_cast<const unsigned char *>(a.pool_idx) + (size_t)a.B * a.Hd * a.pool_nchunks * a.pool_pitch * 4, "pool: end");
}
hipError_t launch_select_clear(const SelectArgs &a, hipStream_t) { check_pipeline(a, "clear"); return hipSuccess; }
hipError_t launch_select_agg(const SelectArgs &a, hipStream_t) { check_select(a, "agg"); return hipSuccess; }
hipError_t launch_select_block(const SelectArgs &a, hipStream_t) { check_select(a, "block"); return hipSuccess; }
hipError_t launch_select_small(const SelectArgs &a, hipStream_t) { check_select(a, "small"); return hipSuccess; }
hipError_t launch_select_rank(const SelectArgs &a, hipStream_t) { check_select(a, "rank"); return hipSuccess; }
bool select_aggblock_ok(const SelectArgs &a) { return a.page >= 4 && a.page <= 256 && (a.page & (a.page - 1)) == 0 && a.N % a.page == 0; }
hipError_t launch_select_aggblock(const SelectArgs &a, hipStream_t) { check_select(a, "aggblock"); return hipSuccess; }
static void check_fused(const SelectArgs &a, const char *what) {
  check_select(a, what);
  in_ws(a.pub, what);
  const int P = a.part_tokens;
  if (P != 8192 && P != 16384 && P != 32768) fail("fused: part size");
  if (a.parts != (a.N + P - 1) / P || a.parts < 1 || a.parts > 256) fail("fused: parts");
  if (a.page != 1 || a.N <= SEL_FUSED_N || !a.pub) fail("fused: shape");
  if (a.fused_spin_limit < 0) fail("fused: spin limit");
  in_ws(reinterpret_cast<const unsigned char *>(a.pub) + (size_t)a.B * a.Hd * 3 * a.parts * 8192, "fused: end");
}
hipError_t launch_select_fused(const SelectArgs &a, hipStream_t) { check_fused(a, "fused"); return hipSuccess; }
hipError_t launch_select_clear_pub(const SelectArgs &a, hipStream_t) { check_fused(a, "clear published words"); return hipSuccess; }
bool select_band_ok(const SelectArgs &a) {
  return a.page == 1 && a.N > 0 && a.N <= BAND_MAX_N && (a.N % 4) == 0 && (reinterpret_cast<uintptr_t>(a.scores) % 16) == 0 &&
         (a.agg == nullptr || (reinterpret_cast<uintptr_t>(a.agg) % 16) == 0);
}
hipError_t launch_select_band(const SelectArgs &a, hipStream_t) {
  check_select(a, "band");
  if (!select_band_ok(a)) fail("band: shape");
  return hipSuccess;
}
bool select_rowpass_ok(const SelectArgs &a) {
  return a.Tq == 1 && a.kind == STS_SCORES_PROBS && a.page == 1 && a.agg == nullptr && a.N > 0 &&
         (a.N % (a.scores_bf16 ? 8 : 4)) == 0 && (reinterpret_cast<uintptr_t>(a.scores) % 16) == 0;
}
hipError_t launch_select_rowpass(const SelectArgs &a, hipStream_t) {
  check_select(a, "rowpass");
  if (!select_rowpass_ok(a)) fail("rowpass: shape");
  if (a.rowpass_threads != 256 && a.rowpass_threads != 1024) fail("rowpass: threads");
  return hipSuccess;
}
hipError_t launch_select_local(const SelectArgs &a, hipStream_t) { check_pool(a, "local"); return hipSuccess; }
hipError_t launch_select_pool(const SelectArgs &a, hipStream_t) { check_pool(a, "pool"); return hipSuccess; }
hipError_t launch_select_hist(const SelectArgs &a, int pass, hipStream_t) { check_pipeline(a, "hist"); if (pass != 1 && pass != 2) fail("hist pass"); return hipSuccess; }
hipError_t launch_select_write(const SelectArgs &a, hipStream_t) { check_pipeline(a, "write"); return hipSuccess; }
hipError_t launch_union_rows(const UnionArgs &a, hipStream_t) {
  ++g_launches;
  if (a.Tq < 1 || a.Tq > 16 || a.Hq < 1 || a.Hd < 1 || !a.indices || !a.row_mask) fail("union: args");
  for (int t = 0; t < a.Hq; ++t)
    if (a.map[t] >= a.Hd) fail("union: head map");
  return hipSuccess;
}
hipError_t launch_headmap_clear(unsigned long long *, int, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_headmap_overlap(const int32_t *, const int32_t *, int, int, int, int, int, int, unsigned long long *, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_headmap_argmax(const unsigned long long *, int, int, int32_t *, hipStream_t) { ++g_launches; return hipSuccess; }

// The sampling plan of the one-pass selection (shared by host and kernel): the sample fits the
// workgroup's store, covers the row from its first token to within one period of its end, and a
// plan that claims to fit leaves the band room with margin.
static void check_band_plans() {
  for (int run : {32, 64})
    for (int nb : {8193, 8200, 20000, 40000, 65536, 131072, 131072 - 13, 262144, 262208, 524288})
      for (uint32_t c : {1u, 100u, 512u, 3000u, 13108u, 26215u, 65536u, 131072u, 524288u}) {
        if (c > (uint32_t)nb) continue;
        const BandPlan p = band_plan(nb, c, run);
        if (p.S < 16 || (p.S & (p.S - 1)) != 0) fail("band plan: sampling period");
        if (p.ns < 1 || p.ns > 2 * BAND_CAP || p.ns > nb) fail("band plan: sample size");
        if ((long long)(p.runs - 1) * p.S * run >= nb) fail("band plan: a sampled run starts past the row");
        if ((long long)p.runs * p.S * run < nb) fail("band plan: the row's end is not within one period of the last run");
        if (p.s_lo <= p.s_hi) fail("band plan: empty band");
        if (p.fits && (p.s_lo > p.ns || (long long)p.S * (p.s_lo - (p.s_hi >= 1 ? p.s_hi : 0)) > BAND_CAP)) fail("band plan: fit");
      }
  // the headline budgets fit at 128K tokens; nearly everything kept does not
  if (!band_plan(131072, 13108, 32).fits || !band_plan(131072, 26215, 64).fits) fail("band plan: 10% / 20% of 128K must fit");
  if (band_plan(131072, 131000, 32).fits) fail("band plan: a budget next to the row length cannot fit");
}

int main() {
  long calls = 0, accepted = 0;
  check_band_plans();
  // made-up, 256-byte aligned "device" addresses: never dereferenced (the launchers are stubs)
  unsigned char *const fake = reinterpret_cast<unsigned char *>(uintptr_t(1) << 40);
  unsigned char *const ws = reinterpret_cast<unsigned char *>(uintptr_t(2) << 40);
  const int Bs[] = {0, 1, 4, 33}, Tqs[] = {1, 5, 8, 16}, Ns[] = {0, 1, 31, 4096, 131072, 1 << 20}, ds[] = {64, 128};
  for (int B : Bs) for (int Tq : Tqs) for (int N : Ns) for (int d : ds)
    for (int Hkv : {1, 8, 16}) for (int G : {1, 4, 8, 16}) {
      const int Hq = Hkv * G;
      if (Hq > 256) continue;
      for (int sparse = 0; sparse < 2; ++sparse)
        for (int page : {0, 8})
          for (int hmk = 0; hmk < 3; ++hmk)
            for (int extra = 0; extra < 3; ++extra) {
              sts_attn_params p;
              memset(&p, 0, sizeof(p));
              p.B = B; p.Tq = Tq; p.Hq = Hq; p.Hkv = Hkv; p.d = d; p.N = N;
              p.kv_stride_n = d; p.kv_stride_h = (int64_t)N * d; p.kv_stride_b = (int64_t)Hkv * N * d;
              p.kmax = sparse ? (N / 10 + 1) : 0;
              p.scale = 0.1f; p.page_size = page;
              std::vector<int32_t> hm(Hq);
              for (int t = 0; t < Hq; ++t) hm[t] = hmk == 0 ? t : (hmk == 1 ? t / 2 : 0);
              p.head_map = sparse ? hm.data() : nullptr;
              p.q = fake; p.k = fake; p.v = fake; p.out = fake;
              if (sparse) p.indices = reinterpret_cast<const int32_t *>(fake);
              if (extra == 1) { p.k_new = fake; p.v_new = fake; p.causal = 1; }
              if (extra == 2 && !sparse && page == 0) p.weights_sum_out = reinterpret_cast<float *>(fake);
              int32_t s = 0, u = 0, nq = 0;
              const size_t need = sts_attn_workspace_bytes(&p, sparse);
              (void)sts_attn_plan(&p, sparse, &s, &u, &nq);
              p.workspace = ws; p.workspace_bytes = need;
              g_ws_lo = ws; g_ws_hi = ws + need;
              const sts_status rc = sparse ? sts_sparse_attn(&p, nullptr) : sts_dense_attn(&p, nullptr);
              accepted += rc == STS_OK;
              if (sparse) {                  // the same call on the static scratch array: accepted iff it fits
                g_ws_lo = g_static_ws; g_ws_hi = g_static_ws + STS_STATIC_SCRATCH_BYTES;
                const sts_status rs = sts_sparse_attn_static(&p, nullptr);
                if (rc == STS_OK && B > 0 && rs != (need <= STS_STATIC_SCRATCH_BYTES ? STS_OK : STS_EWORKSPACE)) fail("static scratch: wrong verdict");
                if (rc != STS_OK && rs == STS_OK) fail("static scratch accepted what the workspace call refuses");
                g_ws_lo = ws; g_ws_hi = ws + need;
                ++calls;
              }
              if (need > 256) {              // one byte short must be refused
                p.workspace_bytes = need - 1;
                if ((sparse ? sts_sparse_attn(&p, nullptr) : sts_dense_attn(&p, nullptr)) == STS_OK && B > 0) fail("short attention workspace accepted");
              }
              calls += 4;
            }
    }
  for (int path : {0, 1, 2, 3, 4, 5}) {
  sts_set_knob(STS_KNOB_SELECT_PATH, path);
  for (int B : Bs) for (int Tq : {1, 5, 64}) for (int N : Ns) for (int Hd : {1, 16, 256}) for (int Hq : {1, 32, 256})
    for (int k : {1, 410, 13108, 1 << 20}) for (int page : {0, 8, 4096}) for (int budgets = 0; budgets < 2; ++budgets) {
      if ((int64_t)B * Hd > 65535) continue;
      sts_select_params p;
      memset(&p, 0, sizeof(p));
      p.B = B; p.Hd = Hd; p.Tq = Tq; p.N = N; p.Hq = Hq; p.k = k; p.page_size = page;
      std::vector<int32_t> hm(Hq), kh(Hd);
      for (int t = 0; t < Hq; ++t) hm[t] = t % Hd;
      for (int j = 0; j < Hd; ++j) kh[j] = 1 + (j % k);
      p.head_map = hm.data();
      p.k_head = budgets ? kh.data() : nullptr;
      p.scores = fake; p.indices = reinterpret_cast<int32_t *>(fake);
      const size_t need = sts_select_workspace_bytes(&p);
      p.workspace = ws; p.workspace_bytes = need;
      g_ws_lo = ws; g_ws_hi = ws + need;
      accepted += sts_select(&p, nullptr) == STS_OK;
      hm[0] = Hd;                           // out of range: must be refused
      if (sts_select(&p, nullptr) == STS_OK) fail("bad head map accepted");
      calls += 3;
    }
  }
  sts_set_knob(STS_KNOB_SELECT_PATH, 0);
  // a split count changed between the size query and the call: refused, never written out of bounds
  {
    sts_attn_params p;
    memset(&p, 0, sizeof(p));
    p.B = 1; p.Tq = 5; p.Hq = 32; p.Hkv = 8; p.d = 128; p.N = 131072; p.kmax = 13108;
    p.kv_stride_n = 128; p.kv_stride_h = (int64_t)p.N * 128; p.kv_stride_b = 8 * p.kv_stride_h;
    p.scale = 0.1f;
    p.q = fake; p.k = fake; p.v = fake; p.out = fake; p.indices = reinterpret_cast<const int32_t *>(fake);
    sts_set_knob(STS_KNOB_ATTN_WGS_PER_CU, 1.0);
    const size_t small_need = sts_attn_workspace_bytes(&p, 1);
    sts_set_knob(STS_KNOB_ATTN_WGS_PER_CU, 4.0);
    const size_t big_need = sts_attn_workspace_bytes(&p, 1);
    if (!(big_need > small_need)) fail("the knob does not change the split count");
    p.workspace = ws; p.workspace_bytes = small_need;
    g_ws_lo = ws; g_ws_hi = ws + small_need;
    if (sts_sparse_attn(&p, nullptr) != STS_EWORKSPACE) fail("workspace sized for another split count accepted");
    p.workspace_bytes = big_need;
    g_ws_lo = ws; g_ws_hi = ws + big_need;
    if (sts_sparse_attn(&p, nullptr) != STS_OK) fail("workspace of the right size refused");
    sts_set_knob(STS_KNOB_ATTN_WGS_PER_CU, NAN);
    if (sts_get_knob(STS_KNOB_ATTN_WGS_PER_CU) == sts_get_knob(STS_KNOB_ATTN_WGS_PER_CU)) fail("knob not reset");
    calls += 4;
  }
  for (int S : {0, 1, 4}) for (int R : {0, 1, 128}) for (int N : {0, 1, 32768}) for (int k : {1, 512}) {
    sts_headmap_params p;
    memset(&p, 0, sizeof(p));
    p.S = S; p.R = R; p.Hd = 16; p.Ht = 32; p.N = N; p.k = k;
    p.a_d = reinterpret_cast<const float *>(fake); p.a_t = reinterpret_cast<const float *>(fake);
    p.map = reinterpret_cast<int32_t *>(fake);
    const size_t need = sts_headmap_workspace_bytes(&p);
    p.workspace = ws; p.workspace_bytes = need;
    g_ws_lo = ws; g_ws_hi = ws + need;
    accepted += sts_head_map(&p, nullptr) == STS_OK;
    calls += 2;
  }
  // Selection slices of different row counts take different paths (and scratch sizes): the size
  // query must cover every slice launched, and a refusal must come before the first enqueue.
  {
    struct { int S, R, Hd, Ht, N, k; } shapes[] = {
        {1, 16, 8, 32, 16384, 64},      // 128 draft rows (pipeline: needs scratch), 512 target rows (one workgroup per row: none)
        {1, 4109, 8, 32, 16384, 64},    // a full 32768-row slice followed by a 104-row tail
        {1, 8, 4, 8, 40000, 100},       // rows beyond what one workgroup ranks out of LDS
        {2, 300, 16, 32, 131072, 512},  // small budget on long rows: chunk-local top-k + pool
    };
    for (const auto &sh : shapes) {
      sts_headmap_params p;
      memset(&p, 0, sizeof(p));
      p.S = sh.S; p.R = sh.R; p.Hd = sh.Hd; p.Ht = sh.Ht; p.N = sh.N; p.k = sh.k;
      p.a_d = reinterpret_cast<const float *>(fake); p.a_t = reinterpret_cast<const float *>(fake);
      p.map = reinterpret_cast<int32_t *>(fake);
      const size_t need = sts_headmap_workspace_bytes(&p);
      p.workspace = ws; p.workspace_bytes = need;
      g_ws_lo = ws; g_ws_hi = ws + need;
      if (sts_head_map(&p, nullptr) != STS_OK) fail("head map refuses the workspace size it asked for");
      const long before = g_launches;
      p.workspace_bytes = need - 257;       // (the query adds one alignment unit of slack)
      if (sts_head_map(&p, nullptr) != STS_EWORKSPACE) fail("short head-map workspace accepted");
      if (g_launches != before) fail("head map enqueued kernels before refusing");
      calls += 3;
      ++accepted;
    }
  }
  for (int Tq : {0, 1, 16, 17}) for (int Hq : {1, 256}) for (int Hd : {1, 16}) for (int bad : {0, 1}) {
    sts_union_params p;
    memset(&p, 0, sizeof(p));
    std::vector<int32_t> hm(Hq);
    for (int t = 0; t < Hq; ++t) hm[t] = t % Hd;
    if (bad) hm[Hq - 1] = Hd;
    p.B = 2; p.Hd = Hd; p.Hq = Hq; p.Tq = Tq; p.N = 5000; p.k = 100; p.pitch = 1600;
    p.row_indices = reinterpret_cast<const int32_t *>(fake);
    p.head_map = hm.data();
    p.indices = reinterpret_cast<int32_t *>(fake); p.row_mask = reinterpret_cast<uint16_t *>(fake);
    const sts_status rc = sts_union_rows(&p, nullptr);
    if ((rc == STS_OK) != (Tq >= 1 && Tq <= 16 && !bad)) fail("union: wrong verdict");
    accepted += rc == STS_OK;
    ++calls;
  }
  for (int s = 1; s >= -6; --s)
    if (!sts_strerror(s)[0]) fail("empty error string");
  if (accepted == 0 || g_launches == 0) fail("nothing was accepted: the driver checks nothing");
  printf("host checks done: %ld calls, %ld accepted, %ld stub launches, version %d\n", calls, accepted, g_launches, sts_version());
  return 0;
}
