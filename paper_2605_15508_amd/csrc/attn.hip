// Split flash-decode attention for the STS verification step (gfx950).
//
// One kernel family serves sparse attention over gathered KV rows (paper Section 4.2: attend
// only to the key-value pairs named by the indices; Section 5: per-head KV sets, scattered
// rows staged in on-chip memory, split-K) and the dense baseline (identity index row).
//
// Work decomposition. A unit is the set of query heads of one KV group that share one index
// row; its nheads*Tq query rows are padded to NQ tiles of 16. The unit's index row is cut
// into num_splits contiguous pieces; one workgroup of 4 waves owns one (batch, unit, split)
// and its waves take alternating 32-key tiles. Each wave keeps its own online-softmax state
// (fp32), the 4 waves are merged through LDS and one partial (max, sum, O) per workgroup goes
// to the workspace; a second kernel combines the splits in fixed order.
//
// Tile arithmetic, all in the transposed orientation so that nothing but K needs LDS:
//   S^T[key, query] = K[key, :] . Q[query, :]      v_mfma_f32_16x16x32_bf16, A = K tile
//   O^T[d,  query] += V^T[d, key] P^T[key, query]                            A = V^T tile
// Lane (a, b) = (lane / 16, lane % 16). The MFMA output S^T gives lane (a, b) the keys
// {4a..4a+3, 16+4a..16+4a+3} of query b: exactly the 8 contraction elements lane (a, b) must
// supply as the B operand of the second product, so P never moves between lanes. The
// contraction order over d (first product) and the d-column owned by a lane (second product)
// are free, so they are chosen to make every global load a full coalesced row read:
//   - 16 consecutive lanes load the 16 chunks of one K or V row (256 B at d = 128);
//   - V^T's A operand for output tile nt is element nt of each of the lane's 8 loaded V
//     chunks (lane b owns d = NT*b + nt), two v_perm_b32 per register pair;
//   - K is written to a wave-private, XOR-swizzled LDS tile and read back as ds_read_b128 in
//     MFMA A layout (the only cross-lane transpose on the path).
// Loads for tile t+1 are issued before tile t is consumed (registers are the staging
// buffer), indices one tile further ahead.
#include "common.h"

#include <mutex>
#include <type_traits>

namespace {

template <int D> struct Chunk;
template <> struct Chunk<128> { typedef u32x4 type; };
template <> struct Chunk<64> { typedef u32x2 type; };

__device__ __forceinline__ int nth_member(uint32_t mask, int n) {
  // position of the n-th set bit (n < popcount)
  int pos = 0;
#pragma unroll
  for (int i = 0; i < STS_MAX_GROUP; ++i) {
    const bool set = (mask >> i) & 1u;
    if (set && n == 0) pos = i;
    n -= set ? 1 : 0;
  }
  return pos;
}

__device__ __forceinline__ float xor_max(float x, int lanemask) {
  return fmaxf(x, __shfl_xor(x, lanemask, 64));
}

// One workgroup per CU (the whole register file for it) for exactly the variants the host plans
// one workgroup per CU for: four query tiles, and head size 128 when dense or with two query tiles.
// ROWMASK: every index entry comes with a 16-bit word, bit i set iff query row i of the block keeps
// the entry (prefill: an index set per query row, gathered once as their union).
template <int D, int NQ, bool SPARSE, bool LOGITS, bool PAGED, bool ROWMASK = false>
__global__ void __launch_bounds__(64 * STS_WG_WAVES, (NQ == 4 || (D == 128 && (!SPARSE || NQ == 2))) ? 1 : 2)
attn_split_kernel(const AttnArgs A) {
  typedef typename Chunk<D>::type chunk_t;
  constexpr int NT = D / 16;         // output tiles of the PV product == elements per lane chunk
  constexpr int KK = D / 32;         // contraction steps of the QK product
  constexpr int CHB = D / 8;         // bytes per lane chunk
  constexpr int ROWB = D * 2;        // bytes per K/V row
  constexpr int NSLOT = D / 8;       // 16-byte slots per LDS row
  constexpr int OPITCH = D + 4;      // floats per row of the merge buffer
  constexpr int KTILE_BYTES = STS_TILE_KEYS * ROWB;
  constexpr int MERGE_BYTES = STS_WG_WAVES * 16 * OPITCH * 4;
  constexpr int LDS_MAIN = (STS_WG_WAVES * KTILE_BYTES > MERGE_BYTES) ? STS_WG_WAVES * KTILE_BYTES : MERGE_BYTES;
  __shared__ __attribute__((aligned(16))) unsigned char lds[LDS_MAIN];
  __shared__ float lds_ml[STS_WG_WAVES][NQ * 16][2];
  // With two or more query tiles the Q operands (NQ*KK registers quads per lane) no longer fit
  // beside the accumulators and the load buffers: they live in LDS, already in MFMA B layout
  // (one 16-byte slot per lane and (tile, step)), and are re-read for every key tile.
  constexpr bool QLDS = NQ >= 2;
  __shared__ __attribute__((aligned(16))) u32x4 ldsQ[QLDS ? NQ * (D / 32) * 64 : 1];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int a = lane >> 4, b = lane & 15;

  const int S = A.num_splits, U = A.num_units;
  const int split = blockIdx.x % S;
  const int u = (blockIdx.x / S) % U;
  const int bt = blockIdx.x / (S * U);
  const uint32_t unit = A.units.unit[u];
  const int g = unit & 0xff;
  const uint32_t mask = (unit >> 8) & 0xffff;
  const int nheads = (unit >> 24) & 0x1f;
  const int rows_valid = nheads * A.Tq;
  const int head0 = g * A.G + nth_member(mask, 0);

  // Length of this unit's key list in token positions. Sparse index entries stand for blocks
  // of `page` consecutive tokens (page = 1: single tokens), so entry e covers positions
  // e*page .. e*page+page-1 of the expanded list. The split boundaries come from the static
  // upper bound (kmax*page or N), so the first index load below does not wait for the count;
  // a unit with fewer keys simply leaves its last splits empty (the longest unit sets the
  // makespan).
  const int psh = A.page_shift, pmask = A.page - 1;
  int c;
  if (SPARSE) {
    c = A.counts ? A.counts[(size_t)bt * A.cnt_stride_b + head0] : A.kmax;
    c = min(max(c, 0), A.kmax) << psh;
  } else {
    c = A.seq_lens ? A.seq_lens[bt] : A.N;
    c = min(max(c, 0), A.N);
  }
  const int len_max = SPARSE ? (A.kmax << psh) : A.N;
  const int tiles_max = (len_max + STS_TILE_KEYS - 1) / STS_TILE_KEYS;
  const int tps = (tiles_max + S - 1) / S;
  const int t_begin = split * tps;
  const int32_t *idx_row = SPARSE ? A.indices + (size_t)bt * A.idx_stride_b + (size_t)head0 * A.kmax : nullptr;
  // first tile's index entries, issued before anything depends on the count (kmax >= 1
  // whenever a sparse grid has tiles to do; the clamp keeps the address inside the row)
  const uint16_t *mask_row = ROWMASK ? A.row_mask + (size_t)bt * A.idx_stride_b + (size_t)head0 * A.kmax : nullptr;
  int rows_first = 0, bits_first = 0;
  if (SPARSE && len_max > 0) {
    rows_first = idx_row[min(((t_begin + wave) * STS_TILE_KEYS + (lane & 31)) >> psh, A.kmax - 1)];
    if (ROWMASK) bits_first = mask_row[min(((t_begin + wave) * STS_TILE_KEYS + (lane & 31)) >> psh, A.kmax - 1)];
  }
  const int tiles_total = (c + STS_TILE_KEYS - 1) / STS_TILE_KEYS;
  const int t_end = min(t_begin + tps, tiles_total);
  const int nb_max = (A.N + A.page - 1) >> psh;   // logical blocks of the cache

  // query rows owned by this lane: row nq*16 + b
  int q_head[NQ], q_tq[NQ];
  bool q_ok[NQ];
  bf16x8 Q[QLDS ? 1 : NQ][QLDS ? 1 : KK];
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    const int r = nq * 16 + b;
    q_ok[nq] = r < rows_valid;
    const int hsel = q_ok[nq] ? r / A.Tq : 0;
    q_tq[nq] = q_ok[nq] ? r - hsel * A.Tq : 0;
    q_head[nq] = g * A.G + nth_member(mask, hsel);
    const uint16_t *qp = A.q + (((size_t)bt * A.Tq + q_tq[nq]) * A.Hq + q_head[nq]) * D;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      u32x4 w = {0u, 0u, 0u, 0u};
      if (q_ok[nq]) w = *reinterpret_cast<const u32x4 *>(qp + 8 * (a + 4 * kk));
      if (QLDS) {
        if (wave == 0) ldsQ[(nq * KK + kk) * 64 + lane] = w;   // identical for every wave
      } else {
        Q[nq][kk] = __builtin_bit_cast(bf16x8, w);
      }
    }
  }
  if (QLDS) __syncthreads();

  // a paged cache is a pool of pages shared by the batch: the page table supplies the batch part
  const int64_t head_off = ((PAGED ? 0 : (int64_t)bt * A.stride_b) + (int64_t)g * A.stride_h) * 2 + b * CHB;
  const unsigned char *kbase = reinterpret_cast<const unsigned char *>(A.k) + head_off;
  const unsigned char *vbase = reinterpret_cast<const unsigned char *>(A.v) + head_off;
  const int64_t row_bytes = A.stride_n * 2;
  const int64_t page_bytes = A.stride_page * 2;
  const int32_t *table_row = PAGED ? A.block_table + (size_t)bt * A.table_stride : nullptr;
  unsigned char *ldsK = lds + wave * KTILE_BYTES;

  // row slot of load m for this lane: 16*(m/4) + 4a + m%4 (the keys the MFMA output hands
  // to lane group a)
  auto slot_of = [&](int m) { return 16 * (m >> 2) + 4 * a + (m & 3); };

  // Three prefetch stages per tile, each one loop half ahead of the next, so that no stage
  // waits on a load that was issued after the K/V loads in flight:
  //   fetch   : raw index entry (sparse) or logical block (dense) for slot (lane & 31);
  //   resolve : validity mask of the tile (one bit per slot) and the row to read: the token
  //             id, or with a page table the physical page (a second, dependent load);
  //   issue   : the 16 K/V row loads of the tile.
  // All three are branch-free and nothing touches a loaded value before the next stage.
  const int safe_pos = (LOGITS ? t_begin + 2 * wave : t_begin + wave) * STS_TILE_KEYS;
  auto fetch_rows = [&](int t) -> int {
    const int pos = t * STS_TILE_KEYS + (lane & 31);
    const int p = (t < t_end) ? min(pos, c - 1) : safe_pos;
    const int e = p >> psh;
    return SPARSE ? idx_row[e] : e;
  };
  // the row bits of the same entry (ROWMASK only)
  auto fetch_bits = [&](int t) -> int {
    const int pos = t * STS_TILE_KEYS + (lane & 31);
    const int p = (t < t_end) ? min(pos, c - 1) : safe_pos;
    return ROWMASK ? (int)mask_row[p >> psh] : 0;
  };

  auto resolve = [&](int raw, int t, uint32_t &tile_mask) -> int {
    const int pos = t * STS_TILE_KEYS + (lane & 31);
    const int blk = min(max(raw, 0), nb_max - 1);      // memory safety for arbitrary entries
    const int tok = (blk << psh) + (pos & pmask);
    // past the list, past the tile range, or in the unfilled part of the last page
    const bool ok = (t < t_end) && (pos < c) && (tok < A.N);
    tile_mask = (uint32_t)__ballot(ok);
    if (PAGED) return table_row[min(blk, A.table_stride - 1)];
    return min(tok, A.N - 1);
  };
  // row bits of this lane's slot, cleared where the slot holds no key
  auto slot_bits = [&](int bits, uint32_t tile_mask) -> int {
    return ((tile_mask >> (lane & 31)) & 1u) ? bits : 0;
  };

  auto issue_loads = [&](int x, int t, chunk_t (&Kr)[8], chunk_t (&Vr)[8]) {
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const int slot = slot_of(m);
      int64_t off;
      if (!SPARSE && !PAGED) {
        // contiguous dense cache: the row is the position itself, no cross-lane traffic
        const int row = (t < t_end) ? min(t * STS_TILE_KEYS + slot, c - 1) : 0;
        off = (int64_t)row * row_bytes;
      } else {
        int X = __shfl(x, slot, 64);
        if (PAGED) {
          X = min(max(X, 0), A.num_pages - 1);
          off = (int64_t)X * page_bytes + (int64_t)(slot & pmask) * row_bytes;
        } else {
          off = (int64_t)X * row_bytes;
        }
      }
      // every K/V row is consumed once per launch: stream it past the caches
      Kr[m] = __builtin_nontemporal_load(reinterpret_cast<const chunk_t *>(kbase + off));
      Vr[m] = __builtin_nontemporal_load(reinterpret_cast<const chunk_t *>(vbase + off));
    }
  };

  float m_run[NQ], l_run[NQ];
  f32x4 acc[NQ][NT];
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    m_run[nq] = -INFINITY;
    l_run[nq] = 0.f;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[nq][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // bf16 dump: the words of the first tile of a pair wait here for the second one, so that both
  // halves of every 128-byte line of a logits row are stored back to back (a half-line write
  // costs the memory system as much as a whole line)
  u32x2 stash[NQ][2];
  int stash_pos = -1;            // first token of the stashed tile, or -1
  auto store_bf16_tile = [&](const u32x2 (&w)[NQ][2], int pos0) {
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
      if (!q_ok[nq]) continue;
      uint16_t *lp = static_cast<uint16_t *>(A.logits_out) +
                     (((size_t)bt * A.Hq + q_head[nq]) * A.Tq + q_tq[nq]) * (size_t)A.N;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const int p = pos0 + 16 * ks + 4 * a;
        if (p + 3 < c && (A.N & 3) == 0) {
          *reinterpret_cast<u32x2 *>(lp + p) = w[nq][ks];
        } else {
          const uint16_t h4[4] = {(uint16_t)(w[nq][ks][0] & 0xffffu), (uint16_t)(w[nq][ks][0] >> 16),
                                  (uint16_t)(w[nq][ks][1] & 0xffffu), (uint16_t)(w[nq][ks][1] >> 16)};
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (p + r < c) lp[p + r] = h4[r];
        }
      }
    }
  };

  auto consume = [&](int t, const chunk_t (&Kr)[8], const chunk_t (&Vr)[8], const uint32_t tile_mask, const bool second,
                     const int tile_bits) {
    const int pos0 = t * STS_TILE_KEYS;
    // ---- K: registers -> swizzled LDS tile (row = slot, 16-byte slot index XOR row)
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const int row = slot_of(m);
      if (D == 128) {
        const int sl = b ^ (row & (NSLOT - 1));
        *reinterpret_cast<chunk_t *>(ldsK + row * ROWB + sl * 16) = Kr[m];
      } else {
        const int sl = (b >> 1) ^ (row & (NSLOT - 1));
        *reinterpret_cast<chunk_t *>(ldsK + row * ROWB + sl * 16 + (b & 1) * 8) = Kr[m];
      }
    }
    // ---- S^T = K Q^T
    f32x4 St[NQ][2];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) St[nq][0] = St[nq][1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      bf16x8 Ka[2];
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const int row = 16 * ks + b;
        const int sl = (a + 4 * kk) ^ (row & (NSLOT - 1));
        Ka[ks] = *reinterpret_cast<const bf16x8 *>(ldsK + row * ROWB + sl * 16);
      }
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq) {
        const bf16x8 Qb = QLDS ? __builtin_bit_cast(bf16x8, ldsQ[(nq * KK + kk) * 64 + lane]) : Q[QLDS ? 0 : nq][QLDS ? 0 : kk];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
          St[nq][ks] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Ka[ks], Qb, St[nq][ks], 0, 0, 0);
      }
    }
    if constexpr (LOGITS) {
      if (A.logits_bf16) {
        u32x2 w[NQ][2];
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
          for (int ks = 0; ks < 2; ++ks) {
            const f32x4 sc = St[nq][ks] * A.scale;
            const bf16x2 lo = __builtin_convertvector(f32x2{sc[0], sc[1]}, bf16x2);   // round to nearest even
            const bf16x2 hi = __builtin_convertvector(f32x2{sc[2], sc[3]}, bf16x2);
            w[nq][ks] = u32x2{__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
          }
        if (!second) {
#pragma unroll
          for (int nq = 0; nq < NQ; ++nq) {
            stash[nq][0] = w[nq][0];
            stash[nq][1] = w[nq][1];
          }
          stash_pos = pos0;
        } else {
          if (stash_pos >= 0) store_bf16_tile(stash, stash_pos);
          stash_pos = -1;
          store_bf16_tile(w, pos0);
        }
      } else {
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
          if (!q_ok[nq]) continue;
          float *lp = static_cast<float *>(A.logits_out) +
                      (((size_t)bt * A.Hq + q_head[nq]) * A.Tq + q_tq[nq]) * (size_t)A.N;
#pragma unroll
          for (int ks = 0; ks < 2; ++ks) {
            const int p = pos0 + 16 * ks + 4 * a;
            const f32x4 sc = St[nq][ks] * A.scale;
            if (p + 3 < c && (A.N & 3) == 0) {
              *reinterpret_cast<f32x4 *>(lp + p) = sc;
            } else {
#pragma unroll
              for (int r = 0; r < 4; ++r)
                if (p + r < c) lp[p + r] = sc[r];
            }
          }
        }
      }
    }
    // ---- online softmax (log2 domain) and P^T as bf16 B operands, then O^T += V^T P^T.
    // With four query tiles at head size 128 the two steps are done for two tiles at a time (the
    // V operands are permuted twice): all four P tiles next to both K/V buffers do not fit the
    // 256 registers that ordinary instructions can address.
    constexpr int NQH = (NQ == 4 && D == 128) ? 2 : NQ;   // query tiles per round
    int key_bits[8];                // ROWMASK: the row bits of this lane's 8 keys
    if constexpr (ROWMASK) {
#pragma unroll
      for (int m = 0; m < 8; ++m) key_bits[m] = __shfl(tile_bits, slot_of(m), 64);
    }
#pragma unroll
    for (int q0 = 0; q0 < NQ; q0 += NQH) {
      bf16x8 Pb[NQH];
#pragma unroll
      for (int nq = q0; nq < q0 + NQH; ++nq) {
        float s[8];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const bool ok = ROWMASK ? ((key_bits[4 * ks + r] >> q_tq[nq]) & 1) != 0
                                    : ((tile_mask >> (16 * ks + 4 * a + r)) & 1u) != 0;
            s[4 * ks + r] = ok ? St[nq][ks][r] * A.scale_log2 : -INFINITY;
          }
        float mt = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
        mt = xor_max(mt, 16);
        mt = xor_max(mt, 32);
        const float m_new = fmaxf(m_run[nq], mt);          // finite: every consumed tile has a valid key ...
        // ... except with row bits: a row may keep none of a tile's keys, nor of any tile so far
        const float m_ref = (ROWMASK && m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run[nq] - m_ref);
        float p[8], psum = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          p[i] = __builtin_amdgcn_exp2f(s[i] - m_ref);
          psum += p[i];
        }
        l_run[nq] = l_run[nq] * alpha + psum;
        m_run[nq] = m_new;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[nq][nt] *= alpha;
        u32x4 pw;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const f32x2 pr = {p[2 * i], p[2 * i + 1]};
          pw[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
        }
        Pb[nq - q0] = __builtin_bit_cast(bf16x8, pw);
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const uint32_t sel = (nt & 1) ? 0x07060302u : 0x05040100u;
        u32x4 vw;
#pragma unroll
        for (int j = 0; j < 4; ++j)
          vw[j] = __builtin_amdgcn_perm(Vr[2 * j + 1][nt >> 1], Vr[2 * j][nt >> 1], sel);
        const bf16x8 Va = __builtin_bit_cast(bf16x8, vw);
#pragma unroll
        for (int nq = q0; nq < q0 + NQH; ++nq)
          acc[nq][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Va, Pb[nq - q0], acc[nq][nt], 0, 0, 0);
      }
    }
  };

  // ---- main loop over this wave's tiles. Wave w takes tiles t_begin + w, + 4, + 8, ...; the
  // kernels that dump the logits take pairs of neighbouring tiles instead (2w, 2w + 1, then + 8),
  // so that one wave writes whole 128-byte lines of the dump.
  constexpr int W = STS_WG_WAVES;
  auto tile_of = [&](int v) -> int {
    return LOGITS ? t_begin + (v >> 1) * (2 * W) + 2 * wave + (v & 1) : t_begin + wave + v * W;
  };
  if (tile_of(0) < t_end) {   // wave-uniform; a wave without tiles touches no memory
    chunk_t K0[8], V0[8], K1[8], V1[8];
    uint32_t m0, m1, mk_next, mk_new;
    int b0 = 0, b1 = 0, bk_next = 0, bk_new = 0;   // ROWMASK: the tiles' row bits, staged like the masks
    int v = 0;
    // prologue: tile v in flight, tile v+1 resolved, tile v+2 fetched
    // The first tile's K/V loads go out as soon as its own index entries are there: the entries of
    // the second tile are asked for before them (so that waiting for those entries later does not
    // wait for the K/V rows, which return in order), but not waited for.
    int raw_a = SPARSE ? rows_first : fetch_rows(tile_of(0));
    int rbits_a = ROWMASK ? bits_first : 0;
    int raw_b = fetch_rows(tile_of(1));
    int rbits_b = fetch_bits(tile_of(1));
    int x_a = resolve(raw_a, tile_of(0), m0);
    if (ROWMASK) b0 = slot_bits(rbits_a, m0);
    if (SPARSE) __builtin_amdgcn_sched_barrier(0);
    issue_loads(x_a, tile_of(0), K0, V0);
    if (SPARSE) __builtin_amdgcn_sched_barrier(0);
    raw_a = fetch_rows(tile_of(2));
    rbits_a = fetch_bits(tile_of(2));
    int x_b = resolve(raw_b, tile_of(1), mk_next);
    if (ROWMASK) bk_next = slot_bits(rbits_b, mk_next);
    if (SPARSE) __builtin_amdgcn_sched_barrier(0);
    for (;;) {
      raw_b = fetch_rows(tile_of(v + 3));
      rbits_b = fetch_bits(tile_of(v + 3));
      x_a = resolve(raw_a, tile_of(v + 2), mk_new);
      if (ROWMASK) bk_new = slot_bits(rbits_a, mk_new);
      if (SPARSE) __builtin_amdgcn_sched_barrier(0);   // index traffic stays ahead of the K/V loads
      issue_loads(x_b, tile_of(v + 1), K1, V1);
      m1 = mk_next;
      b1 = bk_next;
      if (SPARSE) __builtin_amdgcn_sched_barrier(0);   // loads are in flight before the tile is consumed
      consume(tile_of(v), K0, V0, m0, false, b0);      // even step: first tile of a pair
      mk_next = mk_new;
      bk_next = bk_new;
      ++v;
      if (tile_of(v) >= t_end) break;
      raw_a = fetch_rows(tile_of(v + 3));
      rbits_a = fetch_bits(tile_of(v + 3));
      x_b = resolve(raw_b, tile_of(v + 2), mk_new);
      if (ROWMASK) bk_new = slot_bits(rbits_b, mk_new);
      if (SPARSE) __builtin_amdgcn_sched_barrier(0);
      issue_loads(x_a, tile_of(v + 1), K0, V0);
      m0 = mk_next;
      b0 = bk_next;
      if (SPARSE) __builtin_amdgcn_sched_barrier(0);
      consume(tile_of(v), K1, V1, m1, true, b1);       // odd step: second tile of the pair
      mk_next = mk_new;
      bk_next = bk_new;
      ++v;
      if (tile_of(v) >= t_end) break;
    }
    if (LOGITS && stash_pos >= 0) store_bf16_tile(stash, stash_pos);   // a range that ends on a first tile
  }

  // ---- merge the 4 waves, write one partial per workgroup
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    float l = l_run[nq];
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    l_run[nq] = l;
    if (a == 0) {
      lds_ml[wave][nq * 16 + b][0] = m_run[nq];
      lds_ml[wave][nq * 16 + b][1] = l;
    }
  }
  __syncthreads();   // K staging is dead from here on; lds_ml visible
  float *Om = reinterpret_cast<float *>(lds);
  const size_t pidx = ((size_t)bt * U + u) * S + split;
  float *po = A.part_o + pidx * (size_t)(NQ * 16 * D);
  float *pml = A.part_ml + pidx * (size_t)(NQ * 16 * 2);
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    float mstar = -INFINITY;
#pragma unroll
    for (int w = 0; w < STS_WG_WAVES; ++w) mstar = fmaxf(mstar, lds_ml[w][nq * 16 + b][0]);
    const float f = (m_run[nq] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m_run[nq] - mstar);
    float *orow = Om + (wave * 16 + b) * OPITCH;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int d0 = NT * (4 * a + r);
#pragma unroll
      for (int v4 = 0; v4 < NT / 4; ++v4) {
        f32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = acc[nq][4 * v4 + e][r] * f;
        *reinterpret_cast<f32x4 *>(orow + d0 + 4 * v4) = o;
      }
    }
    __syncthreads();
    {
      // 256 threads: row = tid / 16, D/16 consecutive floats each
      const int row = threadIdx.x >> 4, seg = threadIdx.x & 15;
      constexpr int SEGF = D / 16;
      float sum[SEGF];
#pragma unroll
      for (int e = 0; e < SEGF; ++e) sum[e] = 0.f;
#pragma unroll
      for (int w = 0; w < STS_WG_WAVES; ++w) {
        const float *src = Om + (w * 16 + row) * OPITCH + seg * SEGF;
#pragma unroll
        for (int e = 0; e < SEGF; e += 4) {
          const f32x4 x = *reinterpret_cast<const f32x4 *>(src + e);
          sum[e] += x[0]; sum[e + 1] += x[1]; sum[e + 2] += x[2]; sum[e + 3] += x[3];
        }
      }
      if (A.direct) {
        // single split: this workgroup holds the whole result of its
        // rows, so it normalises and writes them itself and no combine kernel is launched
        const int r = nq * 16 + row;
        if (r < rows_valid) {
          float ms = -INFINITY;
#pragma unroll
          for (int w = 0; w < STS_WG_WAVES; ++w) ms = fmaxf(ms, lds_ml[w][r][0]);
          float L = 0.f;
#pragma unroll
          for (int w = 0; w < STS_WG_WAVES; ++w) {
            const float mw = lds_ml[w][r][0];
            L += (mw == -INFINITY) ? 0.f : lds_ml[w][r][1] * __builtin_amdgcn_exp2f(mw - ms);
          }
          const int hsel = r / A.Tq, tq = r - hsel * A.Tq;
          const int head = g * A.G + nth_member(mask, hsel);
          // The speculative block's own tokens (see the combine kernel, which does the same for
          // split lists): candidate tq also attends to candidates 0..tq, merged here like one more
          // partial each, in order. The 16 threads of a row hold D/16 channels each.
          if (A.k_new) {
            typedef typename Chunk<D>::type seg_t;          // D/16 bf16 values = 16 or 8 bytes
            auto widen = [](uint32_t w, int hi) -> float {
              return __builtin_bit_cast(float, hi ? (w & 0xffff0000u) : (w << 16));
            };
            const seg_t qw = *reinterpret_cast<const seg_t *>(A.q + (((size_t)bt * A.Tq + tq) * A.Hq + head) * D + seg * SEGF);
            const int nnew = A.causal ? tq + 1 : A.Tq;
            for (int j = 0; j < nnew; ++j) {               // the 16 threads of a row share nnew
              const size_t nrow = (((size_t)bt * A.Tq + j) * A.Hkv + g) * D + seg * SEGF;
              const seg_t kw = *reinterpret_cast<const seg_t *>(A.k_new + nrow);
              const seg_t vw = *reinterpret_cast<const seg_t *>(A.v_new + nrow);
              float dot = 0.f;
#pragma unroll
              for (int e = 0; e < SEGF; ++e) dot += widen(qw[e >> 1], e & 1) * widen(kw[e >> 1], e & 1);
              dot += __shfl_xor(dot, 1, 64);
              dot += __shfl_xor(dot, 2, 64);
              dot += __shfl_xor(dot, 4, 64);
              dot += __shfl_xor(dot, 8, 64);
              const float m2 = dot * A.scale_log2;
              const float mnew = fmaxf(ms, m2);
              const float fo = __builtin_amdgcn_exp2f(ms - mnew);   // 0 while nothing is accumulated
              const float fn = __builtin_amdgcn_exp2f(m2 - mnew);
              L = L * fo + fn;
#pragma unroll
              for (int e = 0; e < SEGF; ++e) sum[e] = sum[e] * fo + widen(vw[e >> 1], e & 1) * fn;
              ms = mnew;
            }
          }
          const float inv = (L > 0.f) ? 1.f / L : 0.f;
          const size_t orow = (((size_t)bt * A.Tq + tq) * A.Hq + head) * D + seg * SEGF;
          if (A.out_dtype == STS_F32) {
            float *dst = reinterpret_cast<float *>(A.out) + orow;
#pragma unroll
            for (int e = 0; e < SEGF; e += 4)
              *reinterpret_cast<f32x4 *>(dst + e) =
                  f32x4{sum[e] * inv, sum[e + 1] * inv, sum[e + 2] * inv, sum[e + 3] * inv};
          } else {
            uint32_t *dst = reinterpret_cast<uint32_t *>(reinterpret_cast<uint16_t *>(A.out) + orow);
#pragma unroll
            for (int e = 0; e < SEGF; e += 2) {
              const f32x2 pr = {sum[e] * inv, sum[e + 1] * inv};
              dst[e >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
            }
          }
          if (A.lse_out && seg == 0) {
            const float ln2 = 0.69314718055994530942f;
            A.lse_out[((size_t)bt * A.Hq + head) * A.Tq + tq] =
                (L > 0.f) ? (ms + __builtin_amdgcn_logf(L)) * ln2 : -INFINITY;
          }
        }
      } else {
      float *dst = po + (size_t)(nq * 16 + row) * D + seg * SEGF;
#pragma unroll
      for (int e = 0; e < SEGF; e += 4)
        *reinterpret_cast<f32x4 *>(dst + e) = f32x4{sum[e], sum[e + 1], sum[e + 2], sum[e + 3]};
      if (threadIdx.x < 16) {
        const int r = nq * 16 + threadIdx.x;
        float ms = -INFINITY;
#pragma unroll
        for (int w = 0; w < STS_WG_WAVES; ++w) ms = fmaxf(ms, lds_ml[w][r][0]);
        float L = 0.f;
#pragma unroll
        for (int w = 0; w < STS_WG_WAVES; ++w) {
          const float mw = lds_ml[w][r][0];
          L += (mw == -INFINITY) ? 0.f : lds_ml[w][r][1] * __builtin_amdgcn_exp2f(mw - ms);
        }
        pml[r * 2 + 0] = ms;
        pml[r * 2 + 1] = L;
      }
      }
    }
    __syncthreads();
  }
}

// Combine the per-split partials and write the final rows. One workgroup of 256 threads per
// (batch, unit, query tile, group of 4 rows): wave w merges the splits w, w+4, w+8, ... of its
// 4 rows (thread = row, D/16 channels; loads in independent batches), the four waves are then
// merged through LDS in wave order by wave 0, which writes the result; the block's own tokens
// enter as the first entries of wave 3's share. The order of all merges is fixed, so results are identical run to run.
template <int D>
__global__ void __launch_bounds__(256) attn_combine_kernel(const AttnArgs A, const int NQ) {
  constexpr int SEGF = D / 16;
  constexpr int BATCH = 4;
  __shared__ float sm_ml[4][4][2];
  __shared__ __attribute__((aligned(16))) float sm_o[4][4][D];
  const int S = A.num_splits, U = A.num_units;
  const int quarter = blockIdx.x & 3;
  const int nq = (blockIdx.x >> 2) % NQ;
  const int u = ((blockIdx.x >> 2) / NQ) % U;
  const int bt = (blockIdx.x >> 2) / (NQ * U);
  const uint32_t unit = A.units.unit[u];
  const int g = unit & 0xff;
  const uint32_t mask = (unit >> 8) & 0xffff;
  const int nheads = (unit >> 24) & 0x1f;
  const int wave = threadIdx.x >> 6, row4 = (threadIdx.x >> 4) & 3, seg = threadIdx.x & 15;
  const int r = nq * 16 + quarter * 4 + row4;
  if (nq * 16 + quarter * 4 >= nheads * A.Tq) return;          // whole workgroup has no valid row
  const bool valid = r < nheads * A.Tq;
  const int rr = valid ? r : nq * 16 + quarter * 4;             // padding rows mirror a valid one
  const size_t p0 = ((size_t)bt * U + u) * S;
  const size_t rows_per = (size_t)NQ * 16;

  float mstar = -INFINITY, L = 0.f;
  float o[SEGF];
#pragma unroll
  for (int e = 0; e < SEGF; ++e) o[e] = 0.f;
  auto merge = [&](float ms, float ls, const float *x) {
    if (ms == -INFINITY) return;
    const float mnew = fmaxf(mstar, ms);
    const float fo = __builtin_amdgcn_exp2f(mstar - mnew);   // 0 while nothing is accumulated
    const float fn = __builtin_amdgcn_exp2f(ms - mnew);
    L = L * fo + ls * fn;
#pragma unroll
    for (int e = 0; e < SEGF; ++e) o[e] = o[e] * fo + x[e] * fn;
    mstar = mnew;
  };
  // The speculative block's own tokens: candidate tq also attends to candidates 0..tq (all of
  // them when not causal). They are the first entries of the last wave's share, so their loads
  // go out together with the partials' and add no latency of their own. The 16 threads of a row
  // each hold D/16 channels: partial dot products are summed across the row's 16 lanes, then
  // every token is merged like one more partial, in order.
  if (A.k_new && wave == 3 && valid) {
    const int hsel_t = r / A.Tq, tq_t = r - hsel_t * A.Tq;
    const int head_t = g * A.G + nth_member(mask, hsel_t);
    typedef typename Chunk<D>::type seg_t;          // D/16 bf16 values = 16 or 8 bytes
    auto widen = [](uint32_t w, int hi) -> float {
      return __builtin_bit_cast(float, hi ? (w & 0xffff0000u) : (w << 16));
    };
    const seg_t qw = *reinterpret_cast<const seg_t *>(A.q + (((size_t)bt * A.Tq + tq_t) * A.Hq + head_t) * D + seg * SEGF);
    const int nnew = A.causal ? tq_t + 1 : A.Tq;
    // all rows are asked for before the first one is used (a load per trip would cost a
    // memory latency per token)
    seg_t kw[16], vw[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      if (j < A.Tq) {                               // Tq <= 16
        const size_t nrow = (((size_t)bt * A.Tq + j) * A.Hkv + g) * D + seg * SEGF;
        kw[j] = *reinterpret_cast<const seg_t *>(A.k_new + nrow);
        vw[j] = *reinterpret_cast<const seg_t *>(A.v_new + nrow);
      }
    }
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      if (j < nnew) {                               // the 16 threads of a row share nnew
        float dot = 0.f;
#pragma unroll
        for (int e = 0; e < SEGF; ++e) dot += widen(qw[e >> 1], e & 1) * widen(kw[j][e >> 1], e & 1);
        dot += __shfl_xor(dot, 1, 64);
        dot += __shfl_xor(dot, 2, 64);
        dot += __shfl_xor(dot, 4, 64);
        dot += __shfl_xor(dot, 8, 64);
        float vs[SEGF];
#pragma unroll
        for (int e = 0; e < SEGF; ++e) vs[e] = widen(vw[j][e >> 1], e & 1);
        merge(dot * A.scale_log2, 1.f, vs);
      }
    }
  }
  for (int s0 = wave; s0 < S; s0 += 4 * BATCH) {
    float ms[BATCH], ls[BATCH];
    f32x4 x[BATCH][SEGF / 4];
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {
      const int sj = min(s0 + 4 * j, S - 1);
      const size_t pr = (p0 + sj) * rows_per + rr;
      ms[j] = (s0 + 4 * j < S) ? A.part_ml[pr * 2] : -INFINITY;
      ls[j] = A.part_ml[pr * 2 + 1];
      const float *src = A.part_o + pr * D + seg * SEGF;
#pragma unroll
      for (int e = 0; e < SEGF / 4; ++e) x[j][e] = *reinterpret_cast<const f32x4 *>(src + 4 * e);
    }
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {
      float xs[SEGF];
#pragma unroll
      for (int e = 0; e < SEGF; ++e) xs[e] = x[j][e >> 2][e & 3];
      merge(ms[j], ls[j], xs);
    }
  }
  if (seg == 0) {
    sm_ml[wave][row4][0] = mstar;
    sm_ml[wave][row4][1] = L;
  }
#pragma unroll
  for (int e = 0; e < SEGF; ++e) sm_o[wave][row4][seg * SEGF + e] = o[e];
  __syncthreads();
  if (wave != 0 || !valid) return;
  // wave 0 already holds its own share; fold in waves 1..3 in order
#pragma unroll
  for (int w = 1; w < 4; ++w) merge(sm_ml[w][row4][0], sm_ml[w][row4][1], &sm_o[w][row4][seg * SEGF]);

  const int hsel = r / A.Tq, tq = r - hsel * A.Tq;
  const int head = g * A.G + nth_member(mask, hsel);
  const float inv = (L > 0.f) ? 1.f / L : 0.f;
  const size_t orow = (((size_t)bt * A.Tq + tq) * A.Hq + head) * D + seg * SEGF;
  if (A.out_dtype == STS_F32) {
    float *dst = reinterpret_cast<float *>(A.out) + orow;
#pragma unroll
    for (int e = 0; e < SEGF; e += 4)
      *reinterpret_cast<f32x4 *>(dst + e) = f32x4{o[e] * inv, o[e + 1] * inv, o[e + 2] * inv, o[e + 3] * inv};
  } else {
    uint32_t *dst = reinterpret_cast<uint32_t *>(reinterpret_cast<uint16_t *>(A.out) + orow);
#pragma unroll
    for (int e = 0; e < SEGF; e += 2) {
      const f32x2 pr = {o[e] * inv, o[e + 1] * inv};
      dst[e >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
    }
  }
  if (A.lse_out && seg == 0) {
    const float ln2 = 0.69314718055994530942f;
    A.lse_out[((size_t)bt * A.Hq + head) * A.Tq + tq] =
        (L > 0.f) ? (mstar + __builtin_amdgcn_logf(L)) * ln2 : -INFINITY;
  }
}

template <int D, int NQ, bool PAGED>
hipError_t launch_split_dnp(const AttnArgs &a, bool sparse, hipStream_t s) {
  const dim3 grid((unsigned)((size_t)a.B * a.num_units * a.num_splits)), block(64 * STS_WG_WAVES);
  if (sparse && a.row_mask) {
    if constexpr (!PAGED) STS_LAUNCH((attn_split_kernel<D, NQ, true, false, false, true>), grid, block, 0, s, a);
    else return hipErrorInvalidValue;           // (the host refuses row bits on a paged cache)
  } else if (sparse)
    STS_LAUNCH((attn_split_kernel<D, NQ, true, false, PAGED>), grid, block, 0, s, a);
  else if (a.logits_out) {
    // the dump at head size 128 is planned with at most two query tiles per unit (its four-tile
    // form does not fit the register file)
    if constexpr (D == 128 && NQ == 4) return hipErrorInvalidValue;
    else STS_LAUNCH((attn_split_kernel<D, NQ, false, true, PAGED>), grid, block, 0, s, a);
  } else
    STS_LAUNCH((attn_split_kernel<D, NQ, false, false, PAGED>), grid, block, 0, s, a);
  return sts_take_launch_status();
}

template <int D, int NQ>
hipError_t launch_split_dn(const AttnArgs &a, bool sparse, hipStream_t s) {
  return a.block_table ? launch_split_dnp<D, NQ, true>(a, sparse, s)
                       : launch_split_dnp<D, NQ, false>(a, sparse, s);
}

template <int D>
hipError_t launch_split_d(const AttnArgs &a, int nq, bool sparse, hipStream_t s) {
  switch (nq) {
    case 1: return launch_split_dn<D, 1>(a, sparse, s);
    case 2: return launch_split_dn<D, 2>(a, sparse, s);
    case 4: return launch_split_dn<D, 4>(a, sparse, s);
  }
  return hipErrorInvalidValue;
}

// -------------------------------------------------- summed attention weights of a query block
// A second pass over K for the draft layer: agg[b, head, n] = sum over the Tq query rows, in row
// order, of exp(s[row, n] - lse[row]) -- the aggregate sts_select ranks (paper Section 4.3: one
// mask per speculative batch) -- without writing the Tq times larger logits to memory and
// reading them back. s comes from the same MFMA instruction on the same operands as in the
// logits dump (operands swapped, which transposes the result tile) and goes through the same
// fp32 arithmetic, so the result is bit for bit what the dump followed by the selection's own
// aggregation gives. One workgroup of 4 waves per (batch, KV head, set of heads, piece of the key
// range); dense, contiguous cache.
//
// Layout: S = Q K^T leaves lane (a, b) with rows 4a..4a+3 of a 16-row query tile for key b, so
// with Tq padded to a power of two Tp (padding rows weigh +0) a head's rows are registers of one
// lane (Tp <= 4) or of Tp/4 lanes 16 apart (Tp = 8, 16). The sum over rows is a left-to-right
// fold: inside the lane, then handed on from lane to lane (a fold along 16 lanes with shifted
// adds took more than twice the vector instructions per tile). What bounds the kernel is the
// memory system: a thin write stream mixed into the read stream.
template <int TP>
__device__ __forceinline__ void fold_rows(const float (&p)[4], float (&s)[4], int a) {
  constexpr int RPL = TP < 4 ? TP : 4;       // rows of one head held by a lane
  constexpr int HPL = 4 / RPL;               // heads per lane
  constexpr int CH = TP > 4 ? TP / 4 : 1;    // lanes a head's rows are spread over
#pragma unroll
  for (int j = 0; j < HPL; ++j) {
    s[j] = p[j * RPL];
#pragma unroll
    for (int i = 1; i < RPL; ++i) s[j] = s[j] + p[j * RPL + i];
  }
  if constexpr (CH > 1) {
    const int from = (((int)threadIdx.x - 16) & 63) << 2;   // the lane holding the four rows before mine
#pragma unroll
    for (int step = 1; step < CH; ++step) {
      float t = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(from, __builtin_bit_cast(int, s[0])));
#pragma unroll
      for (int i = 0; i < 4; ++i) t = t + p[i];
      s[0] = ((a & (CH - 1)) == step) ? t : s[0];
    }
  }
}

template <int D, int NQ>
__global__ void __launch_bounds__(64 * STS_WG_WAVES) attn_probsum_kernel(const AttnArgs A) {
  typedef typename Chunk<D>::type chunk_t;
  constexpr int KK = D / 32;
  constexpr int CHB = D / 8;
  constexpr int ROWB = D * 2;
  constexpr int NSLOT = D / 8;
  constexpr int KTILE_BYTES = STS_TILE_KEYS * ROWB;
  constexpr int W = STS_WG_WAVES;
  constexpr int PS_STAGES = 3;
  __shared__ __attribute__((aligned(16))) unsigned char ldsK_all[W * KTILE_BYTES];
  __shared__ __attribute__((aligned(16))) u32x4 ldsQ[NQ * KK * 64];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: tile addresses stay wave-uniform
  const int a = lane >> 4, b = lane & 15;
  const int S = A.ps_splits;
  const int split = blockIdx.x % S;
  const int set = (blockIdx.x / S) % A.ps_sets;
  const int g = (blockIdx.x / (S * A.ps_sets)) % A.Hkv;
  const int bt = blockIdx.x / (S * A.ps_sets * A.Hkv);
  const int Tp = A.ps_tp;                                // Tq rounded up to a power of two, <= 16
  const int tp_shift = 31 - __builtin_clz(Tp);
  const int h0 = set * A.ps_heads;                       // first head of the set handled here
  const int nh = min(A.ps_heads, A.G - h0);
  int c = A.seq_lens ? A.seq_lens[bt] : A.N;
  c = min(max(c, 0), A.N);
  const int tiles_all = (A.N + STS_TILE_KEYS - 1) / STS_TILE_KEYS;   // every key position gets a value
  const int tps = (tiles_all + S - 1) / S;
  const int t_begin = split * tps;
  const int t_end = min(t_begin + tps, tiles_all);

  // Q tiles into LDS in the MFMA operand layout (lane (a, b): row b, channels 8(a + 4kk)..)
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    const int r = nq * 16 + b;
    const int hsel = r >> tp_shift, tq = r & (Tp - 1);
    const bool ok = hsel < nh && tq < A.Tq;
    const uint16_t *qp = A.q + (((size_t)bt * A.Tq + (ok ? tq : 0)) * A.Hq + g * A.G + h0 + (ok ? hsel : 0)) * D;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      u32x4 w = {0u, 0u, 0u, 0u};
      if (ok) w = *reinterpret_cast<const u32x4 *>(qp + 8 * (a + 4 * kk));
      if (wave == 0) ldsQ[(nq * KK + kk) * 64 + lane] = w;
    }
  }
  // normalisers of the rows this lane holds after the MFMA: 4a..4a+3 of every query tile.
  // +inf for padding rows: their logits are 0 (zero Q rows), so their weights come out as +0.
  float lse_r[NQ][4];
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = nq * 16 + 4 * a + r;
      const int hsel = row >> tp_shift, tq = row & (Tp - 1);
      const bool ok = hsel < nh && tq < A.Tq;
      lse_r[nq][r] = ok ? A.lse_out[((size_t)bt * A.Hq + g * A.G + h0 + hsel) * A.Tq + tq] : INFINITY;
    }
  __syncthreads();

  // addresses: a wave-uniform base per tile plus a 32-bit lane offset (the host checks that it fits)
  const unsigned char *kuni = reinterpret_cast<const unsigned char *>(A.k) +
                              ((int64_t)bt * A.stride_b + (int64_t)g * A.stride_h) * 2;
  const int64_t row_bytes = A.stride_n * 2;
  const unsigned lane_off = (unsigned)(4 * a) * (unsigned)row_bytes + (unsigned)(b * CHB);
  unsigned char *ldsK = ldsK_all + wave * KTILE_BYTES;
  auto slot_of = [&](int m) { return 16 * (m >> 2) + 4 * a + (m & 3); };
  float *agg_set = A.agg_out + ((size_t)bt * A.Hq + g * A.G + h0) * (size_t)A.N;

  auto issue_loads = [&](int t, chunk_t (&Kr)[8]) {
    if (t >= t_end) return;        // wave-uniform: the slot is never consumed
    if ((t + 1) * STS_TILE_KEYS <= c) {
      const unsigned char *tb = kuni + (int64_t)t * STS_TILE_KEYS * row_bytes;
#pragma unroll
      for (int m = 0; m < 8; ++m)
        Kr[m] = __builtin_nontemporal_load(
            reinterpret_cast<const chunk_t *>(tb + (int64_t)(16 * (m >> 2) + (m & 3)) * row_bytes + lane_off));
    } else {                       // the tile holding the end of the sequence, and tiles past it
#pragma unroll
      for (int m = 0; m < 8; ++m) {
        const int row = c > 0 ? min(t * STS_TILE_KEYS + slot_of(m), c - 1) : 0;
        Kr[m] = __builtin_nontemporal_load(
            reinterpret_cast<const chunk_t *>(kuni + (int64_t)row * row_bytes + b * CHB));
      }
    }
  };

  // weights of the tile, folded over each head's rows; the lane at the end of a head's rows
  // holds the sums for keys b and 16 + b of the tile
  auto finish = [&](auto tp_c, const f32x4 (&Sq)[NQ][2], int pos0) {
    constexpr int TP = decltype(tp_c)::value;
    constexpr int HPL = TP >= 4 ? 1 : 4 / TP;
    constexpr int CH = TP > 4 ? TP / 4 : 1;
    constexpr int TPS = TP == 1 ? 0 : (TP == 2 ? 1 : (TP == 4 ? 2 : (TP == 8 ? 3 : 4)));
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
      float sum[2][4];
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
#pragma clang fp contract(off)   // the scaled logit is rounded before the subtraction, as in the dump
        float pr[4];
        const f32x4 sc = Sq[nq][ks] * A.scale;
#pragma unroll
        for (int r = 0; r < 4; ++r)
          pr[r] = __builtin_amdgcn_exp2f((sc[r] - lse_r[nq][r]) * 1.44269504088896340736f);
        fold_rows<TP>(pr, sum[ks], a);
      }
      // Stores. Lanes a and a^1 (16 apart) swap one half each, so that one store instruction
      // covers a head's whole 128-byte line with 32 lanes (a line written as two 64-byte halves
      // costs the memory system about three times as much). First the line of the even lane's
      // head, then the line of the odd lane's head; a lane pair whose lane is not the end of a
      // head's rows has nothing to store.
      const int odd = a & 1;
      const int pos = pos0 + 16 * odd + b;
      const bool in_row = pos < A.N;
      const bool live = pos < c;
#pragma unroll
      for (int j = 0; j < HPL; ++j) {
        const float mine = odd ? sum[0][j] : sum[1][j];
        const float theirs = __builtin_bit_cast(
            float, __builtin_amdgcn_ds_bpermute(((int)threadIdx.x ^ 16) << 2, __builtin_bit_cast(int, mine)));
        const int a_e = a & ~1, a_o = a | 1;
        const int head_e = ((nq * 16 + 4 * a_e) >> TPS) + j, head_o = ((nq * 16 + 4 * a_o) >> TPS) + j;
        if (CH == 1 && head_e < nh && in_row) {
          const float v = odd ? theirs : sum[0][j];
          agg_set[(size_t)head_e * (size_t)A.N + pos] = live ? v : 0.f;
        }
        if ((a_o & (CH - 1)) == CH - 1 && head_o < nh && in_row) {
          const float v = odd ? sum[1][j] : theirs;
          agg_set[(size_t)head_o * (size_t)A.N + pos] = live ? v : 0.f;
        }
      }
    }
  };

  auto consume = [&](int t, const chunk_t (&Kr)[8]) {
    const int pos0 = t * STS_TILE_KEYS;
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const int row = slot_of(m);
      if (D == 128) {
        const int sl = b ^ (row & (NSLOT - 1));
        *reinterpret_cast<chunk_t *>(ldsK + row * ROWB + sl * 16) = Kr[m];
      } else {
        const int sl = (b >> 1) ^ (row & (NSLOT - 1));
        *reinterpret_cast<chunk_t *>(ldsK + row * ROWB + sl * 16 + (b & 1) * 8) = Kr[m];
      }
    }
    // S = Q K^T: lane (a, b) gets rows 4a..4a+3 of each query tile for keys b and 16 + b
    f32x4 Sq[NQ][2];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) Sq[nq][0] = Sq[nq][1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      bf16x8 Ka[2];
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const int row = 16 * ks + b;
        const int sl = (a + 4 * kk) ^ (row & (NSLOT - 1));
        Ka[ks] = *reinterpret_cast<const bf16x8 *>(ldsK + row * ROWB + sl * 16);
      }
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq) {
        const bf16x8 Qb = __builtin_bit_cast(bf16x8, ldsQ[(nq * KK + kk) * 64 + lane]);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
          Sq[nq][ks] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Qb, Ka[ks], Sq[nq][ks], 0, 0, 0);
      }
    }
    switch (Tp) {
      case 1: finish(std::integral_constant<int, 1>(), Sq, pos0); break;
      case 2: finish(std::integral_constant<int, 2>(), Sq, pos0); break;
      case 4: finish(std::integral_constant<int, 4>(), Sq, pos0); break;
      case 8: finish(std::integral_constant<int, 8>(), Sq, pos0); break;
      default: finish(std::integral_constant<int, 16>(), Sq, pos0); break;
    }
  };

  // ring of PS_STAGES tiles in flight per wave
  if (t_begin + wave < t_end) {
    chunk_t Kst[PS_STAGES][8];
    int t = t_begin + wave;
#pragma unroll
    for (int u = 0; u < PS_STAGES - 1; ++u) issue_loads(t + u * W, Kst[u]);
    bool more = true;
    while (more) {
#pragma unroll
      for (int u = 0; u < PS_STAGES; ++u) {
        if (more) {
          issue_loads(t + (PS_STAGES - 1) * W, Kst[(u + PS_STAGES - 1) % PS_STAGES]);
          consume(t, Kst[u]);
          t += W;
          more = t < t_end;
        }
      }
    }
  }
}

}  // namespace

hipError_t launch_attn_split(const AttnArgs &a, int d, int nq, bool sparse, hipStream_t s) {
  if ((size_t)a.B * a.num_units * a.num_splits == 0) return hipSuccess;
  if (d == 128) return launch_split_d<128>(a, nq, sparse, s);
  if (d == 64) return launch_split_d<64>(a, nq, sparse, s);
  return hipErrorInvalidValue;
}

hipError_t launch_attn_combine(const AttnArgs &a, int d, int nq, hipStream_t s) {
  const size_t blocks = (size_t)a.B * a.num_units * nq * 4;   // 4 groups of 4 rows per query tile
  if (blocks == 0) return hipSuccess;
  const dim3 grid((unsigned)blocks), block(256);
  if (d == 128)
    STS_LAUNCH((attn_combine_kernel<128>), grid, block, 0, s, a, nq);
  else if (d == 64)
    STS_LAUNCH((attn_combine_kernel<64>), grid, block, 0, s, a, nq);
  else
    return hipErrorInvalidValue;
  return sts_take_launch_status();
}

// resident workgroups per CU of the second-pass kernel for this head size and query-tile count
// (register use differs a lot between the variants), asked from the runtime once per variant
int attn_probsum_wgs_per_cu(int d, int nq) {
  static std::mutex mu;
  static int cached[2][5] = {{0}};
  if ((d != 64 && d != 128) || (nq != 1 && nq != 2 && nq != 4)) return 1;
  std::lock_guard<std::mutex> lk(mu);
  int &slot = cached[d == 128][nq];
  if (slot == 0) {
    int n = 0;
    hipError_t rc = hipErrorInvalidValue;
#define STS_OCC(DD, QQ) rc = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, attn_probsum_kernel<DD, QQ>, 64 * STS_WG_WAVES, 0)
    if (d == 128 && nq == 1) STS_OCC(128, 1);
    else if (d == 128 && nq == 2) STS_OCC(128, 2);
    else if (d == 128 && nq == 4) STS_OCC(128, 4);
    else if (d == 64 && nq == 1) STS_OCC(64, 1);
    else if (d == 64 && nq == 2) STS_OCC(64, 2);
    else STS_OCC(64, 4);
#undef STS_OCC
    slot = (rc == hipSuccess && n > 0) ? n : 1;
  }
  return slot;
}

hipError_t launch_attn_probsum(const AttnArgs &a, int d, int nq, hipStream_t s) {
  const size_t blocks = (size_t)a.B * a.Hkv * a.ps_sets * a.ps_splits;
  if (blocks == 0) return hipSuccess;
  const dim3 grid((unsigned)blocks), block(64 * STS_WG_WAVES);
#define STS_PROBSUM(DD, QQ) STS_LAUNCH((attn_probsum_kernel<DD, QQ>), grid, block, 0, s, a)
  if (d == 128 && nq == 1) STS_PROBSUM(128, 1);
  else if (d == 128 && nq == 2) STS_PROBSUM(128, 2);
  else if (d == 128 && nq == 4) STS_PROBSUM(128, 4);
  else if (d == 64 && nq == 1) STS_PROBSUM(64, 1);
  else if (d == 64 && nq == 2) STS_PROBSUM(64, 2);
  else if (d == 64 && nq == 4) STS_PROBSUM(64, 4);
  else return hipErrorInvalidValue;
#undef STS_PROBSUM
  return sts_take_launch_status();
}
