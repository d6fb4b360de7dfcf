/* Host-side sanitizer driver for the oracle (test infrastructure): exercises every oracle
 * function on small inputs, including ragged and empty cases, under
 *   gcc -fsanitize=address,undefined -fno-omit-frame-pointer -g -fopenmp
 * Exit code 0 and no sanitizer report = clean. Built and run by tests/test_oracle_sanitize.py. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "sts_oracle.h"

static uint16_t bf16(float f) {
  uint32_t w;
  memcpy(&w, &f, 4);
  return (uint16_t)((w + 0x7fffu + ((w >> 16) & 1u)) >> 16);
}

static float frand(unsigned *s) {
  *s = *s * 1664525u + 1013904223u;
  return (float)((*s >> 8) & 0xffff) / 65536.0f - 0.5f;
}

int main(void) {
  unsigned seed = 1;
  enum { B = 2, Hd = 3, Tq = 4, N = 37, Hq = 6, Hkv = 2, D = 16, K = 9, PAGE = 4 };
  const int NB = (N + PAGE - 1) / PAGE;
  float *P = malloc(sizeof(float) * B * Hd * Tq * N), *lse = malloc(sizeof(float) * B * Hd * Tq);
  float *A = malloc(sizeof(float) * B * Hd * N), *blk = malloc(sizeof(float) * B * Hd * NB);
  for (int i = 0; i < B * Hd * Tq * N; ++i) P[i] = frand(&seed) + 0.5f;
  for (int i = 0; i < B * Hd * Tq; ++i) lse[i] = 1.0f;
  int32_t lens[B] = {N, 5}, lens0[B] = {0, N};
  int rc = 0;
  rc |= oracle_aggregate(P, NULL, B, Hd, Tq, N, ORACLE_SCORES_PROBS, ORACLE_REDUCE_SUM, A);
  rc |= oracle_aggregate(P, lse, B, Hd, Tq, N, ORACLE_SCORES_LOGITS_LSE, ORACLE_REDUCE_MAX, A);
  int32_t *sel = malloc(sizeof(int32_t) * B * Hd * (N + 3)), *cnt = malloc(sizeof(int32_t) * B * Hd);
  rc |= oracle_select(A, B, Hd, N, NULL, K, sel, cnt);
  rc |= oracle_select(A, B, Hd, N, lens, N + 3, sel, cnt);      /* k > N pads the tail */
  rc |= oracle_select(A, B, Hd, N, lens0, 1, sel, cnt);         /* an empty row */
  rc |= oracle_select(A, B, Hd, N, lens, K, sel, cnt);
  rc |= oracle_block_scores(A, B, Hd, N, lens, PAGE, blk);
  rc |= oracle_block_scores(A, B, Hd, N, NULL, 1, A);           /* page 1 in place is the identity */
  int32_t hm[Hq] = {0, 0, 2, 1, 1, 2};
  int32_t *idx = malloc(sizeof(int32_t) * B * Hq * K), *cn = malloc(sizeof(int32_t) * B * Hq);
  rc |= oracle_remap(sel, cnt, B, Hd, Hq, K, hm, idx, cn);
  uint16_t *q = malloc(2 * B * Tq * Hq * D), *k = malloc(2 * B * Hkv * N * D), *v = malloc(2 * B * Hkv * N * D);
  uint16_t *kn = malloc(2 * B * Tq * Hkv * D), *vn = malloc(2 * B * Tq * Hkv * D);
  for (int i = 0; i < B * Tq * Hq * D; ++i) q[i] = bf16(frand(&seed));
  for (int i = 0; i < B * Hkv * N * D; ++i) { k[i] = bf16(frand(&seed)); v[i] = bf16(frand(&seed)); }
  for (int i = 0; i < B * Tq * Hkv * D; ++i) { kn[i] = bf16(frand(&seed)); vn[i] = bf16(frand(&seed)); }
  float *out = malloc(sizeof(float) * B * Tq * Hq * D), *l2 = malloc(sizeof(float) * B * Hq * Tq);
  float *lg = malloc(sizeof(float) * B * Hq * Tq * N);
  rc |= oracle_attn(q, k, v, B, Tq, Hq, Hkv, D, N, (int64_t)Hkv * N * D, (int64_t)N * D, D, idx, cn, K, NULL, 0.25f,
                    out, l2, NULL, 0, B, 0, Hq, NULL, NULL, 0);
  rc |= oracle_attn(q, k, v, B, Tq, Hq, Hkv, D, N, (int64_t)Hkv * N * D, (int64_t)N * D, D, idx, cn, K, NULL, 0.25f,
                    out, l2, NULL, 1, B, 2, 5, kn, vn, 1);
  rc |= oracle_attn(q, k, v, B, Tq, Hq, Hkv, D, N, (int64_t)Hkv * N * D, (int64_t)N * D, D, NULL, NULL, 0, lens0,
                    0.25f, out, l2, lg, 0, B, 0, Hq, kn, vn, 0);
  int32_t map[4];
  int64_t ov[4 * Hd];
  /* traces: reuse P as [S=2,Hd,R=Tq,N] for the draft and its first 4 "heads" reordered for the target */
  float *at = malloc(sizeof(float) * 2 * 4 * Tq * N);
  for (int s = 0; s < 2; ++s)
    for (int h = 0; h < 4; ++h)
      memcpy(at + ((size_t)s * 4 + h) * Tq * N, P + ((size_t)s * Hd + (h % Hd)) * Tq * N, sizeof(float) * Tq * N);
  rc |= oracle_head_mapping(P, at, 2, Hd, 4, Tq, N, 5, map, ov);
  rc |= oracle_head_mapping(P, at, 2, Hd, 4, Tq, N, N + 10, map, NULL);
  /* argument errors must be reported, not crash */
  if (oracle_select(A, B, Hd, N, NULL, 0, sel, cnt) == 0) rc |= 64;
  idx[0] = N;   /* out-of-range index */
  if (oracle_attn(q, k, v, B, Tq, Hq, Hkv, D, N, (int64_t)Hkv * N * D, (int64_t)N * D, D, idx, cn, K, NULL, 0.25f, out,
                  l2, NULL, 0, B, 0, Hq, NULL, NULL, 0) == 0)
    rc |= 128;
  for (int t = 0; t < 4; ++t)
    if (map[t] != t % Hd && map[t] > t % Hd) rc |= 256;
  free(P); free(lse); free(A); free(blk); free(sel); free(cnt); free(idx); free(cn); free(q); free(k); free(v);
  free(kn); free(vn); free(out); free(l2); free(lg); free(at);
  printf("oracle sanitizer driver: rc=%d threads=%d\n", rc, oracle_num_threads());
  return rc;
}
