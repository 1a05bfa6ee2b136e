/* Runs the CPU checker's entry points on a small ragged batch; built with -fsanitize=address,undefined by
 * tests/test_sanitizers.py, so that out-of-bounds accesses, overflows and misaligned accesses in the checker show up
 * as a non-zero exit. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "../../oracle/sparsebal_oracle.c"

static float rnd(uint64_t *s) {
  *s = *s * 6364136223846793005ull + 1442695040888963407ull;
  return (float)((double)(*s >> 33) / 2147483648.0 - 1.0);
}

int main(void) {
  const int lens[] = {200, 64, 1, 130, 0, 77};
  const int S = 6, Hq = 4, Hkv = 2, D = 8, B = 64;
  int32_t cu[7] = {0};
  for (int s = 0; s < S; ++s) cu[s + 1] = cu[s] + lens[s];
  const int T = cu[S];
  uint64_t seed = 12345;
  float *Q = malloc(sizeof(float) * T * Hq * D), *dO = malloc(sizeof(float) * T * Hq * D);
  float *K = malloc(sizeof(float) * T * Hkv * D), *V = malloc(sizeof(float) * T * Hkv * D);
  for (int i = 0; i < T * Hq * D; ++i) { Q[i] = rnd(&seed); dO[i] = rnd(&seed); }
  for (int i = 0; i < T * Hkv * D; ++i) { K[i] = rnd(&seed); V[i] = rnd(&seed); }
  const float rho[6] = {0.5f, 1.0f, 0.1f, 0.34f, 0.7f, 0.0f};
  int32_t topk[6];
  if (orc_keep_ratio_to_topk(cu, S, B, rho, topk)) return 2;
  for (int mode = 0; mode < 2; ++mode) {
    orc_shape sh = {T, S, Hq, Hkv, D, B, mode, cu};
    const int64_t nqb = orc_num_qblocks(&sh), ne = orc_scores_elems(&sh);
    const int Hs = mode == 0 ? Hq : Hkv;
    double *kbar = malloc(sizeof(double) * nqb * Hkv * D), *sc = malloc(sizeof(double) * (ne + 1));
    float *scf = malloc(sizeof(float) * (ne + 1));
    if (orc_block_mean(&sh, K, Hkv, kbar) || orc_block_scores(&sh, Q, K, 0.35, sc)) return 3;
    for (int64_t i = 0; i < ne; ++i) scf[i] = (float)sc[i];
    int32_t *rowptr = malloc(sizeof(int32_t) * (Hs * nqb + 1));
    if (orc_sel_rowptr(&sh, topk, rowptr)) return 4;
    int32_t *idx = malloc(sizeof(int32_t) * (rowptr[Hs * nqb] + 1));
    if (orc_select_topk(&sh, scf, topk, rowptr, idx)) return 5;
    double *O = malloc(sizeof(double) * T * Hq * D), *LSE = malloc(sizeof(double) * Hq * T);
    double *dQ = malloc(sizeof(double) * T * Hq * D), *dK = malloc(sizeof(double) * T * Hkv * D), *dV = malloc(sizeof(double) * T * Hkv * D);
    if (orc_attn_fwd(&sh, Q, K, V, rowptr, idx, 0.35, O, LSE)) return 6;
    if (orc_attn_bwd(&sh, Q, K, V, dO, rowptr, idx, 0.35, dQ, dK, dV)) return 7;
    const int32_t toks[3] = {0, 199, T - 1}, heads[3] = {0, 3, 1};
    double o3[3 * 8], l3[3], dq3[3 * 8], bk[64 * 8], bv[64 * 8], row[8];
    if (orc_attn_rows(&sh, Q, K, V, dO, rowptr, idx, 0.35, 3, toks, heads, o3, l3, dq3)) return 8;
    if (orc_attn_bwd_kvblock(&sh, Q, K, V, dO, rowptr, idx, 0.35, 0, 1, 3, bk, bv)) return 9;
    if (orc_block_scores_row(&sh, Q, K, 0.35, 0, Hs - 1, 3, row)) return 10;
    double chk = 0;
    for (int i = 0; i < T * Hq * D; ++i) chk += O[i] + dQ[i];
    for (int i = 0; i < T * Hkv * D; ++i) chk += dK[i] + dV[i];
    if (!isfinite(chk)) return 11;
    printf("mode %d checksum %.6f\n", mode, chk);
    free(kbar); free(sc); free(scf); free(rowptr); free(idx); free(O); free(LSE); free(dQ); free(dK); free(dV);
  }
  free(Q); free(dO); free(K); free(V);
  return 0;
}
