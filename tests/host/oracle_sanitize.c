/* Host build of the CPU oracle under -fsanitize=address,undefined: runs the attention, the single-row
 * attention, the append and the acceptance rule on small seeded inputs (ragged lengths, grouped heads,
 * a context of zero, a sequence without drafts, tiny and odd vocabularies) so that every array access of
 * the oracle has been executed once under the sanitizers.  Prints "ok" and exits 0. */
#include "../../oracle/bass_oracle.c"

#include <stdio.h>

static unsigned long long rng_state = 88172645463325252ull;
static double rnd(void) { /* xorshift, uniform in [0,1) */
  rng_state ^= rng_state << 13;
  rng_state ^= rng_state >> 7;
  rng_state ^= rng_state << 17;
  return (double)(rng_state >> 11) / 9007199254740992.0;
}

int main(void) {
  /* attention, fp32 and bf16 bit patterns */
  for (int dtype = 0; dtype < 2; ++dtype) {
    const int B = 3, kmax = 4, Hq = 4, Hkv = 2, D = 8, Lrows = 21;
    const int32_t ctx[3] = {0, 17, 5}, dl[3] = {4, 0, 3};
    const size_t nq = (size_t)B * kmax * Hq * D, nk = (size_t)B * Lrows * Hkv * D;
    void* Q = malloc(nq * 4);
    void* K = malloc(nk * 4);
    void* V = malloc(nk * 4);
    for (size_t i = 0; i < nq; ++i) {
      if (dtype == 1) ((float*)Q)[i] = (float)(rnd() - 0.5);
      else ((uint16_t*)Q)[i] = (uint16_t)(0x3C00 + (int)(rnd() * 512));
    }
    for (size_t i = 0; i < nk; ++i) {
      if (dtype == 1) { ((float*)K)[i] = (float)(rnd() - 0.5); ((float*)V)[i] = (float)(rnd() - 0.5); }
      else { ((uint16_t*)K)[i] = (uint16_t)(0x3C00 + (int)(rnd() * 512)); ((uint16_t*)V)[i] = (uint16_t)(0xBC00 + (int)(rnd() * 512)); }
    }
    double* O = (double*)malloc(nq * sizeof(double));
    double* lse = (double*)malloc((size_t)B * kmax * Hq * sizeof(double));
    oracle_verify_attention(B, kmax, Hq, Hkv, D, Lrows, dtype, 0.35, Q, K, V, ctx, dl, O, lse);
    double row[8], probs[32];
    for (int b = 0; b < B; ++b)
      for (int i = 0; i < dl[b]; ++i)
        for (int h = 0; h < Hq; ++h) {
          const double l = oracle_verify_attention_row(kmax, Hq, Hkv, D, Lrows, dtype, 0.35, Q, K, V, b, i, h, ctx[b], row, probs);
          const size_t o = (((size_t)b * kmax + i) * Hq + h) * D;
          for (int d = 0; d < D; ++d)
            if (fabs(row[d] - O[o + d]) > 1e-12) { printf("FAIL: row vs batch\n"); return 1; }
          if (fabs(l - lse[((size_t)b * kmax + i) * Hq + h]) > 1e-12) { printf("FAIL: lse\n"); return 1; }
        }
    free(Q); free(K); free(V); free(O); free(lse);
  }
  /* acceptance: vocabularies 1, 5, 64; k = 0 .. kmax; a rejected and an accepted run */
  const int Vs[3] = {1, 5, 64};
  for (int vi = 0; vi < 3; ++vi) {
    const int B = 4, kmax = 3, V = Vs[vi];
    float* p = (float*)malloc(sizeof(float) * B * (kmax + 1) * V);
    float* q = (float*)malloc(sizeof(float) * B * kmax * V);
    for (int r = 0; r < B * (kmax + 1); ++r) {
      double s = 0;
      for (int j = 0; j < V; ++j) { p[r * V + j] = (float)(rnd() + 1e-3); s += p[r * V + j]; }
      for (int j = 0; j < V; ++j) p[r * V + j] = (float)(p[r * V + j] / s);
    }
    for (int r = 0; r < B * kmax; ++r) {
      double s = 0;
      for (int j = 0; j < V; ++j) { q[r * V + j] = (float)(rnd() + 1e-3); s += q[r * V + j]; }
      for (int j = 0; j < V; ++j) q[r * V + j] = (float)(q[r * V + j] / s);
    }
    int32_t tok[12], nd[4] = {0, 1, 3, 3}, na[4], nt[4], ctx[4] = {1, 2, 3, 4}, status = 0;
    float u[16];
    for (int i = 0; i < 12; ++i) tok[i] = (int32_t)(rnd() * V);
    for (int i = 0; i < 16; ++i) u[i] = (float)rnd() * 0.999f;
    oracle_spec_accept(B, kmax, V, p, q, tok, nd, u, na, nt, ctx, &status);
    for (int b = 0; b < B; ++b)
      if (na[b] < 0 || na[b] > nd[b] || nt[b] < 0 || nt[b] >= V) { printf("FAIL: accept range\n"); return 1; }
    free(p); free(q);
  }
  printf("ok\n");
  return 0;
}
