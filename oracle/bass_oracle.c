/*
 * CPU oracle for the batched verification step of BASS (batched speculative
 * sampling with ragged attention).  TEST INFRASTRUCTURE ONLY: it is slow,
 * plain and written to be checked against the paper by eye.  It shares no code
 * with the HIP library and must never be reached from the product path.
 *
 * What it follows
 *   - attention:  Section 3.2 ("Proposed method"): scores between the query
 *     tensor of the current tokens and the keys of all tokens processed so
 *     far, P = softmax(Q^T K / c), then P times V.  Each sequence has its own
 *     length (ragged K, V, P); a padded position has probability exactly zero
 *     (BASS-PAD) which is the same as computing each sequence at its true
 *     length (BASS-SPLIT).  Section 2.2: the draft tokens are processed by the
 *     main model as incremental context encoding, hence causal among
 *     themselves and full attention to the sequence's own cache.
 *   - acceptance: Section 2.2: how many drafts are accepted is decided from the
 *     main- and draft-model probabilities; on rejection a corrected token is
 *     drawn from the main model's outputs; the whole is equivalent to sampling
 *     from the main model.  The paper gives the rule by citation (speculative
 *     sampling): accept draft x with probability min(1, p(x)/q(x)), on the
 *     first rejection draw from max(p-q,0) renormalised, after k acceptances
 *     draw a bonus token from the next main-model row.
 *
 * Arithmetic: fp64 throughout for attention (inputs are widened exactly from
 * the bit patterns the GPU receives).  Acceptance is an exact rule: the test
 * u < p/q is evaluated as u*q < p in fp64 (the product of two fp32 numbers is
 * exact in fp64), the residual weight is ONE IEEE fp32 subtraction, and the
 * inverse-CDF draw uses 2^44 fixed-point integer weights so that the result
 * does not depend on summation order.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC (no fast-math).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_DTYPE_BF16 0
#define ORACLE_DTYPE_FP32 1

/* status bits (same meaning as the library's device status word) */
#define ORACLE_STATUS_LEN_CLAMPED 1
#define ORACLE_STATUS_TOKEN_CLAMPED 2
#define ORACLE_STATUS_ZERO_MASS 4

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* exact widening of one element to fp64 */
static double widen(const void* base, size_t idx, int dtype) {
  if (dtype == ORACLE_DTYPE_FP32) return (double)((const float*)base)[idx];
  uint32_t bits = ((uint32_t)((const uint16_t*)base)[idx]) << 16; /* bf16 = top half of fp32 */
  float f;
  memcpy(&f, &bits, sizeof f);
  return (double)f;
}

/*
 * Ragged verify attention, Section 3.2 (attention flow) + Section 2.2 (drafts as
 * incremental context encoding).
 *
 *   Q      [B, kmax, Hq, D]        queries of the current (draft) tokens
 *   K, V   [B, Lrows, Hkv, D]      logical per-sequence cache, token-major; row j
 *                                  of sequence b is token j; rows
 *                                  [0, ctx_len[b]+draft_len[b]) are valid and the
 *                                  draft tokens' own K/V sit at the end of them
 *   O      [B, kmax, Hq, D] fp64   rows i >= draft_len[b] are 0
 *   lse    [B, kmax, Hq]    fp64   natural-log of the softmax denominator
 *                                  (including the max), 0 for unused rows; may be NULL
 *
 * Query i of sequence b sees tokens j <= ctx_len[b] + i.  Query head h uses
 * kv head h / (Hq/Hkv).
 */
void oracle_verify_attention(int B, int kmax, int Hq, int Hkv, int D, int Lrows, int dtype,
                             double scale, const void* Q, const void* K, const void* V,
                             const int32_t* ctx_len, const int32_t* draft_len, double* O,
                             double* lse) {
  const int g = Hq / Hkv;
  memset(O, 0, sizeof(double) * (size_t)B * kmax * Hq * D);
  if (lse) memset(lse, 0, sizeof(double) * (size_t)B * kmax * Hq);
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int b = 0; b < B; ++b) {
    for (int h = 0; h < Hq; ++h) {
      const int L = ctx_len[b];
      const int nq = draft_len[b];
      const int hk = h / g;
      double* s = (double*)malloc(sizeof(double) * (size_t)(L + nq + 1));
      for (int i = 0; i < nq; ++i) {
        const int n = L + i + 1; /* tokens visible to query i */
        const size_t qoff = (((size_t)b * kmax + i) * Hq + h) * D;
        double m = -INFINITY;
        for (int j = 0; j < n; ++j) {
          const size_t koff = (((size_t)b * Lrows + j) * Hkv + hk) * D;
          double dot = 0.0;
          for (int d = 0; d < D; ++d) dot += widen(Q, qoff + d, dtype) * widen(K, koff + d, dtype);
          s[j] = dot * scale;
          if (s[j] > m) m = s[j];
        }
        double denom = 0.0;
        for (int j = 0; j < n; ++j) {
          s[j] = exp(s[j] - m); /* unnormalised probability of token j */
          denom += s[j];
        }
        double* out = O + qoff;
        for (int j = 0; j < n; ++j) {
          const size_t voff = (((size_t)b * Lrows + j) * Hkv + hk) * D;
          const double pj = s[j] / denom; /* P[i, j]; rows of P sum to 1 */
          for (int d = 0; d < D; ++d) out[d] += pj * widen(V, voff + d, dtype);
        }
        if (lse) lse[((size_t)b * kmax + i) * Hq + h] = m + log(denom);
      }
      free(s);
    }
  }
}

/*
 * The same attention for ONE output row (b, i, h): used to spot-check full-size
 * workloads where computing every row would take too long.  out[D]; probs (may
 * be NULL) receives the ctx_len_b+i+1 entries of row i of P; returns lse.
 */
double oracle_verify_attention_row(int kmax, int Hq, int Hkv, int D, int Lrows, int dtype,
                                   double scale, const void* Q, const void* K, const void* V,
                                   int b, int i, int h, int ctx_len_b, double* out, double* probs) {
  const int g = Hq / Hkv, hk = h / g, n = ctx_len_b + i + 1;
  const size_t qoff = (((size_t)b * kmax + i) * Hq + h) * D;
  double* s = (double*)malloc(sizeof(double) * (size_t)n);
  double m = -INFINITY, denom = 0.0;
  for (int j = 0; j < n; ++j) {
    const size_t koff = (((size_t)b * Lrows + j) * Hkv + hk) * D;
    double dot = 0.0;
    for (int d = 0; d < D; ++d) dot += widen(Q, qoff + d, dtype) * widen(K, koff + d, dtype);
    s[j] = dot * scale;
    if (s[j] > m) m = s[j];
  }
  for (int j = 0; j < n; ++j) {
    s[j] = exp(s[j] - m);
    denom += s[j];
  }
  for (int d = 0; d < D; ++d) out[d] = 0.0;
  for (int j = 0; j < n; ++j) {
    const size_t voff = (((size_t)b * Lrows + j) * Hkv + hk) * D;
    const double pj = s[j] / denom;
    if (probs) probs[j] = pj;
    for (int d = 0; d < D; ++d) out[d] += pj * widen(V, voff + d, dtype);
  }
  free(s);
  return m + log(denom);
}

/*
 * Cache append (Section 2.1: keys and values of processed tokens are cached;
 * Section 3.2: each sequence proceeds at its own pace, so the write offset is
 * per sequence; a rejected draft's rows are simply overwritten by the next step).
 *   cache  [B, Lrows, Hkv, D]   logical, token-major
 *   rows   [B, kmax, Hkv, D]    this step's rows; the first n_new[b] are written at
 *                               cache positions ctx_len[b] .. ctx_len[b]+n_new[b]-1
 * elt_bytes = 2 (bf16) or 4 (fp32): a byte copy.
 */
void oracle_kv_append(int B, int kmax, int Hkv, int D, int Lrows, int elt_bytes, void* cache,
                      const void* rows, const int32_t* ctx_len, const int32_t* n_new) {
  const size_t row = (size_t)Hkv * D * elt_bytes;
  for (int b = 0; b < B; ++b)
    for (int i = 0; i < n_new[b]; ++i)
      memcpy((char*)cache + ((size_t)b * Lrows + ctx_len[b] + i) * row,
             (const char*)rows + ((size_t)b * kmax + i) * row, row);
}

/* floor(min(w,1) * 2^44) as an integer; w >= 0.  Exact: scaling by a power of two. */
static uint64_t fixed44(float w) {
  double x = (double)w;
  if (x > 1.0) x = 1.0;
  return (uint64_t)floor(x * 17592186044416.0 /* 2^44 */);
}

/*
 * Speculative-sampling acceptance for a batch (Section 2.2; rule of the cited
 * speculative-sampling papers), one sequence at a time.
 *
 *   p          [B, kmax+1, V]  main-model probabilities; row i judges draft i, row
 *                              n_draft[b] is the bonus row
 *   q          [B, kmax,   V]  draft-model probabilities
 *   draft_tok  [B, kmax]
 *   n_draft    [B]             k_b in 0..kmax
 *   u          [B, kmax+1]     uniforms in [0,1): u[b,i] judges draft i, u[b,kmax]
 *                              drives the corrected/bonus draw
 *   n_accept   [B] out         length of the accepted prefix
 *   next_token [B] out         corrected token (rejection) or bonus token
 *   ctx_len    [B] in/out, may be NULL: += n_accept + 1  (the previous last token
 *                              and the accepted drafts now have valid cache rows)
 *   status     out, may be NULL: OR of ORACLE_STATUS_* bits
 */
void oracle_spec_accept(int B, int kmax, int V, const float* p, const float* q,
                        const int32_t* draft_tok, const int32_t* n_draft, const float* u,
                        int32_t* n_accept, int32_t* next_token, int32_t* ctx_len, int32_t* status) {
  int32_t st = 0;
  for (int b = 0; b < B; ++b) {
    int k = n_draft[b];
    if (k < 0) { k = 0; st |= ORACLE_STATUS_LEN_CLAMPED; }
    if (k > kmax) { k = kmax; st |= ORACLE_STATUS_LEN_CLAMPED; }
    const float* pb = p + (size_t)b * (kmax + 1) * V;
    const float* qb = q + (size_t)b * kmax * V;
    /* accepted prefix: accept draft i iff u_i < p_i(x_i) / q_i(x_i), strict */
    int n = 0;
    for (int i = 0; i < k; ++i) {
      int x = draft_tok[(size_t)b * kmax + i];
      if (x < 0) { x = 0; st |= ORACLE_STATUS_TOKEN_CLAMPED; }
      if (x >= V) { x = V - 1; st |= ORACLE_STATUS_TOKEN_CLAMPED; }
      const double lhs = (double)u[(size_t)b * (kmax + 1) + i] * (double)qb[(size_t)i * V + x];
      const double rhs = (double)pb[(size_t)i * V + x];
      if (lhs < rhs) ++n; else break;
    }
    /* weights of the new token: residual max(p-q,0) after a rejection, p itself
       after k acceptances (bonus) or when the residual has no mass */
    const float* prow = pb + (size_t)n * V;
    const float* qrow = (n < k) ? qb + (size_t)n * V : NULL;
    uint64_t S = 0;
    if (qrow) {
      for (int j = 0; j < V; ++j) {
        const float w = prow[j] - qrow[j]; /* one fp32 subtraction */
        if (w > 0.0f) S += fixed44(w);
      }
      if (S == 0) qrow = NULL; /* p <= q everywhere in fp32: fall back to p */
    }
    if (!qrow) {
      S = 0;
      for (int j = 0; j < V; ++j) if (prow[j] > 0.0f) S += fixed44(prow[j]);
    }
    int tok = 0;
    if (S == 0) {
      st |= ORACLE_STATUS_ZERO_MASS;
    } else {
      float ur = u[(size_t)b * (kmax + 1) + kmax];
      const float umax = 1.0f - 5.9604644775390625e-08f; /* 1 - 2^-24 */
      if (!(ur >= 0.0f)) ur = 0.0f;
      if (ur > umax) ur = umax;
      const uint64_t U = (uint64_t)floor((double)ur * 4294967296.0 /* 2^32 */);
      const uint64_t T = (uint64_t)(((unsigned __int128)U * (unsigned __int128)S) >> 32); /* T < S */
      uint64_t c = 0;
      for (int j = 0; j < V; ++j) {
        float w = qrow ? prow[j] - qrow[j] : prow[j];
        if (w > 0.0f) c += fixed44(w);
        if (c > T) { tok = j; break; } /* first token whose cumulative weight exceeds T */
      }
    }
    n_accept[b] = n;
    next_token[b] = tok;
    if (ctx_len) ctx_len[b] += n + 1;
  }
  if (status) *status = st;
}
