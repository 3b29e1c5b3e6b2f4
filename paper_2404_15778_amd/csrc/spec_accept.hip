// Speculative-sampling acceptance of libbass: bass_spec_accept.
//
// BASS paper, Section 2.2: how many draft tokens are accepted is decided from the
// probabilities the main and the draft model give them; on rejection a corrected token is
// sampled from the main model's outputs; the procedure is equivalent to sampling from the
// main model.  Section 3.2: every sequence stops at its own rejection point.  The rule
// itself is speculative sampling: accept draft x with probability min(1, p(x)/q(x)); at the
// first rejection draw from max(p - q, 0) renormalised; after k acceptances draw a bonus
// token from the next main-model row.
//
// Exactness.  The test u < p/q is evaluated as u*q < p in fp64 (the product of two fp32
// values is exact there).  The draw uses integer weights floor(min(w,1) * 2^44), so sums
// are associative and the wavefront-parallel reduction order cannot change the result.
//
// One workgroup of 16 wavefronts per sequence.  Each wavefront sums chunks of 1024 consecutive
// entries of the chosen row (pair) -- four 16-byte loads per lane and row -- and keeps the chunk
// sums in LDS; the first wavefront then locates the chunk and the entry where the cumulative
// weight first exceeds the threshold, re-reading only that chunk.  The pass over the row is bound
// by the instruction stream of the one compute unit that has the sequence (V entries x instructions
// per entry), so the weight is five instructions and there is one wave reduction per 1024 entries.
#include "bass_common.h"

namespace bass {

constexpr int kAcceptThreads = 1024;
constexpr int kAcceptWaves = kAcceptThreads / kWave;
constexpr int kTile = 256;                    // entries per wavefront load: 4 per lane
constexpr int kChunk = 4 * kTile;             // entries per chunk sum: 16 per lane
constexpr int kMaxVocab = 1 << 19;            // keeps the weight sum below 2^63
constexpr int kMaxChunks = kMaxVocab / kChunk;  // 512

struct AcceptParams {
  int B, kmax, V;
  const float* p;
  const float* q;
  const int32_t* draft_tok;
  const int32_t* n_draft;
  const float* u;
  int32_t* n_accept;
  int32_t* next_token;
  int32_t* ctx_len;
  int32_t* status;
};

// floor(min(w, 1) * 2^44) in two exact steps: the integer part of w * 2^12, and the fraction of it
// times 2^32 (scalings by powers of two and v_fract are exact; the conversions truncate).
__device__ inline uint64_t fixed44(float w) {
  // negative residuals and NaN carry no weight: max(NaN, 0) = 0
  const float a = fminf(fmaxf(w, 0.f), 1.0f) * 4096.0f;
  const uint32_t hi = (uint32_t)a;
  const uint32_t lo = (uint32_t)(__builtin_amdgcn_fractf(a) * 4294967296.0f);
  return ((uint64_t)hi << 32) | lo;
}

// The four weights of entries j0..j0+3 (entries >= V weigh 0).  qrow == nullptr: weights are p.
__device__ inline void weights4(const float* prow, const float* qrow, int j0, int V, bool vec, uint64_t (&w)[4]) {
  float pv[4] = {0.f, 0.f, 0.f, 0.f}, qv[4] = {0.f, 0.f, 0.f, 0.f};
  if (vec && j0 + 3 < V) {
    const float4 a = *(const float4*)(prow + j0);
    pv[0] = a.x; pv[1] = a.y; pv[2] = a.z; pv[3] = a.w;
    if (qrow) {
      const float4 c = *(const float4*)(qrow + j0);
      qv[0] = c.x; qv[1] = c.y; qv[2] = c.z; qv[3] = c.w;
    }
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (j0 + e < V) {
        pv[e] = prow[j0 + e];
        if (qrow) qv[e] = qrow[j0 + e];
      }
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) w[e] = fixed44(qrow ? __fsub_rn(pv[e], qv[e]) : pv[e]);
}

__global__ __launch_bounds__(kAcceptThreads) void spec_accept_kernel(AcceptParams a) {
  __shared__ uint64_t chunk_sum[kMaxChunks];
  __shared__ int sh_first_reject;
  __shared__ int sh_status;
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int V = a.V, kmax = a.kmax;
  const float* pb = a.p + (size_t)b * (kmax + 1) * V;
  const float* qb = a.q + (size_t)b * kmax * V;
  const float* ub = a.u + (size_t)b * (kmax + 1);

  int k = a.n_draft[b];
  int st = 0;
  if (k < 0) { k = 0; st |= BASS_STATUS_LEN_CLAMPED; }
  if (k > kmax) { k = kmax; st |= BASS_STATUS_LEN_CLAMPED; }
  if (tid == 0) { sh_first_reject = k; sh_status = 0; }
  __syncthreads();

  // accept tests of all drafts in parallel; the prefix ends at the first rejection
  for (int i = tid; i < k; i += kAcceptThreads) {
    int x = a.draft_tok[(size_t)b * kmax + i];
    if (x < 0) { x = 0; atomicOr(&sh_status, BASS_STATUS_TOKEN_CLAMPED); }
    if (x >= V) { x = V - 1; atomicOr(&sh_status, BASS_STATUS_TOKEN_CLAMPED); }
    const double lhs = (double)ub[i] * (double)qb[(size_t)i * V + x];
    const double rhs = (double)pb[(size_t)i * V + x];
    if (!(lhs < rhs)) atomicMin(&sh_first_reject, i);
  }
  __syncthreads();
  const int n = sh_first_reject;
  st |= sh_status;

  const float* prow = pb + (size_t)n * V;
  const float* qrow = (n < k) ? qb + (size_t)n * V : nullptr;
  const int nchunks = (V + kChunk - 1) / kChunk;
  const bool vec = (V % 4 == 0) && (((uintptr_t)a.p | (uintptr_t)a.q) % 16 == 0);

  uint64_t S = 0;
  int tok = 0;
  for (int attempt = 0; attempt < 2; ++attempt) {
    // a chunk per wavefront and round: all eight 16-byte loads are in flight before the first sum
    for (int c = wave; c < nchunks; c += kAcceptWaves) {
      uint64_t w[4][4];
#pragma unroll
      for (int r = 0; r < 4; ++r) weights4(prow, qrow, c * kChunk + r * kTile + 4 * lane, V, vec, w[r]);  // entries >= V weigh 0
      uint64_t mine = 0;
#pragma unroll
      for (int r = 0; r < 4; ++r) mine += w[r][0] + w[r][1] + w[r][2] + w[r][3];
      const uint64_t sum = wave_sum_u64(mine);
      if (lane == 0) chunk_sum[c] = sum;
    }
    __syncthreads();
    // every wavefront derives the total the same way (integer sums: order is irrelevant)
    uint64_t part = 0;
    for (int c = lane; c < nchunks; c += 64) part += chunk_sum[c];
    S = wave_sum_u64(part);
    if (S != 0 || qrow == nullptr) break;
    qrow = nullptr;  // p <= q everywhere in fp32: the residual has no mass, draw from p itself
    __syncthreads();
  }

  if (wave == 0) {
    if (S == 0) {
      st |= BASS_STATUS_ZERO_MASS;
    } else {
      float ur = ub[kmax];
      const float umax = 1.0f - 5.9604644775390625e-08f;  // 1 - 2^-24
      if (!(ur >= 0.f)) ur = 0.f;
      if (ur > umax) ur = umax;
      const uint64_t U = (uint64_t)((double)ur * 4294967296.0);
      // T = (U * S) >> 32 without a 128-bit product: U < 2^32, S < 2^63
      uint64_t T = U * (S >> 32) + ((U * (S & 0xFFFFFFFFull)) >> 32);
      // chunk holding the first cumulative weight > T: lanes own contiguous runs of chunks
      const int per = (nchunks + 63) / 64;
      const int t_lo = lane * per, t_hi = min(nchunks, t_lo + per);
      uint64_t run = 0;
      for (int t = t_lo; t < t_hi; ++t) run += chunk_sum[t];
      const uint64_t incl = wave_incl_scan_u64(run, lane);
      const uint64_t excl = incl - run;
      const unsigned long long hit = __ballot(incl > T);
      const int src = __ffsll((long long)hit) - 1;  // S > T guarantees a hit
      int chunk = 0;
      uint64_t before = 0;
      if (lane == src) {
        uint64_t c = excl;
        chunk = t_lo;
        for (int t = t_lo; t < t_hi; ++t) {
          if (c + chunk_sum[t] > T) { chunk = t; break; }
          c += chunk_sum[t];
        }
        before = c;
      }
      chunk = __builtin_amdgcn_readlane(chunk, src);  // src is wave-uniform
      before = read_lane_u64(before, src);
      // inside the chunk: lane l takes its 16 consecutive entries
      uint64_t w[4][4];
      uint64_t mine = 0;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        weights4(prow, qrow, chunk * kChunk + 16 * lane + 4 * r, V, vec, w[r]);
        mine += w[r][0] + w[r][1] + w[r][2] + w[r][3];
      }
      const uint64_t incl2 = before + wave_incl_scan_u64(mine, lane);
      const unsigned long long hit2 = __ballot(incl2 > T);
      const int src2 = __ffsll((long long)hit2) - 1;
      if (lane == src2) {
        uint64_t c = incl2 - mine;
        int e = 0;
        bool found = false;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          if (!found) {
            if (c + w[j >> 2][j & 3] > T) { e = j; found = true; }
            else c += w[j >> 2][j & 3];
          }
        }
        tok = chunk * kChunk + 16 * lane + e;
      }
      tok = __builtin_amdgcn_readlane(tok, src2);
    }
    if (lane == 0) {
      a.n_accept[b] = n;
      a.next_token[b] = tok;
      if (a.ctx_len) a.ctx_len[b] += n + 1;
      if (st && a.status) atomicOr(a.status, st);
    }
  }
}

}  // namespace bass

extern "C" int bass_spec_accept(int32_t B, int32_t kmax, int32_t V, const float* p, const float* q,
                                const int32_t* draft_tok, const int32_t* n_draft, const float* u, int32_t* n_accept,
                                int32_t* next_token, int32_t* ctx_len, int32_t* dev_status, void* stream) {
  using namespace bass;
  if (B <= 0 || kmax < 0 || V <= 0) return BASS_ERR_INVALID_ARG;
  if (!p || !n_draft || !u || !n_accept || !next_token) return BASS_ERR_INVALID_ARG;
  if (kmax > 0 && (!q || !draft_tok)) return BASS_ERR_INVALID_ARG;
  if (V > kMaxVocab) return BASS_ERR_UNSUPPORTED;
  AcceptParams a{B, kmax, V, p, q, draft_tok, n_draft, u, n_accept, next_token, ctx_len, dev_status};
  hipLaunchKernelGGL(spec_accept_kernel, dim3((unsigned)B), dim3(kAcceptThreads), 0, (hipStream_t)stream, a);
  return launch_status();
}
