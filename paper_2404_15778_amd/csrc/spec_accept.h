// Device code of the speculative-sampling acceptance, shared by bass_spec_accept (probability rows in memory)
// and bass_warp_accept (probabilities evaluated on the fly from logits and row summaries).
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
// Workgroups of 16 wavefronts.  Each wavefront sums chunks of 1024 consecutive entries of the chosen
// row (pair) -- four 16-byte loads per lane and row -- into one 64-bit chunk sum; one wavefront then
// locates the chunk and the entry where the cumulative weight first exceeds the threshold, re-reading
// only that chunk.  The pass over the row is bound by the instruction stream of the compute unit that
// runs it (V entries x instructions per entry), so the weight is five instructions and there is one
// wave reduction per 1024 entries.
//
// A row source `Src` provides
//   void load4(int j0, int V, float (&pv)[4], float (&qv)[4]) const   entries j0 .. j0+3 of the row pair
//                                                                      (0 beyond V; qv untouched without q)
//   bool has_q() const / void drop_q()                                 residual p - q, or p alone
#pragma once
#include "bass_common.h"

namespace bass {

constexpr int kAcceptThreads = 1024;
constexpr int kAcceptWaves = kAcceptThreads / kWave;
constexpr int kTile = 256;                    // entries per wavefront load: 4 per lane
constexpr int kChunk = 4 * kTile;             // entries per chunk sum: 16 per lane
constexpr int kMaxVocab = 1 << 19;            // keeps the weight sum below 2^63
constexpr int kMaxChunks = kMaxVocab / kChunk;  // 512

// floor(min(w, 1) * 2^44) in two exact steps: the integer part of w * 2^12, and the fraction of it
// times 2^32 (scalings by powers of two and v_fract are exact; the conversions truncate).
__device__ inline uint64_t fixed44(float w) {
  // negative residuals and NaN carry no weight: max(NaN, 0) = 0
  const float a = fminf(fmaxf(w, 0.f), 1.0f) * 4096.0f;
  const uint32_t hi = (uint32_t)a;
  const uint32_t lo = (uint32_t)(__builtin_amdgcn_fractf(a) * 4294967296.0f);
  return ((uint64_t)hi << 32) | lo;
}

// Probability rows in memory.  qrow == nullptr: weights are p.
struct ProbRows {
  const float* prow;
  const float* qrow;
  bool vec;  // V a multiple of 4 and both tensors 16-byte aligned: 16-byte loads
  __device__ bool has_q() const { return qrow != nullptr; }
  __device__ void drop_q() { qrow = nullptr; }
  __device__ void load4(int j0, int V, float (&pv)[4], float (&qv)[4]) const {
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
  }
};

// The four weights of entries j0..j0+3 (entries >= V weigh 0).
template <class Src>
__device__ inline void weights4(const Src& src, int j0, int V, uint64_t (&w)[4]) {
  float pv[4] = {0.f, 0.f, 0.f, 0.f}, qv[4] = {0.f, 0.f, 0.f, 0.f};
  src.load4(j0, V, pv, qv);
#pragma unroll
  for (int e = 0; e < 4; ++e) w[e] = fixed44(src.has_q() ? __fsub_rn(pv[e], qv[e]) : pv[e]);
}

// Chunk sums c_begin <= c < c_end, one chunk per wavefront and round (all eight 16-byte loads are in flight
// before the first sum); lane 0 of the wavefront stores sums[c] -- with kDeviceScope as a device-scope store
// (written through to where every compute unit of the device reads it), for sums another workgroup adds up.
template <bool kDeviceScope = false, class Src>
__device__ inline void chunk_sums(const Src& src, int V, int c_begin, int c_end, uint64_t* sums, int wave, int lane) {
  for (int c = c_begin + wave; c < c_end; c += kAcceptWaves) {
    uint64_t w[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r) weights4(src, c * kChunk + r * kTile + 4 * lane, V, w[r]);
    uint64_t mine = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) mine += w[r][0] + w[r][1] + w[r][2] + w[r][3];
    const uint64_t sum = wave_sum_u64(mine);
    if (lane == 0) {
      if constexpr (kDeviceScope) __hip_atomic_store(sums + c, sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      else sums[c] = sum;
    }
  }
}

// Total of the chunk sums (in LDS), the same in every lane of every wavefront: integer sums, order irrelevant.
__device__ inline uint64_t total_weight(const uint64_t* chunk_sum, int nchunks, int lane) {
  uint64_t part = 0;
  for (int c = lane; c < nchunks; c += 64) part += chunk_sum[c];
  return wave_sum_u64(part);
}

// The token drawn by inverse CDF (one wavefront): T = (floor(u * 2^32) * S) >> 32, the first entry whose
// cumulative weight exceeds T.  chunk_sum: LDS, all nchunks sums; S > 0 their total.
template <class Src>
__device__ inline int draw_token(const Src& src, int V, int nchunks, const uint64_t* chunk_sum, uint64_t S, float ur,
                                 int lane) {
  const float umax = 1.0f - 5.9604644775390625e-08f;  // 1 - 2^-24
  if (!(ur >= 0.f)) ur = 0.f;
  if (ur > umax) ur = umax;
  const uint64_t U = (uint64_t)((double)ur * 4294967296.0);
  // T = (U * S) >> 32 without a 128-bit product: U < 2^32, S < 2^63
  const uint64_t T = U * (S >> 32) + ((U * (S & 0xFFFFFFFFull)) >> 32);
  // chunk holding the first cumulative weight > T: lanes own contiguous runs of chunks
  const int per = (nchunks + 63) / 64;
  const int t_lo = lane * per, t_hi = min(nchunks, t_lo + per);
  uint64_t run = 0;
  for (int t = t_lo; t < t_hi; ++t) run += chunk_sum[t];
  const uint64_t incl = wave_incl_scan_u64(run, lane);
  const uint64_t excl = incl - run;
  const unsigned long long hit = __ballot(incl > T);
  const int src_lane = __ffsll((long long)hit) - 1;  // S > T guarantees a hit
  int chunk = 0;
  uint64_t before = 0;
  if (lane == src_lane) {
    uint64_t c = excl;
    chunk = t_lo;
    for (int t = t_lo; t < t_hi; ++t) {
      if (c + chunk_sum[t] > T) { chunk = t; break; }
      c += chunk_sum[t];
    }
    before = c;
  }
  chunk = __builtin_amdgcn_readlane(chunk, src_lane);  // src_lane is wave-uniform
  before = read_lane_u64(before, src_lane);
  // inside the chunk: lane l takes its 16 consecutive entries
  uint64_t w[4][4];
  uint64_t mine = 0;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    weights4(src, chunk * kChunk + 16 * lane + 4 * r, V, w[r]);
    mine += w[r][0] + w[r][1] + w[r][2] + w[r][3];
  }
  const uint64_t incl2 = before + wave_incl_scan_u64(mine, lane);
  const unsigned long long hit2 = __ballot(incl2 > T);
  const int src2 = __ffsll((long long)hit2) - 1;
  int tok = 0;
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
  return __builtin_amdgcn_readlane(tok, src2);
}

// Number of drafts of sequence b, clamped to 0..kmax (st receives BASS_STATUS_LEN_CLAMPED).
__device__ inline int clamped_drafts(int k, int kmax, int& st) {
  if (k < 0) { k = 0; st |= BASS_STATUS_LEN_CLAMPED; }
  if (k > kmax) { k = kmax; st |= BASS_STATUS_LEN_CLAMPED; }
  return k;
}

// Drafted token id, clamped into the vocabulary (*sh_status, in LDS, receives BASS_STATUS_TOKEN_CLAMPED).
__device__ inline int clamped_token(int x, int V, int* sh_status) {
  if (x < 0) { x = 0; atomicOr(sh_status, BASS_STATUS_TOKEN_CLAMPED); }
  if (x >= V) { x = V - 1; atomicOr(sh_status, BASS_STATUS_TOKEN_CLAMPED); }
  return x;
}

// Draft with u, q(x), p(x) is accepted iff u q < p, exactly.
__device__ inline bool draft_accepted(float u, float qx, float px) { return (double)u * (double)qx < (double)px; }

}  // namespace bass
