// Logits -> acceptance in one call: bass_warp_accept.
//
// Section 2.2 of the BASS paper decides the accepted prefix and the corrected / bonus token from the
// probabilities of the main and the draft model; the experiments of Section 4 obtain those from the logits at
// temperature 0.2 with nucleus top-p 0.95.  bass_warp_probs followed by bass_spec_accept does that through two
// stored tensors of probabilities (B (2 kmax + 1) rows of V floats written, of which the acceptance reads one
// row pair per sequence plus one entry per draft).  Here no probability row is stored:
//
//  1. warp_summaries_kernel, one workgroup per row of logits (main and draft rows in one launch): the row's
//     warp exactly as bass_warp_probs computes it (the same device function), of which only the RowSummary is
//     kept -- 32 bytes from which the probability of any token of the row follows from its logit and its id.
//  2. warp_accept_kernel, G workgroups per sequence: every workgroup evaluates the sequence's accept tests
//     (one logit of each model per draft), so all of them know the first rejection n; the pass over row n
//     (pair) -- probabilities rebuilt from the logits and the two summaries, integer weights of the residual
//     -- is divided over the G workgroups by chunks of 1024 entries.  Chunk sums go to the workspace; the
//     workgroup that arrives last at the sequence's counter adds them up and draws the token.
//
// Every arithmetic step is the one of the two-call path (the same functions on the same fp32 values), and the
// sums are integers, so n_accept, next_token and the status bits are identical to it, bit for bit.
//
// Exchange between the workgroups of a sequence (the protocol of the attention kernel's partials): chunk sums
// are device-scope stores, written through past the per-XCD L2; a wavefront's vector-memory counter falls to
// zero only when every one of its stores has been acknowledged there, and each wavefront waits for that before
// the workgroup barrier; thread 0 then adds 1 to the sequence's counter (device-scope atomic).  The workgroup
// that reads G - 1 there is the last: all sums are in place, and it reads them with device-scope loads.
// Counters are zeroed by the first launch of every call, so the workspace needs no initialisation and a call
// that was interrupted leaves nothing behind.
#include "logit_warp.h"
#include "spec_accept.h"

namespace bass {

struct SummaryParams {
  int rows_main, rows_all, V;
  const float* logits_main;
  const float* logits_draft;
  float c, top_p;
  RowSummary* summary;   // rows_all of them: the main rows, then the draft rows
  uint32_t* counter;     // B arrival counters, zeroed here
  int B;
  int32_t* status;
};

template <int W, int NG>
__global__ __launch_bounds__(kWarpThreads) void warp_summaries_kernel(SummaryParams a) {
  const int r = blockIdx.x;
  if (r == 0)
    for (int b = threadIdx.x; b < a.B; b += kWarpThreads) a.counter[b] = 0u;
  const float* z = r < a.rows_main ? a.logits_main + (size_t)r * a.V : a.logits_draft + (size_t)(r - a.rows_main) * a.V;
  warp_row<W, NG, true>(z, nullptr, a.V, a.c, a.top_p, a.status, a.summary + r);
}

// Rows of logits and the summaries of their warp: entries are the probabilities bass_warp_probs would store.
struct LogitRows {
  const float* zp;
  const float* zq;  // nullptr: weights are p
  bool vec;
  float c;
  RowSummary sp, sq;
  __device__ bool has_q() const { return zq != nullptr; }
  __device__ void drop_q() { zq = nullptr; }
  __device__ void load4(int j0, int V, float (&pv)[4], float (&qv)[4]) const {
    float a[4] = {0.f, 0.f, 0.f, 0.f}, b[4] = {0.f, 0.f, 0.f, 0.f};
    const bool whole = vec && j0 + 3 < V;
    if (whole) {
      const float4 t = *(const float4*)(zp + j0);
      a[0] = t.x; a[1] = t.y; a[2] = t.z; a[3] = t.w;
      if (zq) {
        const float4 s = *(const float4*)(zq + j0);
        b[0] = s.x; b[1] = s.y; b[2] = s.z; b[3] = s.w;
      }
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (j0 + e < V) {
          a[e] = zp[j0 + e];
          if (zq) b[e] = zq[j0 + e];
        }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (whole || j0 + e < V) {
        pv[e] = warped_prob(sp, c, a[e], j0 + e);
        if (zq) qv[e] = warped_prob(sq, c, b[e], j0 + e);
      }
  }
};

struct WarpAcceptParams {
  int B, kmax, V;
  const float* logits_main;
  const float* logits_draft;
  float c;
  const RowSummary* sum_main;   // [B, kmax + 1]
  const RowSummary* sum_draft;  // [B, kmax]
  const int32_t* draft_tok;
  const int32_t* n_draft;
  const float* u;
  int32_t* n_accept;
  int32_t* next_token;
  int32_t* ctx_len;
  uint64_t* chunk_sum;  // [B, nchunks]
  uint32_t* counter;    // [B]
  int32_t* status;
};

__global__ __launch_bounds__(kAcceptThreads) void warp_accept_kernel(WarpAcceptParams a) {
  __shared__ uint64_t chunk_sum[kMaxChunks];
  __shared__ int sh_first_reject;
  __shared__ int sh_status;
  __shared__ int sh_last;
  constexpr int kStaged = 33;  // rows per model whose summaries are staged in LDS (the paper's l_limit is 32)
  __shared__ RowSummary sh_main[kStaged], sh_draft[kStaged];
  const int b = blockIdx.y, slice = blockIdx.x, G = gridDim.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int V = a.V, kmax = a.kmax;
  const float* zpb = a.logits_main + (size_t)b * (kmax + 1) * V;
  const float* zqb = a.logits_draft + (size_t)b * kmax * V;
  const RowSummary* spb = a.sum_main + (size_t)b * (kmax + 1);
  const RowSummary* sqb = a.sum_draft + (size_t)b * kmax;
  const float* ub = a.u + (size_t)b * (kmax + 1);

  // everything that does not depend on another load is requested at once: the number of drafts, the first
  // round of drafted tokens and uniforms, and the summaries of the sequence's rows (into LDS; beyond kStaged
  // rows per model they are read from memory where needed)
  const int k_given = a.n_draft[b];
  const bool first_round = tid < kmax;
  const int x_first = first_round ? a.draft_tok[(size_t)b * kmax + tid] : 0;
  const float u_first = first_round ? ub[tid] : 0.f;
  if (tid < kStaged && tid <= kmax) sh_main[tid] = spb[tid];
  if (tid >= kWave && tid - kWave < kStaged && tid - kWave < kmax) sh_draft[tid - kWave] = sqb[tid - kWave];
  auto main_summary = [&](int i) { return i < kStaged ? sh_main[i] : spb[i]; };
  auto draft_summary = [&](int i) { return i < kStaged ? sh_draft[i] : sqb[i]; };

  int st = 0;
  const int k = clamped_drafts(k_given, kmax, st);
  if (tid == 0) { sh_first_reject = k; sh_status = 0; }
  __syncthreads();
  // accept tests of all drafts (every workgroup of the sequence: a few loads, and all need the outcome)
  for (int i = tid; i < k; i += kAcceptThreads) {
    const int x = clamped_token(i == tid ? x_first : a.draft_tok[(size_t)b * kmax + i], V, &sh_status);
    const float ui = i == tid ? u_first : ub[i];
    const float zq = zqb[(size_t)i * V + x], zp = zpb[(size_t)i * V + x];
    const float qx = warped_prob(draft_summary(i), a.c, zq, x);
    const float px = warped_prob(main_summary(i), a.c, zp, x);
    if (!draft_accepted(ui, qx, px)) atomicMin(&sh_first_reject, i);
  }
  __syncthreads();
  const int n = sh_first_reject;
  st |= sh_status;

  const bool vec = (V % 4 == 0) && (((uintptr_t)a.logits_main | (uintptr_t)a.logits_draft) % 16 == 0);
  LogitRows rows{zpb + (size_t)n * V, (n < k) ? zqb + (size_t)n * V : nullptr, vec, a.c, main_summary(n),
                 (n < k) ? draft_summary(n) : main_summary(n)};
  const int nchunks = (V + kChunk - 1) / kChunk;
  uint64_t* sums = a.chunk_sum + (size_t)b * nchunks;

  // this workgroup's chunks of the row (pair)
  const int per = (nchunks + G - 1) / G;
  const int c0 = min(nchunks, slice * per), c1 = min(nchunks, c0 + per);
  chunk_sums<true>(rows, V, c0, c1, sums, wave, lane);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wavefront's sums have been acknowledged ...
  __syncthreads();                                  // ... and so have every wavefront's of the workgroup
  if (tid == 0) {
    const uint32_t before = __hip_atomic_fetch_add(a.counter + b, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    sh_last = before == (uint32_t)(G - 1);
  }
  __syncthreads();
  if (!sh_last) return;
  for (int c = tid; c < nchunks; c += kAcceptThreads)
    chunk_sum[c] = __hip_atomic_load(sums + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  uint64_t S = total_weight(chunk_sum, nchunks, lane);
  if (S == 0 && rows.has_q()) {
    // p <= q everywhere in fp32: the residual has no mass, draw from p itself (rare: this workgroup alone)
    rows.drop_q();
    __syncthreads();
    chunk_sums(rows, V, 0, nchunks, chunk_sum, wave, lane);
    __syncthreads();
    S = total_weight(chunk_sum, nchunks, lane);
  }

  if (wave == 0) {
    int tok = 0;
    if (S == 0) st |= BASS_STATUS_ZERO_MASS;
    else tok = draw_token(rows, V, nchunks, chunk_sum, S, ub[kmax], lane);
    if (lane == 0) {
      a.n_accept[b] = n;
      a.next_token[b] = tok;
      if (a.ctx_len) a.ctx_len[b] += n + 1;
      if (st && a.status) atomicOr(a.status, st);
    }
  }
}

struct WarpAcceptLayout {
  size_t summaries, counters, sums, bytes;
};

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

inline WarpAcceptLayout warp_accept_layout(int B, int kmax, int V) {
  WarpAcceptLayout l;
  const size_t nchunks = ((size_t)V + kChunk - 1) / kChunk;
  l.summaries = 0;
  l.counters = align256((size_t)B * (2 * (size_t)kmax + 1) * sizeof(RowSummary));
  l.sums = l.counters + align256((size_t)B * sizeof(uint32_t));
  l.bytes = l.sums + align256((size_t)B * nchunks * sizeof(uint64_t));
  return l;
}

// workgroups per sequence: enough to put the pass on about a chip's worth of compute units, at least one
// chunk each
inline int slices_per_sequence(int B, int V) {
  const int nchunks = (V + kChunk - 1) / kChunk;
  int g = (256 + B - 1) / B;
  if (g > nchunks) g = nchunks;
  if (g < 1) g = 1;
  const int per = (nchunks + g - 1) / g;
  return (nchunks + per - 1) / per;  // no empty slices
}

}  // namespace bass

extern "C" size_t bass_warp_accept_workspace_bytes(int32_t B, int32_t kmax, int32_t V) {
  if (B <= 0 || kmax < 0 || V <= 0 || V > bass::kMaxVocab) return 0;
  return bass::warp_accept_layout(B, kmax, V).bytes;
}

extern "C" int bass_warp_accept(int32_t B, int32_t kmax, int32_t V, const float* logits_main, const float* logits_draft,
                                float temperature, float top_p, const int32_t* draft_tok, const int32_t* n_draft,
                                const float* u, int32_t* n_accept, int32_t* next_token, int32_t* ctx_len, void* workspace,
                                size_t workspace_bytes, int32_t* dev_status, void* stream) {
  using namespace bass;
  if (B <= 0 || kmax < 0 || V <= 0) return BASS_ERR_INVALID_ARG;
  if (!logits_main || !n_draft || !u || !n_accept || !next_token || !workspace) return BASS_ERR_INVALID_ARG;
  if (kmax > 0 && (!logits_draft || !draft_tok)) return BASS_ERR_INVALID_ARG;
  if (!(temperature > 0.f) || !(top_p > 0.f)) return BASS_ERR_INVALID_ARG;
  if (V > kMaxVocab || V > kWarpMaxVocab) return BASS_ERR_UNSUPPORTED;
  if ((int64_t)B * (2 * (int64_t)kmax + 1) > 0x7FFFFFFF || B > 65535) return BASS_ERR_UNSUPPORTED;  // grid limits
  const WarpAcceptLayout lay = warp_accept_layout(B, kmax, V);
  if (workspace_bytes < lay.bytes || ((uintptr_t)workspace & 255) != 0) return BASS_ERR_INVALID_ARG;
  char* base = (char*)workspace;
  RowSummary* summaries = (RowSummary*)(base + lay.summaries);
  uint32_t* counters = (uint32_t*)(base + lay.counters);
  uint64_t* sums = (uint64_t*)(base + lay.sums);
  hipStream_t s = (hipStream_t)stream;
  const float c = warp_exponent_scale(temperature);

  const int rows_main = B * (kmax + 1), rows_all = B * (2 * kmax + 1);
  SummaryParams sp{rows_main, rows_all, V, logits_main, logits_draft, c, top_p, summaries, counters, B, dev_status};
  const bool wide = V % 4 == 0 && (((uintptr_t)logits_main | (uintptr_t)logits_draft) & 15) == 0;
  const dim3 grid((unsigned)rows_all), block(kWarpThreads);
  switch (warp_variant(V, wide)) {
    case 1: hipLaunchKernelGGL((warp_summaries_kernel<1, 0>), grid, block, 0, s, sp); break;
    case 8: hipLaunchKernelGGL((warp_summaries_kernel<4, 8>), grid, block, 0, s, sp); break;
    case 13: hipLaunchKernelGGL((warp_summaries_kernel<4, 13>), grid, block, 0, s, sp); break;
    case 16: hipLaunchKernelGGL((warp_summaries_kernel<4, 16>), grid, block, 0, s, sp); break;
    default: hipLaunchKernelGGL((warp_summaries_kernel<4, 0>), grid, block, 0, s, sp); break;
  }
  if (launch_status() != BASS_OK) return BASS_ERR_HIP;

  WarpAcceptParams ap{B, kmax, V, logits_main, logits_draft, c, summaries, summaries + rows_main, draft_tok, n_draft, u,
                      n_accept, next_token, ctx_len, sums, counters, dev_status};
  const dim3 grid2((unsigned)slices_per_sequence(B, V), (unsigned)B);
  hipLaunchKernelGGL(warp_accept_kernel, grid2, dim3(kAcceptThreads), 0, s, ap);
  return launch_status();
}
