// Speculative-sampling acceptance of libbass: bass_spec_accept (Section 2.2 of the BASS paper; the rule, its
// exact evaluation and the structure of the pass over a row are described in spec_accept.h).
//
// One workgroup of 16 wavefronts per sequence; the chunk sums of the chosen row (pair) stay in LDS.
#include "spec_accept.h"

namespace bass {

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

__global__ __launch_bounds__(kAcceptThreads) void spec_accept_kernel(AcceptParams a) {
  __shared__ uint64_t chunk_sum[kMaxChunks];
  __shared__ int sh_first_reject;
  __shared__ int sh_status;
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int V = a.V, kmax = a.kmax;
  const float* pb = a.p + (size_t)b * (kmax + 1) * V;
  const float* qb = a.q + (size_t)b * kmax * V;
  const float* ub = a.u + (size_t)b * (kmax + 1);

  int st = 0;
  const int k = clamped_drafts(a.n_draft[b], kmax, st);
  if (tid == 0) { sh_first_reject = k; sh_status = 0; }
  __syncthreads();

  // accept tests of all drafts in parallel; the prefix ends at the first rejection
  for (int i = tid; i < k; i += kAcceptThreads) {
    const int x = clamped_token(a.draft_tok[(size_t)b * kmax + i], V, &sh_status);
    if (!draft_accepted(ub[i], qb[(size_t)i * V + x], pb[(size_t)i * V + x])) atomicMin(&sh_first_reject, i);
  }
  __syncthreads();
  const int n = sh_first_reject;
  st |= sh_status;

  const bool vec = (V % 4 == 0) && (((uintptr_t)a.p | (uintptr_t)a.q) % 16 == 0);
  ProbRows rows{pb + (size_t)n * V, (n < k) ? qb + (size_t)n * V : nullptr, vec};
  const int nchunks = (V + kChunk - 1) / kChunk;

  uint64_t S = 0;
  for (int attempt = 0; attempt < 2; ++attempt) {
    chunk_sums(rows, V, 0, nchunks, chunk_sum, wave, lane);
    __syncthreads();
    S = total_weight(chunk_sum, nchunks, lane);
    if (S != 0 || !rows.has_q()) break;
    rows.drop_q();  // p <= q everywhere in fp32: the residual has no mass, draw from p itself
    __syncthreads();
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
