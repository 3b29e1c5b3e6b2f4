// Logits front end of libbass: bass_warp_probs (temperature, nucleus top-p, softmax).
//
// The paper's experiments sample at temperature 0.2 with nucleus top-p 0.95 (captions of the
// result tables of Section 4); the acceptance rule of Section 2.2 compares the probabilities the
// main and the draft model assign after that warp.  This entry point turns rows of logits into those
// probability rows; the method, its exactness and the kernel's structure are described in logit_warp.h.
#include "logit_warp.h"

namespace bass {

struct WarpParams {
  int R, V;
  const float* logits;
  float* probs;
  float c;      // log2(e) / T
  float top_p;
  int32_t* status;
};

template <int W, int NG>
__global__ __launch_bounds__(kWarpThreads) void warp_probs_kernel(WarpParams a) {
  warp_row<W, NG, false>(a.logits + (size_t)blockIdx.x * a.V, a.probs + (size_t)blockIdx.x * a.V, a.V, a.c, a.top_p,
                         a.status, nullptr);
}

}  // namespace bass

extern "C" int bass_warp_probs(int32_t R, int32_t V, const float* logits, float temperature, float top_p,
                               float* probs, int32_t* dev_status, void* stream) {
  using namespace bass;
  if (R <= 0 || V <= 0 || !logits || !probs) return BASS_ERR_INVALID_ARG;
  if (!(temperature > 0.f) || !(top_p > 0.f)) return BASS_ERR_INVALID_ARG;
  if (V > kWarpMaxVocab) return BASS_ERR_UNSUPPORTED;
  WarpParams a{R, V, logits, probs, warp_exponent_scale(temperature), top_p, dev_status};
  const bool wide = V % 4 == 0 && (((uintptr_t)logits | (uintptr_t)probs) & 15) == 0;  // rows 16-byte aligned
  const dim3 grid((unsigned)R), block(kWarpThreads);
  hipStream_t s = (hipStream_t)stream;
  switch (warp_variant(V, wide)) {
    case 1: hipLaunchKernelGGL((warp_probs_kernel<1, 0>), grid, block, 0, s, a); break;
    case 8: hipLaunchKernelGGL((warp_probs_kernel<4, 8>), grid, block, 0, s, a); break;
    case 13: hipLaunchKernelGGL((warp_probs_kernel<4, 13>), grid, block, 0, s, a); break;
    case 16: hipLaunchKernelGGL((warp_probs_kernel<4, 16>), grid, block, 0, s, a); break;
    default: hipLaunchKernelGGL((warp_probs_kernel<4, 0>), grid, block, 0, s, a); break;
  }
  return launch_status();
}
