// Measurement aid of libbass: a plain streaming read, the ceiling the attention launch is held against.
//
// The verification step is bound by reading every valid K and V row once (BASS paper, Section 3.2:
// attention shares no reads between sequences, so batching does not reduce its memory traffic).  What
// the memory system delivers to the access pattern of the attention kernel -- one wavefront per SIMD,
// 1 KiB per wavefront load instruction, non-temporal, a contiguous share of 8 KiB K blocks and 8 KiB V
// blocks per wavefront, two blocks in flight while one is consumed -- with no arithmetic, no schedule,
// no partial results and no merge is measured by this kernel on the same buffers.
#include "bass_common.h"

namespace bass {

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

struct StreamBlock {
  u32x4 k[8], v[8];
};

constexpr int kStreamVec = 512;  // uint4 per 8 KiB block

__device__ inline void stream_fetch(StreamBlock& r, const uint4* k, const uint4* v, long blk, int lane) {
  const u32x4* kp = (const u32x4*)(k + blk * kStreamVec + lane);
  const u32x4* vp = (const u32x4*)(v + blk * kStreamVec + lane);
#pragma unroll
  for (int i = 0; i < 8; ++i) r.k[i] = __builtin_nontemporal_load(kp + 64 * i);
#pragma unroll
  for (int i = 0; i < 8; ++i) r.v[i] = __builtin_nontemporal_load(vp + 64 * i);
}

__device__ inline unsigned stream_consume(const StreamBlock& r) {
  unsigned a = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) a ^= r.k[i][0] ^ r.k[i][1] ^ r.k[i][2] ^ r.k[i][3] ^ r.v[i][0] ^ r.v[i][1] ^ r.v[i][2] ^ r.v[i][3];
  return a;
}

__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* k, const uint4* v, int nblocks, int nwaves,
                                                          uint32_t* sink) {
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6));
  const Split sp = make_split(nblocks, nwaves);
  const int base = sp.first(w), n = sp.first(w + 1) - base;
  // all fetches unconditional, as in the attention kernel; one past the end re-reads 16 bytes of the
  // share's first block (block 0 for an empty share: nblocks >= 1)
  const long safe = n > 0 ? base : 0;
  StreamBlock r0, r1, r2;
  auto fetch = [&](StreamBlock& r, int s) { stream_fetch(r, k, v, s < n ? (long)base + s : safe, s < n ? lane : 0); };
  unsigned acc = 0;
  fetch(r0, 0);
  fetch(r1, 1);
  for (int s = 0; s < n; s += 3) {
    fetch(r2, s + 2);
    acc ^= stream_consume(r0);
    fetch(r0, s + 3);
    if (s + 1 < n) acc ^= stream_consume(r1);
    fetch(r1, s + 4);
    if (s + 2 < n) acc ^= stream_consume(r2);
  }
  // keeps the loads alive; buffers of ordinary data do not produce this value in every lane
  if (acc == 0x9E3779B9u && sink) sink[w] = acc;
}

}  // namespace bass

extern "C" int64_t bass_bench_stream_read(const void* K, const void* V, size_t bytes_each, int32_t waves, uint32_t* sink,
                                          void* stream) {
  if (!K || !V || waves < bass::kWavesPerWorkgroup || waves > bass::kMaxWaves || waves % bass::kWavesPerWorkgroup != 0)
    return BASS_ERR_INVALID_ARG;
  if (((uintptr_t)K & 15) != 0 || ((uintptr_t)V & 15) != 0) return BASS_ERR_INVALID_ARG;
  const size_t nblocks = bytes_each / 8192;
  if (nblocks < 1 || nblocks > 0x7fffffff) return BASS_ERR_INVALID_ARG;
  const int wpw = bass::waves_per_workgroup(waves);  // the workgroup shape of an attention launch of as many wavefronts
  hipLaunchKernelGGL(bass::stream_read_kernel, dim3(waves / wpw), dim3(64 * wpw), 0, (hipStream_t)stream, (const uint4*)K,
                     (const uint4*)V, (int)nblocks, (int)waves, sink);
  if (bass::launch_status() != BASS_OK) return BASS_ERR_HIP;
  return (int64_t)(nblocks * 2 * 8192);
}
