// Internal helpers shared by the HIP translation units of libbass (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bass.h"

namespace bass {

constexpr int kWave = 64;          // CDNA wavefront
constexpr int kBlockTokens = 32;   // tokens per cache block (one PV contraction step of the bf16 MFMA)
constexpr int kMaxWaves = 8192;    // upper bound of the attention work spread (sizes the workspace)
// The registers of the streaming kernel allow one wavefront per SIMD (256 CUs x 4 SIMDs = 1024
// resident wavefronts).  Measured on the paper-shaped batches, three quarters of that is fastest:
// the memory system is saturated either way, and fewer wavefronts mean fewer partials to merge.
constexpr int kDefaultWaves = 768;

// ---------------------------------------------------------------------------------------
// bf16 cache layout (library-owned).  A cache is [B][Hkv][nblk] blocks of 32 tokens; a block
// holds 32*D bf16 stored in the order the matrix cores consume them, so that a wavefront
// reads 1 KiB per load instruction (lane l reads bytes [16 l, 16 l + 16)) straight into an
// MFMA operand.
//   K block: [tile tt (2)][k-step t (D/32)][lane (64)][j (8)]
//            lane = grp*16 + r holds token 16*tt + r, head elements d = 32*t + 8*grp + j
//   V block: [d-tile mt (D/16)][lane (64)][j (8)]
//            lane = grp*16 + dr holds head element d = 16*mt + dr of the eight tokens
//            (j < 4: 4*grp + j ; j >= 4: 16 + 4*grp + (j-4))
// The V token order is the order in which the score tile leaves the QK^T MFMA, which is why
// the probabilities need no shuffle before the PV MFMA.
// ---------------------------------------------------------------------------------------
__host__ __device__ inline int num_blocks(int Lcap) { return (Lcap + kBlockTokens - 1) / kBlockTokens; }

__host__ __device__ inline size_t k_elem_offset(int D, int tok_in_blk, int d) {
  const int tt = tok_in_blk >> 4, r = tok_in_blk & 15;
  const int t = d >> 5, grp = (d & 31) >> 3, j = d & 7;
  return (size_t)(((tt * (D >> 5) + t) * 64 + grp * 16 + r) * 8 + j);
}

__host__ __device__ inline size_t v_elem_offset(int /*D*/, int tok_in_blk, int d) {
  const int half = tok_in_blk >> 4, w = tok_in_blk & 15;
  const int grp = w >> 2, j = half * 4 + (w & 3);
  const int mt = d >> 4, dr = d & 15;
  return (size_t)((mt * 64 + grp * 16 + dr) * 8 + j);
}

// ---------------------------------------------------------------------------------------
// INT8 cache layout (BASS_DTYPE_INT8KV).  Same blocks of 32 tokens; a block holds the 32*D codes as
// 16-byte chunks per lane, so that a wavefront still reads 1 KiB per load instruction, followed by the
// block's 32 fp32 scales in token order (one per token of this kv head).
//   K block: [tile tt (2)][k-step ks (D/64)][lane (64)][j (16)] -- the operand order of the INT8 matrix
//            instruction (16x16x64): lane = grp*16 + r holds token 16*tt + r, head elements 64*ks + 16*grp + j
//   V block: the element order of the bf16 V layout above, fragment mt of a lane being 8 codes = 8 bytes,
//            two consecutive fragments per chunk: byte ((mt/2)*64 + lane)*16 + (mt%2)*8 + j
// ---------------------------------------------------------------------------------------
__host__ __device__ inline size_t i8_block_bytes(int D) { return (size_t)kBlockTokens * D + kBlockTokens * 4; }

__host__ __device__ inline size_t i8_k_offset(int D, int tok_in_blk, int d) {
  const int tt = tok_in_blk >> 4, r = tok_in_blk & 15;
  const int ks = d >> 6, grp = (d & 63) >> 4, j = d & 15;
  return (size_t)(((tt * (D >> 6) + ks) * 64 + grp * 16 + r) * 16 + j);
}

__host__ __device__ inline size_t i8_v_offset(int /*D*/, int tok_in_blk, int d) {
  const int half = tok_in_blk >> 4, w = tok_in_blk & 15;
  const int grp = w >> 2, j = half * 4 + (w & 3);
  const int f = d >> 4, lane = grp * 16 + (d & 15);
  return (size_t)(((f >> 1) * 64 + lane) * 16 + (f & 1) * 8 + j);
}

// Quantizer of the INT8 caches (see bass.h, BASS_DTYPE_INT8KV): every step is one fp32 operation.
#ifdef __HIPCC__
__device__ inline float bf16_bits_to_float(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// codes of 8 bf16 values (in a uint4) for the row scale 127 / amax; returns them packed in 8 bytes
__device__ inline uint2 quantize8(const uint4& v, float inv) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
  uint32_t out[2] = {0u, 0u};
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float x = bf16_bits_to_float((w[e >> 1] >> (16 * (e & 1))) & 0xFFFFu);
    const int code = (int)__builtin_rintf(x * inv);  // one fp32 product, round half to even
    out[e >> 2] |= ((uint32_t)code & 0xFFu) << (8 * (e & 3));
  }
  return make_uint2(out[0], out[1]);
}

__device__ inline float amax8(const uint4& v) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
  float m = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) m = fmaxf(m, fabsf(bf16_bits_to_float((w[e >> 1] >> (16 * (e & 1))) & 0xFFFFu)));
  return m;
}
#endif

// 64-bit inclusive prefix sum and total over a wavefront.  Shifts inside rows of 16 lanes are DPP moves of
// the two halves (a generic shuffle of a 64-bit value is two trips through the LDS crossbar per step); the
// three row totals are then added from scalar registers.  Integer sums: the order is irrelevant.
#ifdef __HIPCC__
template <int N>
__device__ inline uint64_t row_shift_right_u64(uint64_t v) {  // lane i of a row gets lane i - N of the row, 0 for i < N
  const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)v, 0x110 + N, 0xF, 0xF, true);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(v >> 32), 0x110 + N, 0xF, 0xF, true);
  return ((uint64_t)hi << 32) | lo;
}

__device__ inline uint64_t read_lane_u64(uint64_t v, int src) {  // src: wave-uniform
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, src);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), src);
  return ((uint64_t)hi << 32) | lo;
}

__device__ inline uint64_t wave_incl_scan_u64(uint64_t v, int lane) {
  v += row_shift_right_u64<1>(v);
  v += row_shift_right_u64<2>(v);
  v += row_shift_right_u64<4>(v);
  v += row_shift_right_u64<8>(v);
  const uint64_t t0 = read_lane_u64(v, 15), t1 = read_lane_u64(v, 31), t2 = read_lane_u64(v, 47);
  const int row = lane >> 4;
  return v + (row > 0 ? t0 : 0) + (row > 1 ? t1 : 0) + (row > 2 ? t2 : 0);
}

template <int N>
__device__ inline float row_shift_right_keep(float v) {  // lane i of a row gets lane i - N of the row, its own value for i < N
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), 0x110 + N, 0xF, 0xF, false));
}

__device__ inline float wave_max_f32(float v) {  // the same maximum in every lane
  v = fmaxf(v, row_shift_right_keep<1>(v));
  v = fmaxf(v, row_shift_right_keep<2>(v));
  v = fmaxf(v, row_shift_right_keep<4>(v));
  v = fmaxf(v, row_shift_right_keep<8>(v));
  const float a = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 15));
  const float b = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 31));
  const float c = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 47));
  const float d = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
  return fmaxf(fmaxf(a, b), fmaxf(c, d));
}

__device__ inline uint64_t wave_sum_u64(uint64_t v) {  // the same total in every lane
  v += row_shift_right_u64<1>(v);
  v += row_shift_right_u64<2>(v);
  v += row_shift_right_u64<4>(v);
  v += row_shift_right_u64<8>(v);
  return read_lane_u64(v, 15) + read_lane_u64(v, 31) + read_lane_u64(v, 47) + read_lane_u64(v, 63);
}
#endif

// Per-sequence lengths with the clamping the header promises.  L = cached tokens before the
// step, nq = query tokens; on return 0 <= nq <= kmax, 0 <= L, L + nq <= Lcap.
__device__ inline bool clamp_lengths(int& L, int& nq, int kmax, int Lcap) {
  bool bad = false;
  if (nq < 0) { nq = 0; bad = true; }
  if (nq > kmax) { nq = kmax; bad = true; }
  if (nq > Lcap) { nq = Lcap; bad = true; }
  if (L < 0) { L = 0; bad = true; }
  if (L + nq > Lcap) { L = Lcap - nq; bad = true; }
  return bad;
}

inline int check_desc(const bass_attn_desc* d) {
  if (!d) return BASS_ERR_INVALID_ARG;
  if (d->B <= 0 || d->kmax <= 0 || d->Hq <= 0 || d->Hkv <= 0 || d->D <= 0 || d->Lcap <= 0)
    return BASS_ERR_INVALID_ARG;
  if (d->Hq % d->Hkv != 0) return BASS_ERR_INVALID_ARG;
  if (d->dtype == BASS_DTYPE_BF16 || d->dtype == BASS_DTYPE_INT8KV) {
    if (d->D != 64 && d->D != 128) return BASS_ERR_UNSUPPORTED;
  } else if (d->dtype == BASS_DTYPE_FP32) {
    if (d->D % 4 != 0 || d->D > 256) return BASS_ERR_UNSUPPORTED;
  } else {
    return BASS_ERR_UNSUPPORTED;
  }
  // index arithmetic inside the kernels is 32-bit for block counts and 64-bit for bytes
  if ((int64_t)d->B * d->Hkv * (int64_t)num_blocks(d->Lcap) >= (1ll << 30)) return BASS_ERR_UNSUPPORTED;
  return BASS_OK;
}

// Peek, so that the caller can still fetch the HIP error code after a BASS_ERR_HIP return.
inline int launch_status() { return hipPeekAtLastError() == hipSuccess ? BASS_OK : BASS_ERR_HIP; }

}  // namespace bass
