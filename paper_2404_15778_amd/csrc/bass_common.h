// Internal helpers shared by the HIP translation units of libbass (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bass.h"
#include "attn_plan.h"
#include "bass_layout.h"

namespace bass {

constexpr int kWave = 64;          // CDNA wavefront
// The registers of the streaming kernel allow one wavefront per SIMD (256 CUs x 4 SIMDs = 1024
// resident wavefronts).  Measured on the paper-shaped batches, three quarters of that is fastest:
// the memory system is saturated either way, and fewer wavefronts mean fewer partials to merge.
constexpr int kDefaultWaves = 768;

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
  // (the flattened block list counts up to kMaxPad virtual blocks per unit on top of the real ones)
  if ((int64_t)d->B * d->Hkv * ((int64_t)num_blocks(d->Lcap) + kMaxPad) >= (1ll << 30)) return BASS_ERR_UNSUPPORTED;
  return BASS_OK;
}

// ---------------------------------------------------------------------------------------
// Shape of an attention launch: which kernel serves the descriptor, over how many shares the block
// list is divided, and the virtual blocks of a unit.  The plan of a step and the launches that
// consume it derive it from the same inputs.
// ---------------------------------------------------------------------------------------
constexpr int kWavesPerWorkgroup = 4;  // also the grain of a launch's wavefront count
constexpr int kComputeUnits = 256;     // MI355X
// Wavefronts per workgroup of a launch whose wavefronts each fill a SIMD's registers (one workgroup per
// compute unit at a time).  Four, except where three put exactly one workgroup on every compute unit: 768
// wavefronts as 256 x 3 measured 2 % shorter attention launches than as 192 x 4 with 64 units idle (two per
// workgroup, 384 workgroups: 7 % longer; one: 1 % shorter).
inline int waves_per_workgroup(int nwaves) { return nwaves == 3 * kComputeUnits ? 3 : kWavesPerWorkgroup; }
constexpr int kAppendPad = 3;     // virtual blocks per unit when the append is fused (measured best: 3)
constexpr int kPlainPad = 2;      // ... and when it is not (the unit's last blocks are the masked, slower ones)
constexpr int kAppendBefore = 1;  // how many of those sit in front of the unit's last real block (one-tile matrix-core
constexpr int kPlainBefore = 0;   // kernel; measured: +0.5 % with the fused append, slightly slower without)
constexpr int kMaxStagedElems = 2048;  // kmax * D up to which the step's rows are appended inside the attention launch

int attention_waves_setting();  // bass_set_attention_waves (0 = defaults); verify_attention.hip

struct LaunchShape {
  bool mfma;        // bf16 or INT8 caches: the matrix-core kernels
  bool tiles;       // bf16 caches, more than one 16-row query tile per kv head: the workgroup-level kernel
  bool fused_append;  // the step's rows are appended inside the attention launch
  int rows_max, nwaves, nshares, target, pad, pad_before, fused_reduce;
};

// many_rows: more than one 16-row query tile per kv head (grouped-query attention); a separate
// launch merges the partials there, and a wider spread measured best: 896, and with INT8 caches, where the
// kernel is bound by its conversion instructions, every SIMD (1024).  One query tile: 768 for INT8 caches
// too -- as 256 workgroups of three they measured level with 1024 on the long-context shape and 2 - 3 %
// shorter on the benchmark shape (a fourth wavefront on a compute unit costs the others issue slots).
inline int attention_waves(int setting, bool many_rows, bool int8) {
  int w = setting > 0 ? setting : (many_rows ? (int8 ? 1024 : 896) : kDefaultWaves);
  if (w < 64) w = 64;
  if (w > kMaxWaves) w = kMaxWaves;
  return w - w % kWavesPerWorkgroup;
}

inline LaunchShape launch_shape(const bass_attn_desc* d, bool append) {
  LaunchShape s;
  const int setting = attention_waves_setting();
  s.rows_max = d->kmax * (d->Hq / d->Hkv);
  s.mfma = d->dtype != BASS_DTYPE_FP32;
  s.tiles = d->dtype == BASS_DTYPE_BF16 && s.rows_max > 16;
  s.fused_append = append && (d->dtype == BASS_DTYPE_FP32 || (int64_t)d->kmax * d->D <= kMaxStagedElems);
  // (a launch wider than the shares it aims at, with all shares equally long -- plan_split -- was measured
  // 1 - 2 % slower than the even division on the benchmark shapes: more wavefronts, more partials to merge)
  const int aim = attention_waves(setting, s.mfma && s.rows_max > 16, d->dtype == BASS_DTYPE_INT8KV);
  s.nwaves = aim;
  // the workgroup-level kernel takes one stretch per workgroup (default 256, measured best: fewer
  // partials to merge; a wavefront setting W gives W / 2)
  s.nshares = !s.tiles ? s.nwaves : setting > 0 ? (s.nwaves / 2 > 16 ? s.nwaves / 2 : 16) : 256;
  s.target = !s.tiles ? aim : s.nshares;
  s.pad = s.fused_append ? kAppendPad : kPlainPad;
  s.pad_before = 0;
  if (s.mfma && s.rows_max <= 16) s.pad_before = s.fused_append ? kAppendBefore : kPlainBefore;
  // one query tile per kv head: the last-arriving wavefront reduces; more: a second, chip-wide launch
  s.fused_reduce = (d->dtype == BASS_DTYPE_FP32 || s.rows_max <= 16) ? 1 : 0;
  return s;
}

// Peek, so that the caller can still fetch the HIP error code after a BASS_ERR_HIP return.
inline int launch_status() { return hipPeekAtLastError() == hipSuccess ? BASS_OK : BASS_ERR_HIP; }

}  // namespace bass
