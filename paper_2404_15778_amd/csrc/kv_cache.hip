// KV-cache writer / reader of libbass: bass_kv_append, bass_kv_gather, bass_kv_cache_bytes.
//
// Section 2.1 of the BASS paper: keys and values of processed tokens are cached.  Section
// 3.2: sequences advance at their own pace, so every sequence has its own write offset and
// the rows of rejected drafts are discarded by overwriting them in the next step.
//
// The library owns the cache layout: bf16 caches are kept in MFMA fragment order (see
// bass_common.h) so the attention kernel's loads are 1 KiB-contiguous per wavefront and
// need no transposition; fp32 caches are token-major [B][Hkv][Lcap][D].
#include "bass_common.h"

namespace bass {

struct KvParams {
  int B, kmax, Hkv, D, Lcap, nblk;
  void* Kc;
  void* Vc;
  void* Kr;  // rows [B,kmax,Hkv,D] (source for append, destination for gather)
  void* Vr;
  const int32_t* off;  // [B] first cache token
  const int32_t* cnt;  // [B] number of rows
  int32_t* status;
};

// One workgroup per (row slot i, sequence b); threads sweep (kv head, 8-element chunk).
template <bool kGather>
__global__ __launch_bounds__(256) void kv_rows_bf16(KvParams p) {
  const int b = blockIdx.y, i = blockIdx.x;
  int n = p.cnt[b];
  const int off = p.off[b];
  bool bad = false;
  if (n < 0) { n = 0; bad = true; }
  if (n > p.kmax) { n = p.kmax; bad = true; }
  if (i >= n) {
    if (bad && i == 0 && threadIdx.x == 0 && p.status) atomicOr(p.status, BASS_STATUS_LEN_CLAMPED);
    return;
  }
  const long tok = (long)off + i;
  if (tok < 0 || tok >= p.Lcap) bad = true;
  if (bad) {
    if (threadIdx.x == 0 && p.status) atomicOr(p.status, BASS_STATUS_LEN_CLAMPED);
    if (tok < 0 || tok >= p.Lcap) return;
  }
  const int blk = (int)(tok / kBlockTokens), w = (int)(tok % kBlockTokens);
  const int chunks = p.D / 8;
  const size_t blk_elems = (size_t)kBlockTokens * p.D;
  for (int item = threadIdx.x; item < p.Hkv * chunks; item += blockDim.x) {
    const int kvh = item / chunks, d0 = (item % chunks) * 8;
    const size_t row = (((size_t)b * p.kmax + i) * p.Hkv + kvh) * p.D + d0;
    const size_t base = (((size_t)b * p.Hkv + kvh) * p.nblk + blk) * blk_elems;
    uint16_t* kc = (uint16_t*)p.Kc + base;
    uint16_t* vc = (uint16_t*)p.Vc + base;
    if (!kGather) {
      const uint4 kv = *(const uint4*)((const uint16_t*)p.Kr + row);
      *(uint4*)(kc + k_elem_offset(p.D, w, d0)) = kv;  // 8 consecutive d share one 16-byte slot
      const uint4 vv = *(const uint4*)((const uint16_t*)p.Vr + row);
      const uint16_t* ve = (const uint16_t*)&vv;
#pragma unroll
      for (int e = 0; e < 8; ++e) vc[v_elem_offset(p.D, w, d0 + e)] = ve[e];
    } else {
      *(uint4*)((uint16_t*)p.Kr + row) = *(const uint4*)(kc + k_elem_offset(p.D, w, d0));
      uint4 vv;
      uint16_t* ve = (uint16_t*)&vv;
#pragma unroll
      for (int e = 0; e < 8; ++e) ve[e] = vc[v_elem_offset(p.D, w, d0 + e)];
      *(uint4*)((uint16_t*)p.Vr + row) = vv;
    }
  }
}

template <bool kGather>
__global__ __launch_bounds__(256) void kv_rows_fp32(KvParams p) {
  const int b = blockIdx.y, i = blockIdx.x;
  int n = p.cnt[b];
  const int off = p.off[b];
  bool bad = false;
  if (n < 0) { n = 0; bad = true; }
  if (n > p.kmax) { n = p.kmax; bad = true; }
  if (i >= n) {
    if (bad && i == 0 && threadIdx.x == 0 && p.status) atomicOr(p.status, BASS_STATUS_LEN_CLAMPED);
    return;
  }
  const long tok = (long)off + i;
  if (tok < 0 || tok >= p.Lcap) bad = true;
  if (bad) {
    if (threadIdx.x == 0 && p.status) atomicOr(p.status, BASS_STATUS_LEN_CLAMPED);
    if (tok < 0 || tok >= p.Lcap) return;
  }
  const int chunks = p.D / 4;
  for (int item = threadIdx.x; item < p.Hkv * chunks; item += blockDim.x) {
    const int kvh = item / chunks, d0 = (item % chunks) * 4;
    const size_t row = (((size_t)b * p.kmax + i) * p.Hkv + kvh) * p.D + d0;
    const size_t dst = (((size_t)b * p.Hkv + kvh) * p.Lcap + tok) * p.D + d0;
    if (!kGather) {
      *(float4*)((float*)p.Kc + dst) = *(const float4*)((const float*)p.Kr + row);
      *(float4*)((float*)p.Vc + dst) = *(const float4*)((const float*)p.Vr + row);
    } else {
      *(float4*)((float*)p.Kr + row) = *(const float4*)((const float*)p.Kc + dst);
      *(float4*)((float*)p.Vr + row) = *(const float4*)((const float*)p.Vc + dst);
    }
  }
}

template <bool kGather>
static int launch_rows(const bass_attn_desc* d, void* Kc, void* Vc, void* Kr, void* Vr, const int32_t* off,
                       const int32_t* cnt, int32_t* status, void* stream) {
  int rc = check_desc(d);
  if (rc != BASS_OK) return rc;
  if (!Kc || !Vc || !Kr || !Vr || !off || !cnt) return BASS_ERR_INVALID_ARG;
  if (d->B > 65535) return BASS_ERR_UNSUPPORTED;
  KvParams p{d->B, d->kmax, d->Hkv, d->D, d->Lcap, num_blocks(d->Lcap), Kc, Vc, Kr, Vr, off, cnt, status};
  dim3 grid((unsigned)d->kmax, (unsigned)d->B);
  hipStream_t s = (hipStream_t)stream;
  if (d->dtype == BASS_DTYPE_BF16)
    hipLaunchKernelGGL(kv_rows_bf16<kGather>, grid, dim3(256), 0, s, p);
  else
    hipLaunchKernelGGL(kv_rows_fp32<kGather>, grid, dim3(256), 0, s, p);
  return launch_status();
}

}  // namespace bass

extern "C" size_t bass_kv_cache_bytes(const bass_attn_desc* d) {
  if (bass::check_desc(d) != BASS_OK) return 0;
  if (d->dtype == BASS_DTYPE_BF16)
    return (size_t)d->B * d->Hkv * bass::num_blocks(d->Lcap) * bass::kBlockTokens * d->D * 2;
  return (size_t)d->B * d->Hkv * d->Lcap * d->D * 4;
}

extern "C" int bass_kv_append(const bass_attn_desc* desc, void* Kcache, void* Vcache, const void* K_new,
                              const void* V_new, const int32_t* ctx_len, const int32_t* n_new,
                              int32_t* dev_status, void* stream) {
  return bass::launch_rows<false>(desc, Kcache, Vcache, (void*)K_new, (void*)V_new, ctx_len, n_new,
                                  dev_status, stream);
}

extern "C" int bass_kv_gather(const bass_attn_desc* desc, const void* Kcache, const void* Vcache, void* K_out,
                              void* V_out, const int32_t* start, const int32_t* n, int32_t* dev_status,
                              void* stream) {
  return bass::launch_rows<true>(desc, (void*)Kcache, (void*)Vcache, K_out, V_out, start, n, dev_status,
                                 stream);
}
