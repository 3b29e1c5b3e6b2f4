// KV-cache writer / reader of libbass: bass_kv_append, bass_kv_gather, bass_kv_cache_bytes.
//
// Section 2.1 of the BASS paper: keys and values of processed tokens are cached.  Section
// 3.2: sequences advance at their own pace, so every sequence has its own write offset and
// the rows of rejected drafts are discarded by overwriting them in the next step.
//
// The library owns the cache layout: bf16 caches are kept in MFMA fragment order (see
// bass_common.h) so the attention kernel's loads are 1 KiB-contiguous per wavefront and
// need no transposition; fp32 caches are token-major [B][Hkv][Lcap][D]; INT8 caches (the paper's
// appendix: keys and values quantized dynamically per head and per token) hold codes in the same
// fragment order plus one fp32 scale per token and kv head.
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
  float* Ks;  // INT8 gather only: scales out [B,kmax,Hkv]
  float* Vs;
};

// One thread per (sequence b, row slot i, kv head, 16-byte chunk of the row): everything a thread
// needs is two length words and one 16-byte load per tensor, so the whole launch is one short
// dependent chain (lengths -> row loads -> stores) however few rows there are.
// Cache token of row slot i of sequence b; false if the slot is unused or falls outside the
// cache.  The thread that handles the first chunk of the row (report = true) raises the status bit
// for a row count outside [0, kmax] (once, from slot 0) and for a used row outside the cache.
__device__ inline bool row_target(const KvParams& p, int b, int i, bool report, long& tok) {
  int n = p.cnt[b];
  bool bad = false;
  if (n < 0) { n = 0; bad = (i == 0); }
  if (n > p.kmax) { n = p.kmax; bad = (i == 0); }
  tok = (long)p.off[b] + i;
  const bool active = i < n;
  const bool inside = tok >= 0 && tok < p.Lcap;
  if (active && !inside) bad = true;
  if (bad && report && p.status) atomicOr(p.status, BASS_STATUS_LEN_CLAMPED);
  return active && inside;
}

template <bool kGather>
__global__ __launch_bounds__(256) void kv_rows_bf16(KvParams p) {
  const int chunks = p.D / 8;
  const long item = (long)blockIdx.x * 256 + threadIdx.x;  // over [B][kmax][Hkv][chunks]
  if (item >= (long)p.B * p.kmax * p.Hkv * chunks) return;
  const int ck = (int)(item % chunks);
  const int kvh = (int)((item / chunks) % p.Hkv);
  const int i = (int)((item / ((long)chunks * p.Hkv)) % p.kmax);
  const int b = (int)(item / ((long)chunks * p.Hkv * p.kmax));
  long tok;
  if (!row_target(p, b, i, ck == 0 && kvh == 0, tok)) return;
  const int blk = (int)(tok / kBlockTokens), w = (int)(tok % kBlockTokens);
  const int d0 = ck * 8;
  const size_t row = (size_t)item * 8;  // [B][kmax][Hkv][D] element offset of this chunk
  const size_t base = (((size_t)b * p.Hkv + kvh) * p.nblk + blk) * ((size_t)kBlockTokens * p.D);
  uint16_t* kc = (uint16_t*)p.Kc + base;
  uint16_t* vc = (uint16_t*)p.Vc + base;
  if (!kGather) {
    const uint4 kv = *(const uint4*)((const uint16_t*)p.Kr + row);
    const uint4 vv = *(const uint4*)((const uint16_t*)p.Vr + row);
    *(uint4*)(kc + k_elem_offset(p.D, w, d0)) = kv;  // 8 consecutive d share one 16-byte slot
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

// Appends of many rows (a prompt, a moved sequence): one workgroup per (sequence, kv head, 32-token
// cache block).  K rows go out as the 16-byte chunks they already are; the V tile is turned in LDS so
// that the cache receives whole 16-byte chunks (eight tokens of one head element) instead of 2-byte
// scatters.  A block that the rows cover only partly keeps its other tokens (read-modify-write; no
// other workgroup touches the block).
template <int D>
__global__ __launch_bounds__(256) void kv_blocks_bf16(KvParams p, int blocks_per_seq) {
  __shared__ __align__(16) uint16_t vt[kBlockTokens][D + 8];
  const int tid = threadIdx.x;
  const int j = blockIdx.x % blocks_per_seq;
  const int unit = blockIdx.x / blocks_per_seq;
  const int kvh = unit % p.Hkv, b = unit / p.Hkv;
  int n = p.cnt[b];
  bool bad = false;
  if (n < 0) { n = 0; bad = true; }
  if (n > p.kmax) { n = p.kmax; bad = true; }
  const long off = p.off[b];
  const long lo = max(off, 0l), hi = min(off + n, (long)p.Lcap);  // tokens that exist in the cache
  if (n > 0 && (off < 0 || off + n > p.Lcap)) bad = true;
  if (bad && j == 0 && kvh == 0 && tid == 0 && p.status) atomicOr(p.status, BASS_STATUS_LEN_CLAMPED);
  if (hi <= lo) return;
  const int blk = (int)(lo / kBlockTokens) + j;
  const long t0 = max(lo, (long)blk * kBlockTokens), t1 = min(hi, (long)(blk + 1) * kBlockTokens);
  if (t1 <= t0) return;  // uniform for the workgroup
  const size_t base = (((size_t)b * p.Hkv + kvh) * p.nblk + blk) * ((size_t)kBlockTokens * D);
  uint16_t* kc = (uint16_t*)p.Kc + base;
  uint16_t* vc = (uint16_t*)p.Vc + base;
  constexpr int CPR = D / 8;  // 16-byte chunks per row
  for (int c = tid; c < kBlockTokens * CPR; c += 256) {
    const int w = c / CPR, ck = c % CPR;
    const long tok = (long)blk * kBlockTokens + w;
    if (tok >= t0 && tok < t1) {
      const size_t src = ((((size_t)b * p.kmax + (size_t)(tok - off)) * p.Hkv + kvh) * D) + ck * 8;
      *(uint4*)(kc + k_elem_offset(D, w, ck * 8)) = *(const uint4*)((const uint16_t*)p.Kr + src);
      *(uint4*)&vt[w][ck * 8] = *(const uint4*)((const uint16_t*)p.Vr + src);
    }
  }
  __syncthreads();
  const bool whole = t0 == (long)blk * kBlockTokens && t1 == (long)(blk + 1) * kBlockTokens;
  for (int c = tid; c < (D / 16) * 64; c += 256) {
    const int mt = c / 64, l = c % 64, grp = l >> 4, dr = l & 15;
    uint4* dst = (uint4*)(vc + (size_t)c * 8);
    uint4 cur = make_uint4(0, 0, 0, 0);
    if (!whole) cur = *dst;
    uint16_t* e = (uint16_t*)&cur;
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) {
      const int w = jj < 4 ? 4 * grp + jj : 16 + 4 * grp + (jj - 4);
      const long tok = (long)blk * kBlockTokens + w;
      if (whole || (tok >= t0 && tok < t1)) e[jj] = vt[w][16 * mt + dr];
    }
    *dst = cur;
  }
}

template <bool kGather>
__global__ __launch_bounds__(256) void kv_rows_fp32(KvParams p) {
  const int chunks = p.D / 4;
  const long item = (long)blockIdx.x * 256 + threadIdx.x;  // over [B][kmax][Hkv][chunks]
  if (item >= (long)p.B * p.kmax * p.Hkv * chunks) return;
  const int ck = (int)(item % chunks);
  const int kvh = (int)((item / chunks) % p.Hkv);
  const int i = (int)((item / ((long)chunks * p.Hkv)) % p.kmax);
  const int b = (int)(item / ((long)chunks * p.Hkv * p.kmax));
  long tok;
  if (!row_target(p, b, i, ck == 0 && kvh == 0, tok)) return;
  const size_t row = (size_t)item * 4;
  const size_t dst = (((size_t)b * p.Hkv + kvh) * p.Lcap + tok) * p.D + ck * 4;
  if (!kGather) {
    *(float4*)((float*)p.Kc + dst) = *(const float4*)((const float*)p.Kr + row);
    *(float4*)((float*)p.Vc + dst) = *(const float4*)((const float*)p.Vr + row);
  } else {
    *(float4*)((float*)p.Kr + row) = *(const float4*)((const float*)p.Kc + dst);
    *(float4*)((float*)p.Vr + row) = *(const float4*)((const float*)p.Vc + dst);
  }
}

// ---------------------------------------------------------------------------------------
// INT8 caches.  One thread per (sequence, row slot, kv head, chunk of 8 head elements); the D/8
// threads of a row are consecutive lanes of one wavefront and agree on the row's largest
// magnitude through shuffles, so no thread may leave before them.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void kv_rows_i8_append(KvParams p) {
  const int chunks = p.D / 8;  // 8 or 16: a row's threads share an aligned group of lanes
  const long total = (long)p.B * p.kmax * p.Hkv * chunks;
  const long item_raw = (long)blockIdx.x * 256 + threadIdx.x;  // over [B][kmax][Hkv][chunks]
  const bool in_range = item_raw < total;
  const long item = in_range ? item_raw : total - 1;
  const int ck = (int)(item % chunks);
  const int kvh = (int)((item / chunks) % p.Hkv);
  const int i = (int)((item / ((long)chunks * p.Hkv)) % p.kmax);
  const int b = (int)(item / ((long)chunks * p.Hkv * p.kmax));
  long tok = 0;
  const bool ok = in_range && row_target(p, b, i, ck == 0 && kvh == 0, tok);
  uint4 kv = make_uint4(0, 0, 0, 0), vv = kv;
  if (ok) {
    kv = *(const uint4*)((const uint16_t*)p.Kr + (size_t)item * 8);
    vv = *(const uint4*)((const uint16_t*)p.Vr + (size_t)item * 8);
  }
  float ka = amax8(kv), va = amax8(vv);
  for (int o = chunks >> 1; o >= 1; o >>= 1) {
    ka = fmaxf(ka, __shfl_xor(ka, o));
    va = fmaxf(va, __shfl_xor(va, o));
  }
  if (!ok) return;
  const float kinv = ka > 0.f ? 127.0f / ka : 0.f;  // one fp32 division each
  const float vinv = va > 0.f ? 127.0f / va : 0.f;
  const int blk = (int)(tok / kBlockTokens), w = (int)(tok % kBlockTokens);
  const size_t base = (((size_t)b * p.Hkv + kvh) * p.nblk + blk) * i8_block_bytes(p.D);
  uint8_t* kc = (uint8_t*)p.Kc + base;
  uint8_t* vc = (uint8_t*)p.Vc + base;
  *(uint2*)(kc + i8_k_offset(p.D, w, ck * 8)) = quantize8(kv, kinv);  // 8 consecutive d share 8 bytes
  const uint2 vq = quantize8(vv, vinv);
#pragma unroll
  for (int e = 0; e < 8; ++e) vc[i8_v_offset(p.D, w, ck * 8 + e)] = (uint8_t)((e < 4 ? vq.x : vq.y) >> (8 * (e & 3)));
  if (ck == 0) {
    ((float*)(kc + (size_t)kBlockTokens * p.D))[w] = ka / 127.0f;
    ((float*)(vc + (size_t)kBlockTokens * p.D))[w] = va / 127.0f;
  }
}

__global__ __launch_bounds__(256) void kv_rows_i8_gather(KvParams p) {
  const int chunks = p.D / 8;
  const long item = (long)blockIdx.x * 256 + threadIdx.x;  // over [B][kmax][Hkv][chunks]
  if (item >= (long)p.B * p.kmax * p.Hkv * chunks) return;
  const int ck = (int)(item % chunks);
  const int kvh = (int)((item / chunks) % p.Hkv);
  const int i = (int)((item / ((long)chunks * p.Hkv)) % p.kmax);
  const int b = (int)(item / ((long)chunks * p.Hkv * p.kmax));
  long tok;
  if (!row_target(p, b, i, ck == 0 && kvh == 0, tok)) return;
  const int blk = (int)(tok / kBlockTokens), w = (int)(tok % kBlockTokens);
  const size_t base = (((size_t)b * p.Hkv + kvh) * p.nblk + blk) * i8_block_bytes(p.D);
  const uint8_t* kc = (const uint8_t*)p.Kc + base;
  const uint8_t* vc = (const uint8_t*)p.Vc + base;
  *(uint2*)((uint8_t*)p.Kr + (size_t)item * 8) = *(const uint2*)(kc + i8_k_offset(p.D, w, ck * 8));
  uint32_t out[2] = {0u, 0u};
#pragma unroll
  for (int e = 0; e < 8; ++e) out[e >> 2] |= (uint32_t)vc[i8_v_offset(p.D, w, ck * 8 + e)] << (8 * (e & 3));
  *(uint2*)((uint8_t*)p.Vr + (size_t)item * 8) = make_uint2(out[0], out[1]);
  if (ck == 0) {
    const size_t row = item / chunks;  // [B][kmax][Hkv]
    p.Ks[row] = ((const float*)(kc + (size_t)kBlockTokens * p.D))[w];
    p.Vs[row] = ((const float*)(vc + (size_t)kBlockTokens * p.D))[w];
  }
}

template <bool kGather>
static int launch_rows(const bass_attn_desc* d, void* Kc, void* Vc, void* Kr, void* Vr, const int32_t* off,
                       const int32_t* cnt, int32_t* status, void* stream, float* Ks = nullptr, float* Vs = nullptr) {
  int rc = check_desc(d);
  if (rc != BASS_OK) return rc;
  if (!Kc || !Vc || !Kr || !Vr || !off || !cnt) return BASS_ERR_INVALID_ARG;
  if (d->dtype == BASS_DTYPE_INT8KV && (kGather != (Ks != nullptr) || kGather != (Vs != nullptr)))
    return BASS_ERR_UNSUPPORTED;  // INT8 caches are read back with bass_kv_gather_int8
  if (d->dtype != BASS_DTYPE_INT8KV && Ks) return BASS_ERR_UNSUPPORTED;
  const int chunk = d->dtype == BASS_DTYPE_FP32 ? 4 : 8;
  const int64_t items = (int64_t)d->B * d->kmax * d->Hkv * (d->D / chunk);
  if ((items + 255) / 256 > 0x7fffffff) return BASS_ERR_UNSUPPORTED;
  KvParams p{d->B, d->kmax, d->Hkv, d->D, d->Lcap, num_blocks(d->Lcap), Kc, Vc, Kr, Vr, off, cnt, status, Ks, Vs};
  dim3 grid((unsigned)((items + 255) / 256));
  hipStream_t s = (hipStream_t)stream;
  if (d->dtype == BASS_DTYPE_INT8KV) {
    if (kGather) hipLaunchKernelGGL(kv_rows_i8_gather, grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL(kv_rows_i8_append, grid, dim3(256), 0, s, p);
  } else if (d->dtype == BASS_DTYPE_BF16) {
    const int64_t per_seq = (d->kmax + kBlockTokens - 1) / kBlockTokens + 1;  // blocks the rows of a sequence can touch
    const int64_t wgs = (int64_t)d->B * d->Hkv * per_seq;
    if (!kGather && d->kmax >= kBlockTokens && wgs <= 0x7fffffff) {
      if (d->D == 128) hipLaunchKernelGGL(kv_blocks_bf16<128>, dim3((unsigned)wgs), dim3(256), 0, s, p, (int)per_seq);
      else hipLaunchKernelGGL(kv_blocks_bf16<64>, dim3((unsigned)wgs), dim3(256), 0, s, p, (int)per_seq);
    } else {
      hipLaunchKernelGGL(kv_rows_bf16<kGather>, grid, dim3(256), 0, s, p);
    }
  } else
    hipLaunchKernelGGL(kv_rows_fp32<kGather>, grid, dim3(256), 0, s, p);
  return launch_status();
}

}  // namespace bass

extern "C" size_t bass_kv_cache_bytes(const bass_attn_desc* d) {
  if (bass::check_desc(d) != BASS_OK) return 0;
  if (d->dtype == BASS_DTYPE_INT8KV)
    return (size_t)d->B * d->Hkv * bass::num_blocks(d->Lcap) * bass::i8_block_bytes(d->D);
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

extern "C" int bass_kv_gather_int8(const bass_attn_desc* desc, const void* Kcache, const void* Vcache,
                                   int8_t* K_codes, int8_t* V_codes, float* K_scales, float* V_scales,
                                   const int32_t* start, const int32_t* n, int32_t* dev_status, void* stream) {
  if (!desc || desc->dtype != BASS_DTYPE_INT8KV) return desc ? BASS_ERR_UNSUPPORTED : BASS_ERR_INVALID_ARG;
  if (!K_scales || !V_scales) return BASS_ERR_INVALID_ARG;
  return bass::launch_rows<true>(desc, (void*)Kcache, (void*)Vcache, K_codes, V_codes, start, n, dev_status, stream,
                                 K_scales, V_scales);
}
