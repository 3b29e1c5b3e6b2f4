// Logits front end of libbass: bass_warp_probs (temperature, nucleus top-p, softmax).
//
// The paper's experiments sample at temperature 0.2 with nucleus top-p 0.95 (captions of the
// result tables of Section 4); the acceptance rule of Section 2.2 compares the probabilities the
// main and the draft model assign after that warp.  This kernel turns rows of logits into those
// probability rows.
//
// Per row: e_i = 2^((z_i - z_max) * log2(e) / T); order the tokens by decreasing e_i, equal values
// by increasing token id; keep the shortest prefix whose mass reaches top_p of the total; output
// e_i / (kept mass) on the kept tokens and 0 elsewhere.
//
// Exactness.  Which tokens are kept is decided in integer arithmetic: masses are the integers
// w_i = floor(e_i * 2^40), sums of them are associative, the threshold is
// ceil(top_p * sum) evaluated once in fp64, so the kept set and the normaliser do not depend on the
// order in which wavefronts add things up and every run gives the same bits.
//
// One workgroup of 16 wavefronts per row.  The threshold value is found by a radix select over the
// bit patterns of e_i (positive floats order like their bit patterns): four passes of 8 bits, each
// a mass histogram per wavefront in LDS (64-bit LDS atomics) followed by a suffix scan over the 256
// bins.  Tokens that tie with the threshold value are ranked by token id in a pass of their own
// (rare: it runs only if not all of them are kept).  The values e_i are written into the output row in
// the first pass and re-read from L2 by the later ones (16-byte accesses when rows are aligned).
#include "bass_common.h"

namespace bass {

constexpr int kWarpThreads = 1024;
constexpr int kWarpWaves = kWarpThreads / kWave;
constexpr int kWarpMaxVocab = 1 << 19;  // keeps the mass sum below 2^59
constexpr float kMassScale = 1099511627776.0f;  // 2^40

struct WarpParams {
  int R, V;
  const float* logits;
  float* probs;
  float c;      // log2(e) / T
  float top_p;
  int32_t* status;
};

__device__ inline float warp_e(float z, float zmax, float c) {
  return z == zmax ? 1.f : __builtin_amdgcn_exp2f((z - zmax) * c);
}

__device__ inline uint64_t warp_mass(float e) { return e > 0.f ? (uint64_t)(e * kMassScale) : 0; }  // NaN -> 0

__device__ inline uint64_t wave_sum64(uint64_t v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += (uint64_t)__shfl_xor((unsigned long long)v, o);
  return v;
}

__device__ inline uint64_t wave_incl_scan_u64(uint64_t v, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint64_t o = (uint64_t)__shfl_up((unsigned long long)v, d);
    if (lane >= d) v += o;
  }
  return v;
}

constexpr int kWarpUnroll = 8;  // groups a thread keeps in flight

// W logits per thread and load: 4 (16-byte loads; V a multiple of 4 and 16-byte aligned rows) or 1
template <int W>
struct Group {
  float v[W];
};

template <int W>
__device__ inline Group<W> load_group(const float* row, int g) {
  Group<W> r;
  if constexpr (W == 4) {
    const float4 t = ((const float4*)row)[g];
    r.v[0] = t.x; r.v[1] = t.y; r.v[2] = t.z; r.v[3] = t.w;
  } else {
    r.v[0] = row[g];
  }
  return r;
}

template <int W>
__device__ inline void store_group(float* row, int g, const Group<W>& r) {
  if constexpr (W == 4) ((float4*)row)[g] = make_float4(r.v[0], r.v[1], r.v[2], r.v[3]);
  else row[g] = r.v[0];
}

template <int W>
__global__ __launch_bounds__(kWarpThreads) void warp_probs_kernel(WarpParams a) {
  __shared__ uint64_t hist[kWarpWaves][256];
  __shared__ uint64_t red64[kWarpWaves];
  __shared__ float redf[kWarpWaves];
  __shared__ int sh_cross;          // position (255 - bin) where the cumulative mass first reaches the target
  __shared__ uint64_t sh_above;     // mass of the bins above the selected one
  __shared__ uint64_t sh_bin_mass;  // mass of the selected bin
  __shared__ int tie_count[kWarpWaves];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int V = a.V;
  const int groups = V / W;
  const float* z = a.logits + (size_t)blockIdx.x * V;
  float* out = a.probs + (size_t)blockIdx.x * V;

  // f(g, values) for this thread's groups g = tid, tid + 1024, ... of a row: a batch of loads first, then the work
  auto for_each_group = [&](const float* row, auto f) {
    for (int base = tid; base < groups; base += kWarpUnroll * kWarpThreads) {
      Group<W> gr[kWarpUnroll];
#pragma unroll
      for (int k = 0; k < kWarpUnroll; ++k) gr[k] = load_group<W>(row, min(base + k * kWarpThreads, groups - 1));
#pragma unroll
      for (int k = 0; k < kWarpUnroll; ++k) {
        const int g = base + k * kWarpThreads;
        if (g < groups) f(g, gr[k]);
      }
    }
  };

  // largest logit (NaN entries are ignored)
  float m = -INFINITY;
  for_each_group(z, [&](int, const Group<W>& gr) {
#pragma unroll
    for (int e = 0; e < W; ++e) m = fmaxf(m, gr.v[e]);
  });
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
  if (lane == 0) redf[wave] = m;
  __syncthreads();
  float zmax = redf[0];
#pragma unroll
  for (int k = 1; k < kWarpWaves; ++k) zmax = fmaxf(zmax, redf[k]);
  if (!(zmax > -INFINITY)) {  // no finite logit at all: a row without mass
    for (int i = tid; i < V; i += kWarpThreads) out[i] = 0.f;
    if (tid == 0 && a.status) atomicOr(a.status, BASS_STATUS_ZERO_MASS);
    return;
  }

  const bool keep_all = a.top_p >= 1.0f;
  uint32_t prefix = 0;   // selected high bits of the threshold key
  uint64_t above = 0;    // mass of keys above the selected prefix
  uint64_t S = 0, target = 0, bin_mass = 0;

  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    for (int k = tid; k < kWarpWaves * 256; k += kWarpThreads) (&hist[0][0])[k] = 0;
    __syncthreads();
    if (pass == 0) {
      // e_i from the logits, kept in the output row for the later passes (each thread re-reads what it wrote)
      uint64_t mine = 0;
      for_each_group(z, [&](int g, const Group<W>& gr) {
        Group<W> ev;
#pragma unroll
        for (int e = 0; e < W; ++e) {
          ev.v[e] = warp_e(gr.v[e], zmax, a.c);
          const uint64_t w = warp_mass(ev.v[e]);
          mine += w;
          if (w && !keep_all) atomicAdd((unsigned long long*)&hist[wave][__float_as_uint(ev.v[e]) >> 24], (unsigned long long)w);
        }
        store_group<W>(out, g, ev);
      });
      // total mass and the mass the nucleus has to reach
      mine = wave_sum64(mine);
      if (lane == 0) red64[wave] = mine;
      __syncthreads();
      for (int k = 0; k < kWarpWaves; ++k) S += red64[k];
      double t = ceil((double)a.top_p * (double)S);
      if (t < 1.0) t = 1.0;
      target = keep_all || t >= (double)S ? S : (uint64_t)t;
      if (keep_all) break;
    } else {  // only the tokens of the selected bin take part (e >= 2^-40 there: the mass is not 0)
      for_each_group(out, [&](int, const Group<W>& gr) {
#pragma unroll
        for (int e = 0; e < W; ++e) {
          const uint32_t key = __float_as_uint(gr.v[e]);
          if (gr.v[e] > 0.f && (key >> (shift + 8)) == prefix)
            atomicAdd((unsigned long long*)&hist[wave][(key >> shift) & 255u], (unsigned long long)warp_mass(gr.v[e]));
        }
      });
    }
    if (tid == 0) sh_cross = 256;
    __syncthreads();
    // bins in decreasing order: position t holds bin 255 - t; cumulative mass from the top
    uint64_t tot = 0, cum = 0;
    if (tid < 256) {
#pragma unroll
      for (int k = 0; k < kWarpWaves; ++k) tot += hist[k][255 - tid];
      cum = wave_incl_scan_u64(tot, lane);
      if (lane == 63) red64[wave] = cum;
    }
    __syncthreads();
    if (tid < 256) {
      for (int k = 0; k < wave; ++k) cum += red64[k];
      cum += above;
      if (cum >= target) atomicMin(&sh_cross, tid);  // first position that reaches the target
    }
    __syncthreads();
    if (tid < 256 && tid == sh_cross) {
      sh_above = cum - tot;
      sh_bin_mass = tot;
    }
    __syncthreads();
    prefix = (prefix << 8) | (uint32_t)(255 - sh_cross);
    above = sh_above;
    bin_mass = sh_bin_mass;
    __syncthreads();
  }

  // threshold key = prefix; its tokens all weigh w_thr; `need` of the n_thr ties are kept (by token id)
  uint64_t K = S, need = 0, n_thr = 0;
  if (!keep_all) {
    const uint64_t w_thr = warp_mass(__uint_as_float(prefix));
    n_thr = bin_mass / w_thr;
    need = (target - above + w_thr - 1) / w_thr;
    K = above + need * w_thr;
  }
  const bool ties_all_kept = need == n_thr;
  const float inv = (float)((double)kMassScale / (double)K);
  const float e_thr = __uint_as_float(prefix);  // e_i >= 0: floats order like their bit patterns; NaN compares false

  for_each_group(out, [&](int g, const Group<W>& gr) {
    Group<W> pv;
#pragma unroll
    for (int e = 0; e < W; ++e) {
      const float ei = gr.v[e];
      const bool kept = keep_all ? ei > 0.f : (ei > e_thr || (ei == e_thr && ties_all_kept));
      pv.v[e] = kept ? ei * inv : 0.f;
    }
    store_group<W>(out, g, pv);
  });
  if (keep_all || ties_all_kept) return;

  // the first `need` tokens (by id) among those that tie with the threshold: contiguous ids per thread
  __syncthreads();  // the zeros written above must not overtake the values written below
  const int per = (V + kWarpThreads - 1) / kWarpThreads;
  const int lo = min(V, tid * per), hi = min(V, lo + per);
  int cnt = 0;
  for (int i = lo; i < hi; ++i) cnt += warp_e(z[i], zmax, a.c) == e_thr;
  int incl = cnt;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int o = __shfl_up(incl, d);
    if (lane >= d) incl += o;
  }
  if (lane == 63) tie_count[wave] = incl;
  __syncthreads();
  int rank = incl - cnt;
  for (int k = 0; k < wave; ++k) rank += tie_count[k];
  for (int i = lo; i < hi && (uint64_t)rank < need; ++i) {
    const float e = warp_e(z[i], zmax, a.c);
    if (e == e_thr) {
      out[i] = e * inv;
      ++rank;
    }
  }
}

}  // namespace bass

extern "C" int bass_warp_probs(int32_t R, int32_t V, const float* logits, float temperature, float top_p,
                               float* probs, int32_t* dev_status, void* stream) {
  using namespace bass;
  if (R <= 0 || V <= 0 || !logits || !probs) return BASS_ERR_INVALID_ARG;
  if (!(temperature > 0.f) || !(top_p > 0.f)) return BASS_ERR_INVALID_ARG;
  if (V > kWarpMaxVocab) return BASS_ERR_UNSUPPORTED;
  WarpParams a{R, V, logits, probs, (float)(1.4426950408889634 / (double)temperature), top_p, dev_status};
  const bool wide = V % 4 == 0 && (((uintptr_t)logits | (uintptr_t)probs) & 15) == 0;  // rows 16-byte aligned
  if (wide) hipLaunchKernelGGL(warp_probs_kernel<4>, dim3((unsigned)R), dim3(kWarpThreads), 0, (hipStream_t)stream, a);
  else hipLaunchKernelGGL(warp_probs_kernel<1>, dim3((unsigned)R), dim3(kWarpThreads), 0, (hipStream_t)stream, a);
  return launch_status();
}
