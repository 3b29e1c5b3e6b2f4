// Device code of the logits front end (temperature, nucleus top-p, softmax): the warp of one row by one
// workgroup, shared by bass_warp_probs (which stores the probability rows) and bass_warp_accept (which keeps
// only a summary per row).
//
// The paper's experiments sample at temperature 0.2 with nucleus top-p 0.95 (captions of the
// result tables of Section 4); the acceptance rule of Section 2.2 compares the probabilities the
// main and the draft model assign after that warp.
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
// bit patterns of e_i (positive floats order like their bit patterns): digits of 8 bits, each a mass
// histogram per wavefront in LDS (64-bit LDS atomics) followed by a suffix scan over the 256 bins.
// When the bin of the first digit can hold at most 64 tokens (peaked rows: low temperatures), they are
// collected and ranked by one wavefront and the other three digits are skipped.  Tokens that tie with
// the threshold value are ranked by token id in a pass of their own (rare: it runs only if not all of
// them are kept).
//
// A compute unit fetches at most some 150 GB/s, so every pass over a 200 KB row from memory or L2
// costs it microseconds.  Rows of up to 65536 aligned logits are therefore read ONCE, into registers
// (NG 16-byte groups per thread), and all passes run on the registers; only the result is stored.
// Longer or unaligned rows take the streaming variant (NG = 0): e_i is written into the output row in
// the first pass and re-read from L2 by the later ones.
#pragma once
#include "bass_common.h"

namespace bass {

constexpr int kWarpThreads = 1024;
constexpr int kWarpWaves = kWarpThreads / kWave;
constexpr int kWarpMaxVocab = 1 << 19;  // keeps the mass sum below 2^59
constexpr float kMassScale = 1099511627776.0f;  // 2^40

// log2(e) / T: the factor of (z - z_max) in the exponent
inline float warp_exponent_scale(float temperature) { return (float)(1.4426950408889634 / (double)temperature); }

// Which variant serves rows of V logits: 1 = unaligned rows, one logit per load, streaming; 8 / 13 / 16 = that
// many 16-byte groups per thread held in registers; 0 = 16-byte loads, streaming
inline int warp_variant(int V, bool rows_16_byte_aligned) {
  if (!rows_16_byte_aligned) return 1;
  if (V <= 8 * 4 * kWarpThreads) return 8;
  if (V <= 13 * 4 * kWarpThreads) return 13;
  if (V <= 16 * 4 * kWarpThreads) return 16;
  return 0;
}

__device__ inline float warp_e(float z, float zmax, float c) {
  return z == zmax ? 1.f : __builtin_amdgcn_exp2f((z - zmax) * c);
}

// Integer mass floor(e * 2^40) of 2^-40 <= e <= 1 in two exact steps: the integer part of e * 2^8, and
// the fraction of it times 2^32 (scalings by powers of two and v_fract are exact).
constexpr float kMinMassive = 9.094947017729282e-13f;  // 2^-40: smaller e (and NaN) have mass 0
__device__ inline bool has_mass(float e) { return e >= kMinMassive; }
__device__ inline uint64_t mass_of(float e) {  // needs has_mass(e)
  const float a = e * 256.0f;
  const uint32_t hi = (uint32_t)a;
  const uint32_t lo = (uint32_t)(__builtin_amdgcn_fractf(a) * 4294967296.0f);
  return ((uint64_t)hi << 32) | lo;
}
// Keys (bit patterns) of e: positive floats order like their keys, so "e has mass and its key starts with
// these high bits" is one unsigned range test, (key - lo) < width, which NaN patterns fail as well.
constexpr uint32_t kMinMassiveKey = 0x2B800000u;  // key of 2^-40
struct KeyRange {
  uint32_t lo, width;
  __device__ bool has(uint32_t key) const { return key - lo < width; }
};
// keys whose bits above `shift` equal `prefix` (shift < 32), restricted to keys with mass
__device__ inline KeyRange keys_with_prefix(uint32_t prefix, int shift) {
  const uint32_t first = prefix << shift, lo = max(first, kMinMassiveKey);
  const uint32_t end_minus_1 = first | ((1u << shift) - 1u);  // last key of the range
  return KeyRange{lo, end_minus_1 >= lo ? end_minus_1 - lo + 1u : 0u};
}
__device__ inline uint64_t warp_mass(float e) { return has_mass(e) ? mass_of(e) : 0; }

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

// What a token of a warped row gets, given its logit and its id: enough to evaluate single entries of the
// row (the acceptance test needs one per draft, the corrected draw one pass over one row pair) without the
// row ever being stored.
struct RowSummary {
  float zmax, inv;                 // e = 2^((z - zmax) c), probability e * inv
  uint32_t key_first, key_count;   // kept: keys (bit patterns of e) with key - key_first < key_count ...
  uint32_t key_tie;                // ... and the tokens of this key with id <= tie_last (ties at the
  int32_t tie_last;                //     threshold are taken by token id); -1: none
  uint32_t reserved[2];
};

__device__ inline float warped_prob(const RowSummary& s, float c, float z, int id) {
  const float e = warp_e(z, s.zmax, c);
  const uint32_t key = __float_as_uint(e);
  const bool kept = (key - s.key_first < s.key_count) || (key == s.key_tie && id <= s.tie_last);
  return kept ? e * s.inv : 0.f;
}

// The warp of one row by one workgroup of kWarpThreads threads.
// NG > 0: the row lives in registers, NG groups of W = 4 per thread (V <= 4096 NG); NG = 0: streaming.
// kSummary = false: the probabilities are written to `out`.  kSummary = true: nothing of the row is written,
// *summary receives what warped_prob needs (the streaming variant then recomputes e_i from the logits in every
// pass instead of re-reading it from the output row).
template <int W, int NG, bool kSummary>
__device__ __forceinline__ void warp_row(const float* z, float* out, int V, float c_arg, float top_p_arg, int32_t* status_arg,
                                RowSummary* summary) {
  struct { int V; float c, top_p; int32_t* status; } a{V, c_arg, top_p_arg, status_arg};
  __shared__ uint64_t hist[kWarpWaves][256];
  __shared__ uint64_t red64[kWarpWaves];
  __shared__ float redf[kWarpWaves];
  __shared__ int sh_cross[2];       // position (255 - bin) where the cumulative mass first reaches the target (by pass parity)
  __shared__ uint64_t sh_cum[256];  // cumulative mass down to each position, and the mass of the position itself
  __shared__ uint64_t sh_tot[256];
  __shared__ int tie_count[kWarpWaves];
  __shared__ uint32_t sh_cand[kWave];  // keys of the tokens of the first digit's bin, if there are at most 64
  __shared__ int sh_ncand;
  __shared__ int sh_tie_last;       // summary mode: id of the last tie that is kept

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int groups = V / W;

  // register variant: group k of this thread is g = tid + 1024 k (all loads issued at once)
  Group<W> held[NG > 0 ? NG : 1];
  if constexpr (NG > 0) {
#pragma unroll
    for (int k = 0; k < NG; ++k) held[k] = load_group<W>(z, min(tid + k * kWarpThreads, groups - 1));
  }

  // f(g, values, slot) for this thread's groups g = tid, tid + 1024, ... of the row as it stands (the logits at
  // first, the e_i after the first pass).  Streaming variant: a batch of loads from `row` first, then the work.
  auto for_each_group = [&](const float* row, auto&& f) {
    if constexpr (NG > 0) {
#pragma unroll
      for (int k = 0; k < NG; ++k) {
        const int g = tid + k * kWarpThreads;
        if (g < groups) f(g, held[k], k);
      }
    } else {
      for (int base = tid; base < groups; base += kWarpUnroll * kWarpThreads) {
        Group<W> gr[kWarpUnroll];
#pragma unroll
        for (int k = 0; k < kWarpUnroll; ++k) gr[k] = load_group<W>(row, min(base + k * kWarpThreads, groups - 1));
#pragma unroll
        for (int k = 0; k < kWarpUnroll; ++k) {
          const int g = base + k * kWarpThreads;
          if (g < groups) f(g, gr[k], 0);
        }
      }
    }
  };
  // the e_i replace the logits: in the registers, or in the output row
  auto keep_group = [&](int g, int k, const Group<W>& ev) {  // k: the slot for_each_group handed out
    if constexpr (NG > 0) held[k] = ev;
    else if constexpr (!kSummary) store_group<W>(out, g, ev);
  };

  // largest logit (NaN entries are ignored)
  float m = -INFINITY;
  for_each_group(z, [&](int, const Group<W>& gr, int) {
#pragma unroll
    for (int e = 0; e < W; ++e) m = fmaxf(m, gr.v[e]);
  });
  m = wave_max_f32(m);
  if (lane == 0) redf[wave] = m;
  __syncthreads();
  float zmax = redf[0];
#pragma unroll
  for (int k = 1; k < kWarpWaves; ++k) zmax = fmaxf(zmax, redf[k]);
  if (!(zmax > -INFINITY)) {  // no finite logit at all: a row without mass
    if constexpr (kSummary) {
      if (tid == 0) *summary = RowSummary{zmax, 0.f, 0u, 0u, 0xFFFFFFFFu, -1, {0u, 0u}};  // nothing is kept
    } else {
      for (int i = tid; i < V; i += kWarpThreads) out[i] = 0.f;
    }
    if (tid == 0 && a.status) atomicOr(a.status, BASS_STATUS_ZERO_MASS);
    return;
  }
  // f(g, values, slot) on the e_i, once the first pass has made them
  auto for_each_e = [&](auto&& f) {
    if constexpr (NG > 0 || !kSummary) {
      for_each_group(out, f);
    } else {  // nowhere to keep them: recomputed from the logits (the same function of the same inputs: the same bits)
      for_each_group(z, [&](int g, const Group<W>& gr, int k) {
        Group<W> ev;
#pragma unroll
        for (int e = 0; e < W; ++e) ev.v[e] = warp_e(gr.v[e], zmax, a.c);
        f(g, ev, k);
      });
    }
  };

  const bool keep_all = a.top_p >= 1.0f;
  uint32_t prefix = 0;   // selected high bits of the threshold key
  uint64_t above = 0;    // mass of keys above the selected prefix
  uint64_t S = 0, target = 0, bin_mass = 0;
  bool few = false;      // the first digit leaves at most 64 candidates

#pragma unroll 1
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    for (int k = tid; k < kWarpWaves * 256; k += kWarpThreads) (&hist[0][0])[k] = 0;
    if (tid == 0) sh_cross[pass & 1] = 256;
    __syncthreads();
    if (pass == 0) {
      // e_i replace the logits (in the registers, or in the output row: each thread re-reads what it wrote)
      if (keep_all) {  // plain softmax: only the total mass is needed
        uint64_t mine = 0;
        for_each_group(z, [&](int g, const Group<W>& gr, int k) {
          Group<W> ev;
#pragma unroll
          for (int e = 0; e < W; ++e) {
            ev.v[e] = warp_e(gr.v[e], zmax, a.c);
            mine += warp_mass(ev.v[e]);
          }
          keep_group(g, k, ev);
        });
        mine = wave_sum_u64(mine);
        if (lane == 0) red64[wave] = mine;
        __syncthreads();
        for (int k = 0; k < kWarpWaves; ++k) S += red64[k];
        target = S;
        break;
      }
      for_each_group(z, [&](int g, const Group<W>& gr, int k) {
        Group<W> ev;
#pragma unroll
        for (int e = 0; e < W; ++e) {
          ev.v[e] = warp_e(gr.v[e], zmax, a.c);
          if (has_mass(ev.v[e]))
            atomicAdd((unsigned long long*)&hist[wave][__float_as_uint(ev.v[e]) >> 24], (unsigned long long)mass_of(ev.v[e]));
        }
        keep_group(g, k, ev);
      });
    } else {  // only the tokens of the selected bin take part (their mass is not 0)
      const KeyRange bin = keys_with_prefix(prefix, shift + 8);
      for_each_e([&](int, const Group<W>& gr, int) {
        bool in[W], any = false;
#pragma unroll
        for (int e = 0; e < W; ++e) {
          in[e] = bin.has(__float_as_uint(gr.v[e]));
          any |= in[e];
        }
        if (any) {  // one branch per group: most groups hold no token of the bin
#pragma unroll
          for (int e = 0; e < W; ++e)
            if (in[e])
              atomicAdd((unsigned long long*)&hist[wave][(__float_as_uint(gr.v[e]) >> shift) & 255u],
                        (unsigned long long)mass_of(gr.v[e]));
        }
      });
    }
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
    if (pass == 0) {  // total mass = all bins; the mass the nucleus has to reach
      S = red64[0] + red64[1] + red64[2] + red64[3];
      double t = ceil((double)a.top_p * (double)S);
      if (t < 1.0) t = 1.0;
      target = t >= (double)S ? S : (uint64_t)t;
    }
    if (tid < 256) {
      for (int k = 0; k < wave; ++k) cum += red64[k];
      cum += above;
      sh_cum[tid] = cum;
      sh_tot[tid] = tot;
      // first position that reaches the target: one LDS atomic per wavefront
      const unsigned long long reached = __ballot(cum >= target);
      if (reached && lane == 0) atomicMin(&sh_cross[pass & 1], wave * 64 + (int)__builtin_ctzll(reached));
    }
    __syncthreads();
    const int cross = min(sh_cross[pass & 1], 255);  // always found: the cumulative mass of all bins reaches the target
    prefix = (prefix << 8) | (uint32_t)(255 - cross);
    bin_mass = sh_tot[cross];
    above = sh_cum[cross] - bin_mass;
    if (pass == 0) {
      // Every token of the selected bin weighs at least as much as the bin's lower edge (at least 1): if
      // that bounds their number by 64, one wavefront can rank them directly (the usual case at low
      // temperatures, where the row is peaked) and the three remaining digits are not needed.
      const float e_lo = __uint_as_float(prefix << 24);
      const uint64_t w_lo = has_mass(e_lo) ? mass_of(e_lo) : 1;
      if (bin_mass <= (uint64_t)kWave * w_lo) {
        few = true;
        break;
      }
    }
  }
  if (few) {
    if (tid == 0) sh_ncand = 0;
    __syncthreads();
    const KeyRange bin = keys_with_prefix(prefix, 24);
    for_each_e([&](int, const Group<W>& gr, int) {
      bool in[W], any = false;
#pragma unroll
      for (int e = 0; e < W; ++e) {
        in[e] = bin.has(__float_as_uint(gr.v[e]));
        any |= in[e];
      }
      if (any) {
#pragma unroll
        for (int e = 0; e < W; ++e)
          if (in[e]) {
            const int pos = atomicAdd(&sh_ncand, 1);
            if (pos < kWave) sh_cand[pos] = __float_as_uint(gr.v[e]);
          }
      }
    });
    __syncthreads();
    // every wavefront ranks the candidates for itself: lane i holds one, and adds up the mass of those
    // that are at least as large (ge) and strictly larger (gt) than its own
    const int n = min(sh_ncand, kWave);
    const uint32_t key = lane < n ? sh_cand[lane] : 0u;
    uint64_t ge = above, gt = above;
    for (int j = 0; j < n; ++j) {
      const uint32_t kj = (uint32_t)__builtin_amdgcn_readlane((int)key, j);
      const uint64_t mj = mass_of(__uint_as_float(kj));
      if (kj >= key) ge += mj;
      if (kj > key) gt += mj;
    }
    // the threshold is the largest key whose cumulative mass (ties included) reaches the target; the
    // smallest candidate always does (its ge is the mass down to the end of the bin)
    uint32_t kthr = (lane < n && ge >= target) ? key : 0u;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) kthr = max(kthr, (uint32_t)__shfl_xor((int)kthr, o));
    const int src = (int)__builtin_ctzll(__ballot(lane < n && key == kthr) | (1ull << 63));
    auto from_lane = [&](uint64_t v) {  // the builtin returns a signed int: widen both halves as unsigned
      const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), src);
      const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, src);
      return ((uint64_t)hi << 32) | lo;
    };
    const uint64_t ge_t = from_lane(ge), gt_t = from_lane(gt);
    prefix = kthr;
    above = gt_t;
    bin_mass = ge_t - gt_t;
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
  const float e_thr = __uint_as_float(prefix);
  // kept keys: from the threshold (or just above it, if not all ties are kept; from the smallest positive
  // value for the plain softmax) up to the key of 1.0
  const uint32_t key_first = keep_all ? 1u : ties_all_kept ? prefix : prefix + 1u;
  const KeyRange kept_keys{key_first, 0x3F800000u - key_first + 1u};

  if constexpr (!kSummary) {
    for_each_e([&](int g, const Group<W>& gr, int) {
      Group<W> pv;
#pragma unroll
      for (int e = 0; e < W; ++e) {
        const float ei = gr.v[e];
        pv.v[e] = kept_keys.has(__float_as_uint(ei)) ? ei * inv : 0.f;
      }
      store_group<W>(out, g, pv);
    });
    if (keep_all || ties_all_kept) return;
  } else {
    if (tid == 0) {
      sh_tie_last = -1;
      if (keep_all || ties_all_kept) *summary = RowSummary{zmax, inv, kept_keys.lo, kept_keys.width, 0xFFFFFFFFu, -1, {0u, 0u}};
    }
    if (keep_all || ties_all_kept) return;
  }

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
  if constexpr (!kSummary) {
    for (int i = lo; i < hi && (uint64_t)rank < need; ++i) {
      const float e = warp_e(z[i], zmax, a.c);
      if (e == e_thr) {
        out[i] = e * inv;
        ++rank;
      }
    }
  } else {
    // the thread whose range holds the need-th tie names it (1 <= need < number of ties)
    if ((uint64_t)rank < need && need <= (uint64_t)rank + (uint64_t)cnt) {
      for (int i = lo; i < hi; ++i)
        if (warp_e(z[i], zmax, a.c) == e_thr && (uint64_t)++rank == need) sh_tie_last = i;
    }
    __syncthreads();
    if (tid == 0) *summary = RowSummary{zmax, inv, kept_keys.lo, kept_keys.width, prefix, sh_tie_last, {0u, 0u}};
  }
}

}  // namespace bass
