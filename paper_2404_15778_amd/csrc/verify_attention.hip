// Ragged verify attention of libbass: bass_verify_attention.
//
// BASS paper, Section 3.2 (attention flow): scores of the current tokens' queries against
// the keys of all tokens processed so far, P = softmax(Q^T K / c), then P times V, with
// ragged K, V, P because every sequence has its own length.  Section 2.2: the draft tokens
// are processed as incremental context encoding, i.e. causally among themselves.  BASS-PAD
// gives padded positions probability zero, BASS-SPLIT computes every sequence at its true
// length with one launch per sequence; here ONE launch covers all sequences at their true
// lengths, and nothing outside a sequence's valid range is read.
//
// Work decomposition.  Attention shares no reads between sequences (Section 3.2), so the
// cost is streaming every valid K and V row once.  All (sequence, kv-head) units are cut
// into 32-token cache blocks and laid end to end; that flattened list is divided evenly
// over a fixed number of wavefronts.  A wavefront streams its contiguous share of blocks
// (registers are filled by 1 KiB-contiguous loads of MFMA-ordered cache blocks, next block
// in flight while the current one is computed), keeps an online softmax (running max and
// sum per query row) and, for every unit it touches, writes one partial (max, sum,
// unnormalised output).  A second kernel merges the partials of each unit
// (split-context reduction) and writes O and the log-sum-exp.
//
// Matrix-core mapping (v_mfma_f32_16x16x32_bf16, wave64).  Tokens sit on the M side:
//   S^T[16 tokens x 16 query rows] = K[16 x D] * Q^T[D x 16]          (D/32 MFMAs per tile)
//   O^T[D x 16 query rows]        += V^T[D x 32 tokens] * P^T[32 x 16] (D/16 MFMAs per block)
// The result layout of the first (a lane owns 4 consecutive tokens of one query row) is,
// for two 16-token tiles, exactly the operand layout of the second once the V block is
// stored in that token order, so P goes from accumulator to operand with a bf16 pack only.
// Query rows of one kv head are (draft i, head-in-group) pairs, up to 64 rows = 4 tiles.
#include "bass_common.h"

namespace bass {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

static int g_attention_waves = 0;  // 0 = default

static int attention_waves() {
  int w = g_attention_waves > 0 ? g_attention_waves : kDefaultWaves;
  if (w < 64) w = 64;
  if (w > kMaxWaves) w = kMaxWaves;
  return w & ~3;  // four wavefronts per workgroup
}

struct AttnParams {
  int B, kmax, Hq, Hkv, D, Lcap, nblk_cap, g, rows_max, nwaves;
  float scale_log2;  // scale * log2(e): scores are kept in the log2 domain
  const void* Q;
  const void* Kc;
  const void* Vc;
  const int32_t* ctx_len;
  const int32_t* draft_len;
  float* O;
  float* lse;
  float* part_acc;  // [slots][rows_max][D]
  float* part_ml;   // [slots][rows_max][2]  (running max in log2 units, running sum)
  int32_t* status;
};

// ---------------------------------------------------------------------------------------
// Flattened schedule, recomputed by every wavefront from the device-side lengths.
// ---------------------------------------------------------------------------------------
__device__ inline int wave_incl_scan(int v, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int o = __shfl_up(v, d);
    if (lane >= d) v += o;
  }
  return v;
}

__device__ inline int seq_blocks(const AttnParams& p, int b, int& L, int& nq, bool& bad) {
  L = p.ctx_len[b];
  nq = p.draft_len[b];
  bad = clamp_lengths(L, nq, p.kmax, p.Lcap);
  return nq > 0 ? (L + nq + kBlockTokens - 1) / kBlockTokens : 0;
}

// Sum over sequences of blocks per kv head (wave-uniform).  Raises the status bit once.
__device__ inline int total_seq_blocks(const AttnParams& p, int lane, bool report) {
  int total = 0;
  bool any_bad = false;
  for (int c0 = 0; c0 < p.B; c0 += 64) {
    const int b = c0 + lane;
    int L, nq, nb = 0;
    bool bad = false;
    if (b < p.B) nb = seq_blocks(p, b, L, nq, bad);
    any_bad |= bad;
    const int inc = wave_incl_scan(nb, lane);
    total += __shfl(inc, 63);
  }
  if (report && p.status && __any(any_bad) && lane == 0) atomicOr(p.status, BASS_STATUS_LEN_CLAMPED);
  return total;
}

struct Unit {
  int b, kvh, L, nq, nblk;
  int begin;  // flattened index of the unit's first block
};

// Unit containing flattened block x (0 <= x < Hkv * total_seq_blocks); wave-uniform.
__device__ inline Unit locate(const AttnParams& p, int x, int lane) {
  Unit u{0, 0, 0, 0, 0, 0};
  int running = 0;
  for (int c0 = 0; c0 < p.B; c0 += 64) {
    const int b = c0 + lane;
    int L = 0, nq = 0, nb = 0;
    bool bad;
    if (b < p.B) nb = seq_blocks(p, b, L, nq, bad);
    const int inc = running + wave_incl_scan(nb, lane);
    const unsigned long long hit = __ballot((long long)inc * p.Hkv > (long long)x);
    if (hit) {
      const int src = __ffsll((long long)hit) - 1;
      u.b = c0 + src;
      u.L = __shfl(L, src);
      u.nq = __shfl(nq, src);
      u.nblk = __shfl(nb, src);
      const int pre = __shfl(inc, src) - u.nblk;
      u.kvh = (x - pre * p.Hkv) / u.nblk;
      u.begin = pre * p.Hkv + u.kvh * u.nblk;
      return u;
    }
    running = __shfl(inc, 63);
  }
  return u;
}

// Flattened index of the first block of unit (b, kvh); also returns the unit's lengths.
__device__ inline Unit unit_of(const AttnParams& p, int b_want, int kvh, int lane) {
  Unit u{b_want, kvh, 0, 0, 0, 0};
  int running = 0;
  for (int c0 = 0; c0 < p.B; c0 += 64) {
    const int b = c0 + lane;
    int L = 0, nq = 0, nb = 0;
    bool bad;
    if (b < p.B) nb = seq_blocks(p, b, L, nq, bad);
    const int inc = running + wave_incl_scan(nb, lane);
    if (b_want >= c0 && b_want < c0 + 64) {
      const int src = b_want - c0;
      u.L = __shfl(L, src);
      u.nq = __shfl(nq, src);
      u.nblk = __shfl(nb, src);
      u.begin = (__shfl(inc, src) - u.nblk) * p.Hkv + kvh * u.nblk;
      return u;
    }
    running = __shfl(inc, 63);
  }
  return u;
}

__device__ inline int blocks_per_wave(int total, int nwaves) { return total > 0 ? (total + nwaves - 1) / nwaves : 1; }

// ---------------------------------------------------------------------------------------
// bf16 streaming kernel
// ---------------------------------------------------------------------------------------
template <int D>
struct KvRegs {
  uint4 k[2 * (D / 32)];
  uint4 v[D / 16];
};

template <int D>
__device__ inline void load_block(KvRegs<D>& r, const uint4* kb, const uint4* vb, int lane) {
#pragma unroll
  for (int i = 0; i < 2 * (D / 32); ++i) r.k[i] = kb[i * 64 + lane];
#pragma unroll
  for (int i = 0; i < D / 16; ++i) r.v[i] = vb[i * 64 + lane];
}

template <int D, int NT>
struct RowState {
  f32x4 acc[NT][D / 16];
  float m[NT];  // running max (log2 units), identical in the 4 lanes that share a query row
  float l[NT];  // this lane's share of the running sum
};

// One 32-token block against all query tiles.  kMasked: the block reaches beyond ctx_len, so
// causal limits and the valid-token bound apply (wave-uniform choice).
template <int D, int NT, bool kMasked>
__device__ inline void block_step(KvRegs<D>& r, const bf16x8 (&qf)[NT][D / 32], RowState<D, NT>& st, int tok0,
                                  int n_valid, const int (&lim)[NT], float scale_log2, int lane) {
  constexpr int KS = D / 32, MT = D / 16;
  const int grp = lane >> 4;
  if (kMasked) {
    // stale cache rows (token >= n_valid) may hold anything, NaN included: zero them in V so
    // that 0 * garbage cannot reach the accumulator.  Word w of a lane holds slots 2w, 2w+1.
    const int tA = tok0 + 4 * grp, tB = tok0 + 16 + 4 * grp;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      uint32_t* wv = (uint32_t*)&r.v[mt];
#pragma unroll
      for (int wd = 0; wd < 4; ++wd) {
        const int t_lo = (wd < 2 ? tA : tB) + 2 * (wd & 1);
        uint32_t keep = 0;
        if (t_lo < n_valid) keep |= 0x0000FFFFu;
        if (t_lo + 1 < n_valid) keep |= 0xFFFF0000u;
        wv[wd] &= keep;
      }
    }
  }
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < KS; ++t) {
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, r.k[t]), qf[nt][t], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, r.k[KS + t]), qf[nt][t], s1, 0, 0, 0);
    }
    float s[8];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      s[j] = s0[j] * scale_log2;
      s[4 + j] = s1[j] * scale_log2;
    }
    if (kMasked) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (tok0 + 4 * grp + j > lim[nt]) s[j] = -INFINITY;
        if (tok0 + 16 + 4 * grp + j > lim[nt]) s[4 + j] = -INFINITY;
      }
    }
    float mx = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(st.m[nt], mx);
    // a row that has seen no visible token yet keeps m = -inf; subtract 0 instead so that
    // exp2(-inf - 0) = 0 and no inf - inf appears
    const float m_use = (kMasked && m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(st.m[nt] - m_use);
    float psum = 0.f;
    bf16x8 pf;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float pj = __builtin_amdgcn_exp2f(s[j] - m_use);
      psum += pj;
      pf[j] = (__bf16)pj;
    }
    st.l[nt] = st.l[nt] * alpha + psum;
    st.m[nt] = m_new;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      f32x4 a = st.acc[nt][mt];
      a[0] *= alpha; a[1] *= alpha; a[2] *= alpha; a[3] *= alpha;
      st.acc[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, r.v[mt]), pf, a, 0, 0, 0);
    }
  }
}

template <int D, int NT>
__device__ inline void block_dispatch(KvRegs<D>& r, const bf16x8 (&qf)[NT][D / 32], RowState<D, NT>& st, int blk,
                                      int L, int n_valid, const int (&lim)[NT], float scale_log2, int lane) {
  const int tok0 = blk * kBlockTokens;
  if (tok0 + kBlockTokens - 1 <= L)  // every token of the block is visible to every query
    block_step<D, NT, false>(r, qf, st, tok0, n_valid, lim, scale_log2, lane);
  else
    block_step<D, NT, true>(r, qf, st, tok0, n_valid, lim, scale_log2, lane);
}

template <int D, int NT>
__global__ __launch_bounds__(256) void verify_attn_bf16(AttnParams p) {
  constexpr int KS = D / 32, MT = D / 16;
  constexpr size_t kBlkVec = (size_t)kBlockTokens * D * 2 / 16;  // uint4 per block
  const int lane = threadIdx.x & 63;
  const int w = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int col = lane & 15, grp = lane >> 4;

  const int total = total_seq_blocks(p, lane, w == 0) * p.Hkv;
  const int c = blocks_per_wave(total, p.nwaves);
  int x = w * c;
  const int x_end = min(total, x + c);

  while (x < x_end) {
    const Unit u = locate(p, x, lane);
    const int blk0 = x - u.begin;
    const int nseg = min(x_end, u.begin + u.nblk) - x;  // blocks of this unit that are ours
    const int rows = u.nq * p.g;                         // valid query rows of the unit
    const int n_valid = u.L + u.nq;

    // query fragments (B operand): lane (col, grp) holds row 16 nt + col, elements 32 t + 8 grp ..+7
    bf16x8 qf[NT][KS];
    int lim[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int rrow = nt * 16 + col;
      const bool ok = rrow < rows;
      const int i = ok ? rrow / p.g : 0, hg = ok ? rrow % p.g : 0;
      lim[nt] = u.L + i;
      const uint4* qrow = (const uint4*)((const uint16_t*)p.Q + (((size_t)u.b * p.kmax + i) * p.Hq + u.kvh * p.g + hg) * D);
#pragma unroll
      for (int t = 0; t < KS; ++t) {
        uint4 qv = make_uint4(0, 0, 0, 0);
        if (ok) qv = qrow[t * 4 + grp];
        qf[nt][t] = __builtin_bit_cast(bf16x8, qv);
      }
    }

    RowState<D, NT> st;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      st.m[nt] = -INFINITY;
      st.l[nt] = 0.f;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) st.acc[nt][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    const size_t unit_vec = ((size_t)u.b * p.Hkv + u.kvh) * p.nblk_cap * kBlkVec;
    const uint4* kbase = (const uint4*)p.Kc + unit_vec;
    const uint4* vbase = (const uint4*)p.Vc + unit_vec;

    KvRegs<D> ra, rb;
    load_block<D>(ra, kbase + (size_t)blk0 * kBlkVec, vbase + (size_t)blk0 * kBlkVec, lane);
    for (int s = 0; s < nseg; s += 2) {
      const int blk = blk0 + s;
      if (s + 1 < nseg) load_block<D>(rb, kbase + (size_t)(blk + 1) * kBlkVec, vbase + (size_t)(blk + 1) * kBlkVec, lane);
      block_dispatch<D, NT>(ra, qf, st, blk, u.L, n_valid, lim, p.scale_log2, lane);
      if (s + 1 < nseg) {
        if (s + 2 < nseg) load_block<D>(ra, kbase + (size_t)(blk + 2) * kBlkVec, vbase + (size_t)(blk + 2) * kBlkVec, lane);
        block_dispatch<D, NT>(rb, qf, st, blk + 1, u.L, n_valid, lim, p.scale_log2, lane);
      }
    }

    // partial of this (wave, unit) pair; slot ids w + unit are unique because both grow
    // monotonically along the flattened list
    const size_t slot = (size_t)w + (size_t)u.b * p.Hkv + u.kvh;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      float l = st.l[nt];
      l += __shfl_xor(l, 16);
      l += __shfl_xor(l, 32);
      const int rrow = nt * 16 + col;
      if (rrow < rows) {
        float* dst = p.part_acc + (slot * p.rows_max + rrow) * D + 4 * grp;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) *(f32x4*)(dst + 16 * mt) = st.acc[nt][mt];
        if (grp == 0) *(float2*)(p.part_ml + (slot * p.rows_max + rrow) * 2) = make_float2(st.m[nt], l);
      }
    }
    x += nseg;
  }
}

// ---------------------------------------------------------------------------------------
// fp32 kernel: same schedule and partial format, plain fp32 FMA arithmetic (no matrix cores;
// probabilities stay fp32).  Cache is token-major [B][Hkv][Lcap][D].  A wavefront handles up
// to 8 query rows at a time: lanes own tokens for the scores and head elements for P*V.
// ---------------------------------------------------------------------------------------
constexpr int kRowChunk = 8;

__global__ __launch_bounds__(256) void verify_attn_fp32(AttnParams p) {
  const int lane = threadIdx.x & 63;
  const int w = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int D = p.D;
  const int nd = (D + 63) / 64;  // head elements per lane (<= 4)

  const int total = total_seq_blocks(p, lane, w == 0) * p.Hkv;
  const int c = blocks_per_wave(total, p.nwaves);
  int x = w * c;
  const int x_end = min(total, x + c);

  while (x < x_end) {
    const Unit u = locate(p, x, lane);
    const int blk0 = x - u.begin;
    const int nseg = min(x_end, u.begin + u.nblk) - x;
    const int rows = u.nq * p.g;
    const int n_valid = u.L + u.nq;
    const int tok_lo = blk0 * kBlockTokens;
    const int tok_hi = min(n_valid, (blk0 + nseg) * kBlockTokens);
    const float* kbase = (const float*)p.Kc + ((size_t)u.b * p.Hkv + u.kvh) * p.Lcap * D;
    const float* vbase = (const float*)p.Vc + ((size_t)u.b * p.Hkv + u.kvh) * p.Lcap * D;
    const size_t slot = (size_t)w + (size_t)u.b * p.Hkv + u.kvh;

    for (int r0 = 0; r0 < rows; r0 += kRowChunk) {
      const int nr = min(kRowChunk, rows - r0);
      float m[kRowChunk], l[kRowChunk], acc[kRowChunk][4];
#pragma unroll
      for (int r = 0; r < kRowChunk; ++r) {
        m[r] = -INFINITY;
        l[r] = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k) acc[r][k] = 0.f;
      }
      for (int t0 = tok_lo; t0 < tok_hi; t0 += 64) {
        const int tok = t0 + lane;
        const bool tok_ok = tok < tok_hi;
        const float* krow = kbase + (size_t)(tok_ok ? tok : tok_lo) * D;
        float pr[kRowChunk];
#pragma unroll
        for (int r = 0; r < kRowChunk; ++r) {
          pr[r] = 0.f;
          if (r < nr) {
            const int rrow = r0 + r, i = rrow / p.g, hg = rrow % p.g;
            const float* qrow = (const float*)p.Q + (((size_t)u.b * p.kmax + i) * p.Hq + u.kvh * p.g + hg) * D;
            float dot = 0.f;
            for (int d = 0; d < D; d += 4) {
              const float4 kv = *(const float4*)(krow + d);
              const float4 qv = *(const float4*)(qrow + d);
              dot = fmaf(kv.x, qv.x, dot);
              dot = fmaf(kv.y, qv.y, dot);
              dot = fmaf(kv.z, qv.z, dot);
              dot = fmaf(kv.w, qv.w, dot);
            }
            float s = (tok_ok && tok <= u.L + i) ? dot * p.scale_log2 : -INFINITY;
            float mx = s;
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
            const float m_new = fmaxf(m[r], mx);
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = exp2f(m[r] - m_use);
            const float pj = exp2f(s - m_use);
            float ps = pj;
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) ps += __shfl_xor(ps, o);
            l[r] = l[r] * alpha + ps;
            m[r] = m_new;
#pragma unroll
            for (int k = 0; k < 4; ++k) acc[r][k] *= alpha;
            pr[r] = pj;
          }
        }
        // P * V: lanes own head elements lane + 64 k; the probability of token t0 + jj is
        // broadcast from lane jj
        const int ntile = min(64, tok_hi - t0);
        for (int jj = 0; jj < ntile; ++jj) {
          const float* vrow = vbase + (size_t)(t0 + jj) * D;
          float vv[4];
#pragma unroll
          for (int k = 0; k < 4; ++k) vv[k] = (k < nd && lane + 64 * k < D) ? vrow[lane + 64 * k] : 0.f;
#pragma unroll
          for (int r = 0; r < kRowChunk; ++r) {
            const float pj = __shfl(pr[r], jj);
#pragma unroll
            for (int k = 0; k < 4; ++k) acc[r][k] = fmaf(pj, vv[k], acc[r][k]);
          }
        }
      }
#pragma unroll
      for (int r = 0; r < kRowChunk; ++r) {
        if (r < nr) {
          const int rrow = r0 + r;
          float* dst = p.part_acc + (slot * p.rows_max + rrow) * D;
#pragma unroll
          for (int k = 0; k < 4; ++k)
            if (k < nd && lane + 64 * k < D) dst[lane + 64 * k] = acc[r][k];
          if (lane == 0) *(float2*)(p.part_ml + (slot * p.rows_max + rrow) * 2) = make_float2(m[r], l[r]);
        }
      }
    }
    x += nseg;
  }
}

// ---------------------------------------------------------------------------------------
// Split-context reduction: one wavefront per output row (b, i, hq).
//   M = max_s m_s ;  l = sum_s l_s 2^(m_s - M) ;  O = sum_s acc_s 2^(m_s - M) / l
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void combine_partials(AttnParams p) {
  const int lane = threadIdx.x & 63;
  const long row_id = (long)blockIdx.x * 4 + (threadIdx.x >> 6);  // over [B][kmax][Hq]
  if (row_id >= (long)p.B * p.kmax * p.Hq) return;
  const int hq = (int)(row_id % p.Hq);
  const int i = (int)((row_id / p.Hq) % p.kmax);
  const int b = (int)(row_id / ((long)p.Hq * p.kmax));
  const int D = p.D;
  float* out = p.O + (size_t)row_id * D;
  const int kvh = hq / p.g, hg = hq % p.g;
  const Unit u = unit_of(p, b, kvh, lane);
  if (i >= u.nq) {
    for (int d = lane; d < D; d += 64) out[d] = 0.f;
    if (p.lse && lane == 0) p.lse[row_id] = 0.f;
    return;
  }
  const int total = total_seq_blocks(p, lane, false) * p.Hkv;
  const int c = blocks_per_wave(total, p.nwaves);
  const int w_lo = u.begin / c, w_hi = (u.begin + u.nblk - 1) / c;
  const int rrow = i * p.g + hg;
  const size_t unit_id = (size_t)b * p.Hkv + kvh;

  float M = -INFINITY;
  for (int w = w_lo + lane; w <= w_hi; w += 64)
    M = fmaxf(M, p.part_ml[((w + unit_id) * p.rows_max + rrow) * 2]);
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) M = fmaxf(M, __shfl_xor(M, o));

  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  float l = 0.f;
  for (int w = w_lo; w <= w_hi; ++w) {
    const size_t pr = (w + unit_id) * p.rows_max + rrow;
    const float2 ml = *(const float2*)(p.part_ml + pr * 2);
    const float wgt = exp2f(ml.x - M);  // a partial without visible tokens has m = -inf, weight 0
    l = fmaf(ml.y, wgt, l);
    const float* src = p.part_acc + pr * D;
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (lane + 64 * k < D) acc[k] = fmaf(src[lane + 64 * k], wgt, acc[k]);
  }
  const float inv = 1.f / l;
#pragma unroll
  for (int k = 0; k < 4; ++k)
    if (lane + 64 * k < D) out[lane + 64 * k] = acc[k] * inv;
  if (p.lse && lane == 0) p.lse[row_id] = (M + log2f(l)) * 0.6931471805599453f;
}

static size_t workspace_bytes(const bass_attn_desc* d) {
  const size_t slots = (size_t)kMaxWaves + (size_t)d->B * d->Hkv;
  const size_t rows = (size_t)d->kmax * (d->Hq / d->Hkv);
  return slots * rows * ((size_t)d->D + 2) * sizeof(float);
}

}  // namespace bass

extern "C" int bass_set_attention_waves(int waves) {
  bass::g_attention_waves = waves > 0 ? waves : 0;
  return bass::attention_waves();
}

extern "C" size_t bass_verify_attention_workspace_bytes(const bass_attn_desc* d) {
  if (bass::check_desc(d) != BASS_OK) return 0;
  return bass::workspace_bytes(d);
}

extern "C" int bass_verify_attention(const bass_attn_desc* d, const void* Q, const void* Kcache, const void* Vcache,
                                     const int32_t* ctx_len, const int32_t* draft_len, float* O, float* lse,
                                     void* workspace, size_t workspace_bytes, int32_t* dev_status, void* stream) {
  using namespace bass;
  int rc = check_desc(d);
  if (rc != BASS_OK) return rc;
  if (!Q || !Kcache || !Vcache || !ctx_len || !draft_len || !O || !workspace) return BASS_ERR_INVALID_ARG;
  if (((uintptr_t)workspace & 15) != 0) return BASS_ERR_INVALID_ARG;
  const int g = d->Hq / d->Hkv;
  const int rows_max = d->kmax * g;
  if (d->dtype == BASS_DTYPE_BF16 && rows_max > 64) return BASS_ERR_UNSUPPORTED;
  if (workspace_bytes < bass::workspace_bytes(d)) return BASS_ERR_WORKSPACE_TOO_SMALL;

  AttnParams p;
  p.B = d->B; p.kmax = d->kmax; p.Hq = d->Hq; p.Hkv = d->Hkv; p.D = d->D; p.Lcap = d->Lcap;
  p.nblk_cap = num_blocks(d->Lcap); p.g = g; p.rows_max = rows_max; p.nwaves = attention_waves();
  p.scale_log2 = d->scale * 1.4426950408889634f;
  p.Q = Q; p.Kc = Kcache; p.Vc = Vcache; p.ctx_len = ctx_len; p.draft_len = draft_len;
  p.O = O; p.lse = lse; p.status = dev_status;
  const size_t slots = (size_t)kMaxWaves + (size_t)d->B * d->Hkv;
  p.part_acc = (float*)workspace;
  p.part_ml = p.part_acc + slots * rows_max * d->D;

  hipStream_t s = (hipStream_t)stream;
  const dim3 grid(p.nwaves / 4), block(256);
  if (d->dtype == BASS_DTYPE_FP32) {
    hipLaunchKernelGGL(verify_attn_fp32, grid, block, 0, s, p);
  } else {
    const int nt = (rows_max + 15) / 16;
#define BASS_LAUNCH(DD, NN) hipLaunchKernelGGL((verify_attn_bf16<DD, NN>), grid, block, 0, s, p)
    if (d->D == 128) {
      if (nt == 1) BASS_LAUNCH(128, 1); else if (nt == 2) BASS_LAUNCH(128, 2);
      else if (nt == 3) BASS_LAUNCH(128, 3); else BASS_LAUNCH(128, 4);
    } else {
      if (nt == 1) BASS_LAUNCH(64, 1); else if (nt == 2) BASS_LAUNCH(64, 2);
      else if (nt == 3) BASS_LAUNCH(64, 3); else BASS_LAUNCH(64, 4);
    }
#undef BASS_LAUNCH
  }
  if (launch_status() != BASS_OK) return BASS_ERR_HIP;
  const long out_rows = (long)d->B * d->kmax * d->Hq;
  hipLaunchKernelGGL(combine_partials, dim3((unsigned)((out_rows + 3) / 4)), dim3(256), 0, s, p);
  return launch_status();
}
