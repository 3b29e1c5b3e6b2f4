// Ragged verify attention of libbass: bass_verify_attention, bass_append_verify_attention (the
// step's K/V rows appended inside the same launch), bass_verify_attention_pad / _split (the paper's
// BASS-PAD and BASS-SPLIT as launch variants), for bf16, INT8 and fp32 caches.
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
// unnormalised output).  The wavefront that delivers the LAST partial of a unit (found with
// one atomic counter per unit) merges the unit's partials -- the split-context reduction --
// and writes O and the log-sum-exp, so the whole call is a single launch.  (With more than one
// 16-row query tile per kv head -- grouped-query attention -- the merge is a second, chip-wide
// launch: reduce_partials.)
//
// Matrix-core mapping (v_mfma_f32_16x16x32_bf16, wave64).  Tokens sit on the M side:
//   S^T[16 tokens x 16 query rows] = K[16 x D] * Q^T[D x 16]          (D/32 MFMAs per tile)
//   O^T[D x 16 query rows]        += V^T[D x 32 tokens] * P^T[32 x 16] (D/16 MFMAs per block)
// The result layout of the first (a lane owns 4 consecutive tokens of one query row) is,
// for two 16-token tiles, exactly the operand layout of the second once the V block is
// stored in that token order, so P goes from accumulator to operand with a bf16 pack only.
// Query rows of one kv head are (draft i, head-in-group) pairs, up to 64 rows = 4 tiles.
#include <algorithm>
#include <atomic>
#include <mutex>
#include <type_traits>

#include "bass_common.h"

namespace bass {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;

// Tuning knob of bass_set_attention_waves: process wide, read once per call.
static std::atomic<int> g_attention_waves{0};  // 0 = defaults
int attention_waves_setting() { return g_attention_waves.load(std::memory_order_relaxed); }

struct AttnParams {
  int B, kmax, Hq, Hkv, D, Lcap, nblk_cap, g, rows_max, nwaves;
  unsigned g_magic;  // ceil(2^20 / g) if g <= 64 and rows_max <= 2048 (then r / g == (r * g_magic) >> 20 for every row r), else 0
  int wpw;  // wavefronts per workgroup of the attention launch (nwaves is a multiple)
  int nshares;  // stretches the block list is cut into: one per wavefront, or one per workgroup (tile kernel)
  int fused_reduce;  // 1: the last-arriving wavefront merges a unit's partials; 0: a second launch does
  float scale_log2;  // scale * log2(e): scores are kept in the log2 domain
  const void* Q;
  const void* Kc;
  const void* Vc;
  const void* Knew;  // [B,kmax,Hkv,D] rows of this step to append first, or null
  const void* Vnew;
  // the step's plan (attn_plan.h): header, one record per share, the further segments, per-sequence
  // query counts, per-unit contributors
  const PlanHeader* plan;
  int32_t signature;  // plan_signature() of the plan this launch expects
  const ShareRecord* records;
  const Segment* overflow;
  const int32_t* seq_L;
  const int32_t* seq_nq;
  const int32_t* unit_owners;
  float* O;
  float* lse;
  float* part_acc;  // [slots][rows_max][D]
  float* part_ml;   // [slots][rows_max][2]  (running max in log2 units, running sum)
  int32_t* counters;  // [B*Hkv] partials delivered per unit; zero between calls
  int32_t* status;
};

// Query row r of a kv head is query token r / g, head r % g of the group.  The division by the run-time
// group size is a multiplication by a constant the host prepared (a generic integer division is some 35
// instructions, and these sit on the way out).
__device__ inline int row_token(const AttnParams& p, int r) {
  return p.g_magic ? (int)(((unsigned)r * p.g_magic) >> 20) : r / p.g;
}

__device__ inline int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// ---------------------------------------------------------------------------------------
// The share of a wavefront (or workgroup), read from the step's plan.
// ---------------------------------------------------------------------------------------
// A segment whose address is the same in every lane, as wave-uniform values.
__device__ inline Segment load_segment(const Segment* src) {
  const i32x4 a = *(const i32x4*)src, b = *((const i32x4*)src + 1);
  Segment g;
  g.b = uniform(a[0]); g.kvh = uniform(a[1]); g.L = uniform(a[2]); g.nq = uniform(a[3]);
  g.first = uniform(b[0]); g.n = uniform(b[1]); g.owners = uniform(b[2]); g.flags = uniform(b[3]);
  return g;
}

// Segment si >= 1 of a share
__device__ inline const Segment* later_segment_address(const AttnParams& p, const ShareRecord* rec, int overflow, int si) {
  return si == 1 ? &rec->seg[1] : p.overflow + overflow + (si - 2);
}
__device__ inline Segment later_segment(const AttnParams& p, const ShareRecord* rec, int overflow, int si) {
  return load_segment(later_segment_address(p, rec, overflow, si));
}

// A segment requested early and used late (its address is the same in every lane): the request travels while
// the wavefront streams, so that going on to the next units of a long share costs no round trip.
struct SegmentInFlight {
  i32x4 a, b;
};
__device__ inline SegmentInFlight request_segment(const Segment* src) {
  return SegmentInFlight{*(const i32x4*)src, *((const i32x4*)src + 1)};
}
__device__ inline Segment arrived_segment(const SegmentInFlight& f) {
  Segment g;
  g.b = uniform(f.a[0]); g.kvh = uniform(f.a[1]); g.L = uniform(f.a[2]); g.nq = uniform(f.a[3]);
  g.first = uniform(f.b[0]); g.n = uniform(f.b[1]); g.owners = uniform(f.b[2]); g.flags = uniform(f.b[3]);
  return g;
}

// The plan must have been made for this launch: same batch shape, same number of shares, and for a launch
// that appends or does not; every record carries a signature of these.  Anything else (also a buffer that
// holds no plan) stops the wavefront before it stores anything, with BASS_STATUS_PLAN_MISMATCH.
__device__ inline bool record_matches(const AttnParams& p, const ShareRecord* rec) {
  int sig = uniform(rec->signature);
  asm volatile("" : "+s"(sig));  // keeps the comparison (and with it the wait for the record) where it is written
  return sig == p.signature;
}

__device__ inline void report_mismatch(const AttnParams& p, bool first_lane) {
  if (first_lane && p.status) atomicOr(p.status, BASS_STATUS_PLAN_MISMATCH);
}

struct Unit {
  int b, kvh, L, nq;
};
__device__ inline Unit unit_of(const Segment& g) { return Unit{g.b, g.kvh, g.L, g.nq}; }

// Partials travel between wavefronts that may sit on different XCDs, whose L2 caches are not
// coherent with each other for ordinary accesses.  Instead of device-scope fences (which write
// back and invalidate a whole L2 and cost far more than the data is worth), every partial is
// written and read with device-scope relaxed atomic 64-bit accesses, which go through to the
// device-coherent level; "wait for my stores, then bump the counter" orders them.
__device__ inline void store_dev(float* dst, float a, float b) {
  unsigned long long v = ((unsigned long long)__float_as_uint(b) << 32) | __float_as_uint(a);
  __hip_atomic_store((unsigned long long*)dst, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// 128-bit variants through raw buffer accesses with the device-scope cache policy (sc1); the
// buffer descriptor also bounds the access: offsets beyond `bytes` read zero / are dropped.
constexpr int kAuxDeviceScope = 16;  // sc1

// base and bytes are wave-uniform by construction; saying so keeps the descriptor in scalar
// registers (otherwise every access is wrapped in a loop over distinct descriptors).
__device__ inline __amdgpu_buffer_rsrc_t dev_buffer(const float* base, unsigned bytes) {
  const unsigned long long a = (unsigned long long)base;
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)a);
  const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32));
  float* ub = (float*)(((unsigned long long)hi << 32) | lo);
  return __builtin_amdgcn_make_buffer_rsrc(ub, 0, (int)__builtin_amdgcn_readfirstlane(bytes), 0x00020000);
}

__device__ inline void store_dev4(__amdgpu_buffer_rsrc_t rs, unsigned byte_off, f32x4 v) {
  __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), rs, (int)byte_off, 0, kAuxDeviceScope);
}

__device__ inline f32x4 load_dev4(__amdgpu_buffer_rsrc_t rs, unsigned byte_off) {
  return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, (int)byte_off, 0, kAuxDeviceScope));
}

__device__ inline void store_dev1(float* dst, float a) {
  __hip_atomic_store((unsigned*)dst, __float_as_uint(a), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ inline float2 load_dev(const float* src) {
  const unsigned long long v = __hip_atomic_load((const unsigned long long*)src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__uint_as_float((unsigned)v), __uint_as_float((unsigned)(v >> 32)));
}

// ---------------------------------------------------------------------------------------
// Split-context reduction, done by the wavefront that completes a unit:
//   M = max_s m_s ;  l = sum_s l_s 2^(m_s - M) ;  O = sum_s acc_s 2^(m_s - M) / l
// over the partials of wavefronts w_lo..w_hi, then zeros for the unit's unused query slots.
// ---------------------------------------------------------------------------------------
// DC: the head size when it is known at compile time (the divisions below then cost nothing; this code
// runs before a wavefront's first K/V load), 0: read it from the descriptor.
template <int DC>
__device__ inline void zero_rows(const AttnParams& p, int b, int kvh, int row_from, int lane, int row_to = 1 << 30) {
  const int D = DC ? DC : p.D, lpr = D / 4, rpi = 64 / lpr;
  const int rows_all = min(p.kmax * p.g, row_to);
  for (int r0 = row_from; r0 < rows_all; r0 += rpi) {
    const int r = r0 + lane / lpr;
    if (lane < rpi * lpr && r < rows_all) {
      const int i = row_token(p, r), hg = r - i * p.g;
      const size_t orow = ((size_t)b * p.kmax + i) * p.Hq + kvh * p.g + hg;
      *(float4*)(p.O + orow * D + (lane % lpr) * 4) = make_float4(0.f, 0.f, 0.f, 0.f);
      if (p.lse && lane % lpr == 0) p.lse[orow] = 0.f;
    }
  }
}

__device__ inline float group16_max(float v) {
#pragma unroll
  for (int o = 8; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}

__device__ inline float group16_sum(float v) {
#pragma unroll
  for (int o = 8; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// Split-context reduction of a unit, four query rows per sweep: 16 lanes per row, each lane owning
// KC float4 chunks of its row.  Two phases, so that the requests of two sweeps can be in flight
// together:
//   issue : requests, for the first 8 partials, the row's (max, sum) pairs (every lane of a row
//           asks for all of them, so no cross-lane traffic is needed later) and the lane's
//           output chunks -- one round trip to memory in the common case;
//   finish: weights 2^(m_s - M) / L and the weighted sum, all lane-local; units with more than 8
//           partials (work spread very thin) continue one partial at a time; writes O and lse.
// Device-scope requests cost a trip to memory each: partials that do not exist are skipped by
// wave-uniform branches, and idle row slots get an offset beyond the buffer descriptor's size,
// which the hardware answers with zeros without touching memory.
template <int KC>
struct CombineRegs {
  bool rok;
  int r;
  float2 ml[8];
  f32x4 a[8][KC];
};

struct CombineJob {
  Unit u;
  int w_lo, w_hi;
};

// 2 GiB: larger than any descriptor, and adding a partial's offset, which the host keeps below
// 2 GiB, cannot wrap around.
constexpr unsigned kNoSuchOffset = 0x80000000u;

typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

__device__ inline float2 load_dev2(__amdgpu_buffer_rsrc_t rs, unsigned byte_off) {
  const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rs, (int)byte_off, 0, kAuxDeviceScope);
  return make_float2(__uint_as_float(v.x), __uint_as_float(v.y));
}

// A sweep merges 64 / LPR rows: LPR lanes share a row, lane dl of them holds the 16-byte chunks dl + LPR k
// (k < KC) of it.
template <int KC, int DC, int LPR = 16>
__device__ inline void combine_issue(const AttnParams& p, const CombineJob& job, int r0, int lane, CombineRegs<KC>& c) {
  const Unit& u = job.u;
  const int D = DC > 0 ? DC : p.D;
  const int rr = lane / LPR, dl = lane % LPR;
  const int rows = uniform(u.nq * p.g);
  const int S8 = min(uniform(job.w_hi - job.w_lo + 1), 8);
  const size_t slot0 = (size_t)uniform(job.w_lo + u.b * p.Hkv + u.kvh);
  const unsigned slot_bytes = (unsigned)p.rows_max * D * 4, ml_bytes = (unsigned)p.rows_max * 8;
  const __amdgpu_buffer_rsrc_t rs = dev_buffer(p.part_acc + slot0 * p.rows_max * D, (unsigned)S8 * slot_bytes);
  const __amdgpu_buffer_rsrc_t rs_ml = dev_buffer(p.part_ml + slot0 * p.rows_max * 2, (unsigned)S8 * ml_bytes);
  c.rok = r0 + rr < rows;
  c.r = r0 + rr;
  const unsigned ml_off = c.rok ? (unsigned)c.r * 8 : kNoSuchOffset;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    if (j >= S8) break;  // wave-uniform: no such partial (combine_finish never looks at it)
    c.ml[j] = load_dev2(rs_ml, (unsigned)j * ml_bytes + ml_off);
#pragma unroll
    for (int k = 0; k < KC; ++k) {
      const int d = 4 * (dl + LPR * k);
      const unsigned row_off = (c.rok && d < D) ? (unsigned)(c.r * D + d) * 4 : kNoSuchOffset;
      c.a[j][k] = load_dev4(rs, (unsigned)j * slot_bytes + row_off);
    }
  }
}

constexpr int kMore = 2;  // partials beyond the eighth are fetched this many at a time (registers: the streaming kernel is full)

template <int KC, int DC, int LPR = 16>
__device__ inline void combine_finish(const AttnParams& p, const CombineJob& job, int lane, const CombineRegs<KC>& c) {
  const Unit& u = job.u;
  const int D = DC > 0 ? DC : p.D;
  const int dl = lane % LPR;
  const int S = uniform(job.w_hi - job.w_lo + 1);
  const size_t slot0 = (size_t)uniform(job.w_lo + u.b * p.Hkv + u.kvh);
  const unsigned slot_bytes = (unsigned)p.rows_max * D * 4, ml_bytes = (unsigned)p.rows_max * 8;
  const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
  const int r = c.r;
  // M = max_s m_s, L = sum_s l_s 2^(m_s - M).  A valid row has at least one partial with a
  // visible token (token 0), so M ends finite; a partial that saw none has m = -inf, weight 0.
  // (Idle row slots were answered with zeros.)
  float M = -INFINITY;
#pragma unroll
  for (int j = 0; j < 8; ++j)
    if (j < S) M = fmaxf(M, c.ml[j].x);  // wave-uniform guards: partials beyond S were never requested
  const unsigned row8 = c.rok ? (unsigned)r * 8 : kNoSuchOffset;
  if (S > 8) {  // further partials, eight per round trip (a load per iteration would be a round trip each)
    const __amdgpu_buffer_rsrc_t rs_ml = dev_buffer(p.part_ml + slot0 * p.rows_max * 2, (unsigned)S * ml_bytes);
#pragma unroll 1
    for (int j0 = 8; j0 < S; j0 += 8) {
      float2 t[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) t[i] = load_dev2(rs_ml, j0 + i < S ? (unsigned)(j0 + i) * ml_bytes + row8 : kNoSuchOffset);
#pragma unroll
      for (int i = 0; i < 8; ++i) M = fmaxf(M, j0 + i < S ? t[i].x : -INFINITY);
    }
  }
  const float Mf = (M == -INFINITY) ? 0.f : M;  // idle row slots only
  float L = 0.f;
  f32x4 acc[KC];
#pragma unroll
  for (int k = 0; k < KC; ++k) acc[k] = zero4;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    if (j < S) {
      const float wgt = __builtin_amdgcn_exp2f(c.ml[j].x - Mf);
      L = fmaf(c.ml[j].y, wgt, L);
#pragma unroll
      for (int k = 0; k < KC; ++k) acc[k] += c.a[j][k] * wgt;
    }
  }
  if (S > 8) {  // further partials, kMore per round trip: all loads of a round are issued before the first use
    const __amdgpu_buffer_rsrc_t rs = dev_buffer(p.part_acc + slot0 * p.rows_max * D, (unsigned)S * slot_bytes);
    const __amdgpu_buffer_rsrc_t rs_ml = dev_buffer(p.part_ml + slot0 * p.rows_max * 2, (unsigned)S * ml_bytes);
    unsigned row_off[KC];
#pragma unroll
    for (int k = 0; k < KC; ++k) {
      const int d = 4 * (dl + LPR * k);
      row_off[k] = (c.rok && d < D) ? (unsigned)(r * D + d) * 4 : kNoSuchOffset;
    }
#pragma unroll 1
    for (int j0 = 8; j0 < S; j0 += kMore) {
      float2 ml[kMore];
      f32x4 a[kMore][KC];
#pragma unroll
      for (int i = 0; i < kMore; ++i) {
        const bool have = j0 + i < S;  // wave-uniform; a missing partial is requested out of range (zeros, no memory access)
        ml[i] = load_dev2(rs_ml, have ? (unsigned)(j0 + i) * ml_bytes + row8 : kNoSuchOffset);
#pragma unroll
        for (int k = 0; k < KC; ++k) a[i][k] = load_dev4(rs, have ? (unsigned)(j0 + i) * slot_bytes + row_off[k] : kNoSuchOffset);
      }
#pragma unroll
      for (int i = 0; i < kMore; ++i) {
        const float w = j0 + i < S ? __builtin_amdgcn_exp2f(ml[i].x - Mf) : 0.f;
        L = fmaf(ml[i].y, w, L);
#pragma unroll
        for (int k = 0; k < KC; ++k) acc[k] += a[i][k] * w;
      }
    }
  }
  if (c.rok) {
    const float invL = __builtin_amdgcn_rcpf(L);  // 1 ulp: far inside both tolerances, and a fraction of the instructions of a division
    const int i = row_token(p, r), hg = r - i * p.g;
    const size_t orow = ((size_t)u.b * p.kmax + i) * p.Hq + u.kvh * p.g + hg;
#pragma unroll
    for (int k = 0; k < KC; ++k) {
      const int d = 4 * (dl + LPR * k);
      if (d < D) *(f32x4*)(p.O + orow * D + d) = acc[k] * invL;
    }
    if (p.lse && dl == 0) p.lse[orow] = (M + __builtin_amdgcn_logf(L)) * 0.6931471805599453f;
  }
}

// Reduction of the one or two units this wavefront completed.  The sweeps of both jobs are laid end to
// end and handled two at a time, so that two sweeps share one round trip.  With a compile-time head size
// a sweep takes 8 rows (8 lanes per row): a wavefront's merge is bound by its own instruction stream, and
// the kv heads of this path have at most 16 query rows, mostly 8 or fewer -- one sweep per unit.
template <int DC>
__device__ inline void combine_jobs(const AttnParams& p, const CombineJob& ja, bool do_a, const CombineJob& jb, bool do_b,
                                    int lane) {
  constexpr bool kOverlap = DC > 0;  // the run-time-D (fp32) variant has too many chunk registers for two sweeps
  constexpr int LPR = DC > 0 ? 8 : 16, RPS = 64 / LPR;  // lanes per row, rows per sweep
  constexpr int KC = DC > 0 ? DC / 4 / LPR : 4;         // 16-byte chunks per lane (fp32: head sizes up to 256)
  const CombineJob& j0 = do_a ? ja : jb;  // first (or only) job
  const bool two = do_a && do_b;
  const int n0 = (j0.u.nq * p.g + RPS - 1) / RPS;
  const int n1 = two ? (jb.u.nq * p.g + RPS - 1) / RPS : 0;
#pragma unroll 1
  for (int t = 0; t < n0 + n1; t += (kOverlap ? 2 : 1)) {
    const bool has_y = kOverlap && t + 1 < n0 + n1;
    const CombineJob jx = (t < n0) ? j0 : jb;
    const int rx = (t < n0) ? RPS * t : RPS * (t - n0);
    const CombineJob jy = (t + 1 < n0) ? j0 : jb;
    const int ry = (t + 1 < n0) ? RPS * (t + 1) : RPS * (t + 1 - n0);
    CombineRegs<KC> cx;
    combine_issue<KC, DC, LPR>(p, jx, rx, lane, cx);
    if constexpr (kOverlap) {
      CombineRegs<KC> cy;
      if (has_y) combine_issue<KC, DC, LPR>(p, jy, ry, lane, cy);
      combine_finish<KC, DC, LPR>(p, jx, lane, cx);
      if (has_y) combine_finish<KC, DC, LPR>(p, jy, lane, cy);
    } else {
      combine_finish<KC, DC, LPR>(p, jx, lane, cx);
    }
  }
}

// All of this wavefront's partial stores have reached the device-coherent level once their
// acknowledgements are back (the sc1 stores are written through; the vector-memory counter of this
// wavefront falls to zero only when every one of them has been acknowledged); only then may its
// arrival be counted.  The wait is spelled out: a workgroup-scope fence is lowered without it.
__device__ inline void partial_stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Counts this wavefront's arrival at one or two units (after partial_stores_done).  A job's
// `last` result is true if this wavefront delivered the unit's last partial: it then owns the
// reduction over wavefronts w_lo..w_hi.  Both counters are bumped before either result is awaited.
__device__ inline CombineJob job_of(const Segment& g) { return CombineJob{unit_of(g), seg_w_lo(g), seg_w_hi(g)}; }

__device__ inline int32_t* arrival_counter(const AttnParams& p, CombineJob& j, int& nparts) {
  nparts = j.w_hi - j.w_lo + 1;
  return p.counters + (size_t)j.u.b * p.Hkv + j.u.kvh;
}

__device__ inline void arrive(const AttnParams& p, int lane, CombineJob& ja, bool& last_a, bool has_b, CombineJob& jb,
                              bool& last_b) {
  int na, nb = 1, old_a = 0, old_b = 0;
  int32_t* ctr_a = arrival_counter(p, ja, na);
  int32_t* ctr_b = ctr_a;
  if (has_b) ctr_b = arrival_counter(p, jb, nb);
  if (na > 1 && lane == 0) old_a = __hip_atomic_fetch_add(ctr_a, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (has_b && nb > 1 && lane == 0) old_b = __hip_atomic_fetch_add(ctr_b, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  last_a = na == 1 || __builtin_amdgcn_readfirstlane(old_a) == na - 1;
  last_b = has_b && (nb == 1 || __builtin_amdgcn_readfirstlane(old_b) == nb - 1);
  // every contributor has arrived: leave the counter clean for the next call
  if (last_a && na > 1 && lane == 0) __hip_atomic_store(ctr_a, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (last_b && nb > 1 && lane == 0) __hip_atomic_store(ctr_b, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// Query slots beyond draft_len (all of them for an inactive sequence) are zero in O and lse.
// Wavefront w clears them for the units w, w + nw, ...
// kInactiveOnly: only the units of sequences without query tokens (they have no blocks, hence no
// wavefront of their own); the caller then clears the unused rows of the other units elsewhere (the
// one-tile matrix-core kernel: by the wavefront that holds the unit's last block).
template <int DC, bool kInactiveOnly = false>
__device__ inline void zero_unused_rows(const AttnParams& p, int w, int nw, int lane) {
  for (int unit = w; unit < p.B * p.Hkv; unit += nw) {
    const int b = unit / p.Hkv;
    const int nq = uniform(p.seq_nq[b]);
    if (!kInactiveOnly || nq == 0) zero_rows<DC>(p, b, unit - b * p.Hkv, nq * p.g, lane);
  }
}

// ---------------------------------------------------------------------------------------
// bf16 streaming kernel
// ---------------------------------------------------------------------------------------
template <int D>
struct KvRegs {
  uint4 k[2 * (D / 32)];
  uint4 v[D / 16];
};

// kb, vb already include the lane offset
template <int D>
__device__ inline void load_block(KvRegs<D>& r, const uint4* kb, const uint4* vb) {
  // every K/V byte is read once per launch: non-temporal loads keep the stream from displacing
  // other data in the caches (measured: 10 % shorter launches than with ordinary loads)
#pragma unroll
  for (int i = 0; i < 2 * (D / 32); ++i) r.k[i] = __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4*)(kb + i * 64)));
#pragma unroll
  for (int i = 0; i < D / 16; ++i) r.v[i] = __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4*)(vb + i * 64)));
}

// Scales of the eight tokens whose scores / probabilities a lane holds (INT8 caches): slot j is token
// 4 grp + j (j < 4) or 16 + 4 grp + j - 4 of the block.
struct TokenScales {
  float k[8], v[8];
};

// Reductions over the four lanes l, l + 16, l + 32, l + 48 (the lanes that share a query row in the
// matrix-core result layout) with gfx950's lane-swap instructions: v_permlane32_swap of a value with
// itself leaves (low half, low half) and (high half, high half), v_permlane16_swap (rows 0 and 2 twice)
// and (rows 1 and 3 twice) -- two VALU operations per step instead of two trips through the LDS crossbar.
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

__device__ inline float rows4_max(float v) {
  const u32x2 a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  const u32x2 b = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}

__device__ inline float rows4_sum(float v) {
  const u32x2 a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  const u32x2 b = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// INT8 caches: a block's codes and the scales of this lane's tokens.  k[tt * (D/64) + ks]: the 16 codes of
// token 16 tt + lane % 16, head elements 64 ks + 16 grp ..; v[m]: V fragments 2m and 2m + 1 (8 codes each).
template <int D>
struct KvRegsI8 {
  u32x4 k[D / 32], v[D / 32];
  f32x4 ks[2], vs[2];  // tokens 4 grp .. 4 grp + 3 and 16 + 4 grp .. 16 + 4 grp + 3
};

// kb, vb: the block's first uint4; lane16 / grp16 are this lane's offsets (0 for a dummy fetch)
template <int D>
__device__ inline void load_block_i8(KvRegsI8<D>& r, const uint4* kb, const uint4* vb, int lane16, int grp16) {
#pragma unroll
  for (int i = 0; i < D / 32; ++i) r.k[i] = __builtin_nontemporal_load((const u32x4*)(kb + i * 64 + lane16));
#pragma unroll
  for (int i = 0; i < D / 32; ++i) r.v[i] = __builtin_nontemporal_load((const u32x4*)(vb + i * 64 + lane16));
  const f32x4* ks = (const f32x4*)(kb + 2 * D);  // the codes take 32 D bytes = 2 D uint4
  const f32x4* vs = (const f32x4*)(vb + 2 * D);
  r.ks[0] = ks[grp16];
  r.ks[1] = ks[4 + grp16];
  r.vs[0] = vs[grp16];
  r.vs[1] = vs[4 + grp16];
}

// eight INT8 codes (two words) -> eight bf16 (exact: |code| <= 127)
__device__ inline uint4 codes_to_bf16(uint32_t lo, uint32_t hi) {
  bf16x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = (__bf16)(float)(int)(int8_t)((e < 4 ? lo : hi) >> (8 * (e & 3)));
  return __builtin_bit_cast(uint4, o);
}

// V codes -> bf16 fragments (the K codes go to the INT8 matrix instruction as they are) and the scales
template <int D>
__device__ inline void dequant_block(const KvRegsI8<D>& q, KvRegs<D>& r, TokenScales& sc) {
#pragma unroll
  for (int f = 0; f < D / 16; ++f) r.v[f] = codes_to_bf16(q.v[f >> 1][2 * (f & 1)], q.v[f >> 1][2 * (f & 1) + 1]);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    sc.k[j] = q.ks[0][j];
    sc.k[4 + j] = q.ks[1][j];
    sc.v[j] = q.vs[0][j];
    sc.v[4 + j] = q.vs[1][j];
  }
}

// Fused append: the step's own K/V rows of one unit (rows i < nq of K_new, V_new for sequence b,
// kv head kvh).  The wavefront whose share holds the unit's last blocks copies those rows into its
// own slice of LDS before it starts streaming; when it reaches the (masked) blocks the new tokens
// belong to, it patches the fetched K and V fragments from LDS and writes the patched 16-byte
// chunks back into the cache (plain stores that nobody waits for: no other wavefront reads those
// blocks in this launch).  The patch needs no global load, so the ring of outstanding K/V fetches
// is never drained for it.
extern __shared__ __align__(16) unsigned char new_rows_lds[];

struct NewRows {
  unsigned k_off, v_off;    // byte offsets of the unit's K and V rows in new_rows_lds: [row][D] bf16, or INT8 codes
  unsigned ks_off, vs_off;  // INT8 caches: the rows' fp32 scales
  int L, nq;
};

// A pass copies 128 16-byte chunks (2 per lane and tensor): 8 rows of 128 head elements.  The first
// pass overlaps the first K/V fetches; longer drafts take further passes, one after the other.
// The host keeps kmax * D <= kMaxStagedElems so that a workgroup's slices fit in 64 KiB of LDS.
constexpr int kStageLoads = 2;
constexpr int kStagePass = kStageLoads * 64;

struct StageRegs {
  u32x4 k[kStageLoads], v[kStageLoads];
};

// Loads of a unit's nq new rows, chunk c = c0 + 64 i + lane: row c / (D/8), head elements 8 (c % (D/8)) ..
template <int D>
__device__ inline void stage_issue(const AttnParams& p, const Unit& u, int c0, int lane, StageRegs& sr) {
  constexpr int CPR = D / 8;
  const size_t row_stride = (size_t)p.Hkv * D;
  const size_t first = ((size_t)u.b * p.kmax * p.Hkv + u.kvh) * D;
  const uint16_t* kn = (const uint16_t*)p.Knew + first;
  const uint16_t* vn = (const uint16_t*)p.Vnew + first;
  const int nchunks = u.nq * CPR;
  const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int i = 0; i < kStageLoads; ++i) {
    sr.k[i] = zero;
    sr.v[i] = zero;
    if (c0 + i * 64 < nchunks) {  // wave-uniform
      const int c = min(c0 + i * 64 + lane, nchunks - 1);  // lanes past the end repeat the last chunk
      const size_t e = (size_t)(c / CPR) * row_stride + 8 * (c % CPR);
      sr.k[i] = *(const u32x4*)(kn + e);
      sr.v[i] = *(const u32x4*)(vn + e);
    }
  }
}

template <int D>
__device__ inline void stage_commit(const Unit& u, int c0, int lane, const StageRegs& sr, const NewRows& nr) {
  const int nchunks = u.nq * (D / 8);
#pragma unroll
  for (int i = 0; i < kStageLoads; ++i) {
    const int c = c0 + i * 64 + lane;
    if (c < nchunks) {
      *(u32x4*)&new_rows_lds[nr.k_off + 16 * c] = sr.k[i];
      *(u32x4*)&new_rows_lds[nr.v_off + 16 * c] = sr.v[i];
    }
  }
}

// INT8 caches: the staged rows are quantized on the way into LDS (codes [row][D] bytes, one fp32 scale
// per row), exactly as the append kernel does; a row's D/8 chunks sit in consecutive lanes.
template <int D>
__device__ inline void stage_commit_i8(const Unit& u, int c0, int lane, const StageRegs& sr, const NewRows nr) {
  constexpr int CPR = D / 8;
  const int nchunks = u.nq * CPR;
#pragma unroll
  for (int i = 0; i < kStageLoads; ++i) {
    if (c0 + i * 64 < nchunks) {  // wave-uniform
      const int c = c0 + i * 64 + lane;
      const uint4 kv = __builtin_bit_cast(uint4, sr.k[i]), vv = __builtin_bit_cast(uint4, sr.v[i]);
      float ka = amax8(kv), va = amax8(vv);
#pragma unroll
      for (int o = CPR >> 1; o >= 1; o >>= 1) {
        ka = fmaxf(ka, __shfl_xor(ka, o));
        va = fmaxf(va, __shfl_xor(va, o));
      }
      if (c < nchunks) {
        const float kinv = ka > 0.f ? 127.0f / ka : 0.f;
        const float vinv = va > 0.f ? 127.0f / va : 0.f;
        *(uint2*)&new_rows_lds[nr.k_off + 8 * c] = quantize8(kv, kinv);
        *(uint2*)&new_rows_lds[nr.v_off + 8 * c] = quantize8(vv, vinv);
        if (c % CPR == 0) {
          *(float*)&new_rows_lds[nr.ks_off + 4 * (c / CPR)] = ka / 127.0f;
          *(float*)&new_rows_lds[nr.vs_off + 4 * (c / CPR)] = va / 127.0f;
        }
      }
    }
  }
}

// INT8 caches, fused append: put the new tokens' codes and scales into the fetched block (before it is
// widened) and write them into the cache block at kblk / vblk (first byte of the block).
template <int D>
__device__ inline void patch_block_i8(KvRegsI8<D>& q, int tok0, const NewRows nr, int lane, uint8_t* kblk, uint8_t* vblk) {
  constexpr int KS = D / 64, MT = D / 16;
  const int dr = lane & 15, grp = lane >> 4;
  // K: chunk tl * KS + ks of a lane is token 16 tl + lane % 16, head elements 64 ks + 16 grp .. + 15
#pragma unroll
  for (int tl = 0; tl < 2; ++tl) {
    const int i = tok0 + 16 * tl + dr - nr.L;
    if (i >= 0 && i < nr.nq) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const u32x4 c = *(const u32x4*)&new_rows_lds[nr.k_off + i * D + 64 * ks + 16 * grp];
        q.k[tl * KS + ks] = c;
        *(u32x4*)(kblk + ((tl * KS + ks) * 64 + lane) * 16) = c;
      }
    }
  }
  // V codes and both scales: slot j of a lane is token 4 grp + j (j < 4) or 16 + 4 grp + j - 4
  bool v_new = false;
  float* kscale = (float*)(kblk + kBlockTokens * D);
  float* vscale = (float*)(vblk + kBlockTokens * D);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int w = j < 4 ? 4 * grp + j : 16 + 4 * grp + (j - 4);
    const int i = tok0 + w - nr.L;
    if (i >= 0 && i < nr.nq) {
      v_new = true;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const uint32_t code = new_rows_lds[nr.v_off + i * D + 16 * mt + dr];
        const uint32_t word = q.v[mt >> 1][2 * (mt & 1) + (j >> 2)];
        q.v[mt >> 1][2 * (mt & 1) + (j >> 2)] = (word & ~(0xFFu << (8 * (j & 3)))) | (code << (8 * (j & 3)));
      }
      const float ks = *(const float*)&new_rows_lds[nr.ks_off + 4 * i];
      const float vs = *(const float*)&new_rows_lds[nr.vs_off + 4 * i];
      q.ks[j >> 2][j & 3] = ks;
      q.vs[j >> 2][j & 3] = vs;
      if (dr == 0) {  // one lane per token group writes the scales
        kscale[w] = ks;
        vscale[w] = vs;
      }
    }
  }
  if (v_new) {
#pragma unroll
    for (int m = 0; m < D / 32; ++m) *(u32x4*)(vblk + (m * 64 + lane) * 16) = q.v[m];
  }
}

constexpr float kMaxSlack = 8.f;  // see block_step

template <int D, int NT>
struct RowState {
  f32x4 acc[NT][D / 16];
  float m[NT];  // running max (log2 units), identical in the 4 lanes that share a query row
  float l[NT];  // this lane's share of the running sum
};

// One 32-token block against all query tiles.  kMasked: the block reaches beyond ctx_len, so
// causal limits and the valid-token bound apply (wave-uniform choice).
// INT8 caches: what the block step needs besides the widened V fragments -- the block's K codes, the
// quantized queries and all the scales.
template <int D, int NT>
struct I8Operands {
  const u32x4* k;                 // KvRegsI8::k of the block
  const u32x4 (*q)[D / 64];       // query codes, B operand of the INT8 matrix instruction
  const float* q_scale_log2;      // per tile: this lane's query-row scale * softmax scale * log2(e)
  const TokenScales* sc;
};

template <int D, int NT, bool kMasked, bool kI8 = false>
__device__ inline void block_step(KvRegs<D>& r, const bf16x8 (&qf)[NT][D / 32], RowState<D, NT>& st, int tok0,
                                  int n_valid, const int (&lim)[NT], float scale_log2, int lane,
                                  bool fused = false, const NewRows& nr = NewRows{}, uint4* kdst = nullptr,
                                  uint4* vdst = nullptr, const I8Operands<D, NT>* i8 = nullptr) {
  constexpr int KS = D / 32, MT = D / 16;
  const int grp = lane >> 4;
  // INT8 caches: a score is the integer product (q codes . k codes) * q-scale * k-scale, a value is
  // code * v-scale, the latter folded into the probabilities that multiply V (r.v holds the codes as
  // bf16).  Stale tokens may carry any scale.
  float vsl[8];
  if (kI8) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      vsl[j] = i8->sc->v[j];
      if (kMasked && tok0 + (j < 4 ? 4 * grp + j : 16 + 4 * grp + (j - 4)) >= n_valid) vsl[j] = 0.f;
    }
  }
  bool v_new = false;  // this lane's V chunks hold a new token
  if (kMasked && fused) {
    const int dr = lane & 15;
    // K: fragment tl * KS + t of a lane is token 16 tl + lane % 16, head elements 32 t + 8 grp .. + 7:
    // one 16-byte chunk of the new row
#pragma unroll
    for (int tl = 0; tl < 2; ++tl) {
      const int i = tok0 + 16 * tl + dr - nr.L;
      if (i >= 0 && i < nr.nq) {
#pragma unroll
        for (int t = 0; t < KS; ++t) {
          const u32x4 kv = *(const u32x4*)&new_rows_lds[nr.k_off + 2 * (i * D + 32 * t + 8 * grp)];
          r.k[tl * KS + t] = __builtin_bit_cast(uint4, kv);
          *(u32x4*)(kdst + (tl * KS + t) * 64) = kv;
        }
      }
    }
    // V: slot j of a lane is token 4 grp + j (j < 4) or 16 + 4 grp + j - 4, head element 16 mt + lane % 16
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int i = tok0 + (j < 4 ? 4 * grp + j : 16 + 4 * grp + (j - 4)) - nr.L;
      if (i >= 0 && i < nr.nq) {
        v_new = true;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const uint32_t v = *(const uint16_t*)&new_rows_lds[nr.v_off + 2 * (i * D + 16 * mt + dr)];
          uint32_t* wv = (uint32_t*)&r.v[mt];
          wv[j >> 1] = (j & 1) ? (wv[j >> 1] & 0x0000FFFFu) | (v << 16) : (wv[j >> 1] & 0xFFFF0000u) | v;
        }
      }
    }
  }
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
    if (v_new) {  // the patched chunks go back into the cache (stale slots zeroed: they may hold anything)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) *(u32x4*)(vdst + mt * 64) = __builtin_bit_cast(u32x4, r.v[mt]);
    }
  }
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    float s[8];
    if constexpr (kI8) {
      i32x4 a0 = {0, 0, 0, 0}, a1 = {0, 0, 0, 0};
#pragma unroll
      for (int ks = 0; ks < D / 64; ++ks) {
        a0 = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4, i8->k[ks]), __builtin_bit_cast(i32x4, i8->q[nt][ks]), a0, 0, 0, 0);
        a1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4, i8->k[D / 64 + ks]), __builtin_bit_cast(i32x4, i8->q[nt][ks]), a1, 0, 0, 0);
      }
      const float qs = i8->q_scale_log2[nt];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        s[j] = (float)a0[j] * (i8->sc->k[j] * qs);
        s[4 + j] = (float)a1[j] * (i8->sc->k[4 + j] * qs);
      }
    } else {
      f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int t = 0; t < KS; ++t) {
        s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, r.k[t]), qf[nt][t], s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, r.k[KS + t]), qf[nt][t], s1, 0, 0, 0);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        s[j] = s0[j] * scale_log2;
        s[4 + j] = s1[j] * scale_log2;
      }
    }
    if (kMasked) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (tok0 + 4 * grp + j > lim[nt]) s[j] = -INFINITY;
        if (tok0 + 16 + 4 * grp + j > lim[nt]) s[4 + j] = -INFINITY;
      }
    }
    float mx = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
    mx = rows4_max(mx);
    // The reference maximum of a row moves only when a block exceeds it by more than kMaxSlack (log2 units).
    // The probabilities are then at most 2^kMaxSlack -- harmless in the fp32 sums and in the bf16 operand --
    // and the rescale of the running sum and of the accumulator (a third of a block step's instructions at
    // one wavefront per SIMD, where every instruction is paid for) runs in a unit's first block and hardly
    // ever again.  Wave-uniform branch; a row that does not move has alpha = 1.
    const float m_old = st.m[nt];
    const bool grow = mx > m_old + kMaxSlack;
    if (__any(grow)) {
      const float m_new = grow ? mx : m_old;
      const float m_to = (kMasked && m_new == -INFINITY) ? 0.f : m_new;  // rows without a visible token yet
      const float alpha = __builtin_amdgcn_exp2f(m_old - m_to);
      st.l[nt] *= alpha;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) st.acc[nt][mt] *= alpha;
      st.m[nt] = m_new;
    }
    // a row that has seen no visible token yet keeps m = -inf; subtract 0 instead so that
    // exp2(-inf - 0) = 0 and no inf - inf appears
    const float m_use = (kMasked && st.m[nt] == -INFINITY) ? 0.f : st.m[nt];
    float psum = 0.f;
    bf16x8 pf;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float pj = __builtin_amdgcn_exp2f(s[j] - m_use);
      psum += pj;
      pf[j] = (__bf16)(kI8 ? pj * vsl[j] : pj);
    }
    st.l[nt] += psum;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      st.acc[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, r.v[mt]), pf, st.acc[nt][mt], 0, 0, 0);
  }
}

template <int D, int NT, bool kI8 = false>
__device__ inline void block_dispatch(KvRegs<D>& r, const bf16x8 (&qf)[NT][D / 32], RowState<D, NT>& st, int blk,
                                      int L, int n_valid, const int (&lim)[NT], float scale_log2, int lane,
                                      bool fused, const NewRows& nr, uint4* kdst, uint4* vdst,
                                      const I8Operands<D, NT>* i8 = nullptr) {
  const int tok0 = blk * kBlockTokens;
  // plain step: every token of the block is visible to every query (tokens <= L) and, with a fused
  // append, none of them is new (tokens < L)
  if (tok0 + kBlockTokens - 1 < L + (fused ? 0 : 1))
    block_step<D, NT, false, kI8>(r, qf, st, tok0, n_valid, lim, scale_log2, lane, false, NewRows{}, nullptr, nullptr, i8);
  else
    block_step<D, NT, true, kI8>(r, qf, st, tok0, n_valid, lim, scale_log2, lane, fused, nr, kdst, vdst, i8);
}

// fp32 path: the wavefront whose share holds the new rows copies them into the (token-major) cache
// and waits for the stores before it fetches those rows; nobody else reads them in this launch.
__device__ inline bool append_own_rows_fp32(const AttnParams& p, const Unit& u, int blk_lo, int nblk, int lane) {
  const int t_lo = max(u.L, blk_lo * kBlockTokens);
  const int t_hi = min(u.L + u.nq, (blk_lo + nblk) * kBlockTokens);
  if (t_lo >= t_hi) return false;
  float* kc = (float*)const_cast<void*>(p.Kc);
  float* vc = (float*)const_cast<void*>(p.Vc);
  for (int t = t_lo; t < t_hi; ++t) {
    const size_t row = (((size_t)u.b * p.kmax + (t - u.L)) * p.Hkv + u.kvh) * p.D;
    const size_t dst = (((size_t)u.b * p.Hkv + u.kvh) * p.Lcap + t) * p.D;
    for (int d = 4 * lane; d < p.D; d += 256) {
      *(float4*)(kc + dst + d) = *(const float4*)((const float*)p.Knew + row + d);
      *(float4*)(vc + dst + d) = *(const float4*)((const float*)p.Vnew + row + d);
    }
  }
  return true;
}

template <int D, int NT>
struct QFrag {
  bf16x8 q[NT][D / 32];  // B operand: lane (col, grp) holds query row 16 nt + col, elements 32 t + 8 grp .. +7
  int lim[NT];           // last token visible to that row
};

template <int D, int NT>
__device__ inline void load_queries(const AttnParams& p, const Unit& u, bool enable, int col, int grp, QFrag<D, NT>& f,
                                    int row0 = 0) {
  const int rows = u.nq * p.g;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int rrow = row0 + nt * 16 + col;  // row0: first query row of this wavefront (tile kernel)
    const bool ok = enable && rrow < rows;
    const int i = ok ? row_token(p, rrow) : 0, hg = ok ? rrow - i * p.g : 0;
    f.lim[nt] = u.L + i;
    const uint4* qrow = (const uint4*)((const uint16_t*)p.Q + (((size_t)u.b * p.kmax + i) * p.Hq + u.kvh * p.g + hg) * D);
#pragma unroll
    for (int t = 0; t < D / 32; ++t) {
      uint4 qv = make_uint4(0, 0, 0, 0);
      if (ok) qv = qrow[t * 4 + grp];
      f.q[nt][t] = __builtin_bit_cast(bf16x8, qv);
    }
  }
}

// INT8 caches: the queries are quantized like the cache rows (one scale per token and query head, codes
// rint(x * 127 / amax)) so that QK^T runs on the INT8 matrix cores.  B operand of the 16x16x64
// instruction: lane (col, grp) holds query row 16 nt + col, head elements 64 ks + 16 grp .. + 15.
template <int D, int NT>
struct QFragI8 {
  u32x4 q[NT][D / 64];
  float q_scale_log2[NT];  // row scale (amax / 127) * softmax scale * log2(e)
  int lim[NT];
};

template <int D, int NT>
__device__ inline void load_queries_i8(const AttnParams& p, const Unit& u, bool enable, int col, int grp, QFragI8<D, NT>& f) {
  const int rows = u.nq * p.g;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int rrow = nt * 16 + col;
    const bool ok = enable && rrow < rows;
    const int i = ok ? row_token(p, rrow) : 0, hg = ok ? rrow - i * p.g : 0;
    f.lim[nt] = u.L + i;
    const uint4* qrow = (const uint4*)((const uint16_t*)p.Q + (((size_t)u.b * p.kmax + i) * p.Hq + u.kvh * p.g + hg) * D);
    uint4 raw[D / 64][2];
    float amax = 0.f;
#pragma unroll
    for (int ks = 0; ks < D / 64; ++ks)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        raw[ks][h] = ok ? qrow[ks * 8 + grp * 2 + h] : make_uint4(0, 0, 0, 0);
        amax = fmaxf(amax, amax8(raw[ks][h]));
      }
    amax = rows4_max(amax);  // the four lanes of a row hold a quarter of it each
    const float inv = amax > 0.f ? 127.0f / amax : 0.f;
#pragma unroll
    for (int ks = 0; ks < D / 64; ++ks) {
      const uint2 lo = quantize8(raw[ks][0], inv), hi = quantize8(raw[ks][1], inv);
      f.q[nt][ks] = u32x4{lo.x, lo.y, hi.x, hi.y};
    }
    f.q_scale_log2[nt] = amax / 127.0f * p.scale_log2;
  }
}

template <int D, int NT>
__device__ inline void clear_state(RowState<D, NT>& st) {
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    st.m[nt] = -INFINITY;
    st.l[nt] = 0.f;
#pragma unroll
    for (int mt = 0; mt < D / 16; ++mt) st.acc[nt][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
}

// Partial of (wavefront w, unit u): slot ids w + unit are unique because both grow monotonically
// along the flattened list.
template <int D, int NT>
__device__ inline void store_partial(const AttnParams& p, const Unit& u, int w, const RowState<D, NT>& st, int col, int grp,
                                     int row0 = 0) {
  const int rows = u.nq * p.g;
  const size_t slot = (size_t)w + (size_t)u.b * p.Hkv + u.kvh;
  const __amdgpu_buffer_rsrc_t rs = dev_buffer(p.part_acc + slot * p.rows_max * D, (unsigned)p.rows_max * D * 4);
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    float l = st.l[nt];
    l = rows4_sum(l);
    const int rrow = row0 + nt * 16 + col;
    if (rrow < rows) {
      const unsigned off = (unsigned)(rrow * D + 4 * grp) * 4;
#pragma unroll
      for (int mt = 0; mt < D / 16; ++mt) store_dev4(rs, off + 64 * mt, st.acc[nt][mt]);
      if (grp == 0) store_dev(p.part_ml + (slot * p.rows_max + rrow) * 2, st.m[nt], l);
    }
  }
}

// A unit that this wavefront streamed alone needs no exchange: its output rows are written straight from the
// registers.  The arithmetic is that of the merge of a single partial (weight 2^0 = 1, the same reciprocal and
// logarithm), so a unit's result does not depend on which of the two ways it took.
template <int D, int NT>
__device__ inline void finalize_single(const AttnParams& p, const Unit& u, const RowState<D, NT>& st, int col, int grp,
                                       int row0 = 0) {
  const int rows = u.nq * p.g;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const float L = fmaf(rows4_sum(st.l[nt]), 1.0f, 0.f);
    const int rrow = row0 + nt * 16 + col;
    if (rrow < rows) {
      const float M = st.m[nt];
      const float invL = __builtin_amdgcn_rcpf(L);
      const int i = row_token(p, rrow), hg = rrow - i * p.g;
      const size_t orow = ((size_t)u.b * p.kmax + i) * p.Hq + u.kvh * p.g + hg;
#pragma unroll
      for (int mt = 0; mt < D / 16; ++mt) *(f32x4*)(p.O + orow * D + 16 * mt + 4 * grp) = st.acc[nt][mt] * invL;
      if (p.lse && grp == 0) p.lse[orow] = (M + __builtin_amdgcn_logf(L)) * 0.6931471805599453f;
    }
  }
}

template <int D, int NT, bool kI8 = false>
__global__ __launch_bounds__(256) void verify_attn_bf16(AttnParams p) {
  // uint4 per block: 32 tokens of D bf16, or of D INT8 codes followed by 32 fp32 scales
  constexpr ptrdiff_t kBlkVec = kI8 ? 2 * D + 8 : (ptrdiff_t)kBlockTokens * D * 2 / 16;
  using Regs = typename std::conditional<kI8, KvRegsI8<D>, KvRegs<D>>::type;
  // With one query tile there are registers to spare for a second unit's state, so a wavefront
  // whose share of blocks crosses a unit boundary keeps streaming: it parks the first unit's
  // accumulators, carries on with the second unit, and delivers both partials at the end.
  // (Storing the first partial at the boundary instead costs about 1 us per launch: the stores
  // sit in the ring's wait counts.)
  constexpr bool kPair = (NT == 1);
  const int lane = threadIdx.x & 63;
  const int w = uniform(blockIdx.x * p.wpw + (threadIdx.x >> 6));
  const int col = lane & 15, grp = lane >> 4;

  // This wavefront's share: the first two segments come with the record, in one round trip; the plan's
  // header travels at the same time.  Nothing waits for either before the first K/V fetch needs its
  // address: what the loop below sets up once (constants, lane offsets) runs under that round trip.
  const ShareRecord* rec = p.records + w;
  Segment sa = load_segment(&rec->seg[0]);
  Segment sb = load_segment(&rec->seg[1]);
  int nseg_plan = uniform(rec->nseg), overflow = uniform(rec->overflow);
  const int rec_flags = uniform(rec->flags);
  __builtin_amdgcn_sched_barrier(0);  // the loads above are issued here, whatever is scheduled below
  bool ok;
  int nseg;
  int si = 0;
  do {
    // The first fetch is issued before the plan has been checked, so its address is forced into the
    // cache whatever the record holds (a buffer without a plan must not turn into a wild read); stores
    // and everything else wait for the check.
    const int firstA = min(max(sa.first, 0), p.nblk_cap - 1);
    const ptrdiff_t unitA = (ptrdiff_t)min(max(sa.b, 0), p.B - 1) * p.Hkv + min(max(sa.kvh, 0), p.Hkv - 1);
    const ptrdiff_t vecA = (unitA * p.nblk_cap + firstA) * kBlkVec;
    const uint4* kc = (const uint4*)p.Kc;
    const uint4* vc = (const uint4*)p.Vc;
    Regs r0;
    if constexpr (kI8) load_block_i8<D>(r0, kc + vecA, vc + vecA, lane, grp);
    else load_block<D>(r0, kc + vecA + lane, vc + vecA + lane);
    ok = record_matches(p, rec);
    asm volatile("" : "+s"(nseg_plan), "+s"(overflow));  // as in record_matches: no use of the record ahead of the loop
    nseg = ok ? nseg_plan : 0;
    if (si >= nseg) break;  // an idle wavefront, or no plan for this launch
    const Unit uA = unit_of(sa);
    const int nA = sa.n;  // our real blocks of unit A: firstA .. firstA + nA - 1
    const bool hasB = kPair && si + 1 < nseg;
    // the segments after these (shares that touch more units than the record holds) are requested now and
    // looked at when this pair is done; without any, the request re-reads the record (loads stay outside
    // branches: the wait counts of the K/V ring must stay exact)
    const int si_next = si + (hasB ? 2 : 1);
    const SegmentInFlight nextA = request_segment(si_next < nseg ? later_segment_address(p, rec, overflow, si_next) : &rec->seg[0]);
    const SegmentInFlight nextB =
        request_segment(kPair && si_next + 1 < nseg ? later_segment_address(p, rec, overflow, si_next + 1) : &rec->seg[1]);
    const Unit uB = hasB ? unit_of(sb) : uA;
    const int firstB = hasB ? sb.first : 0, nB = hasB ? sb.n : 0;
    const bool lastA = (sa.flags & kSegLast) != 0, lastB = hasB && (sb.flags & kSegLast) != 0;  // we hold the unit's last block
    const int n = nA + nB;

    typename std::conditional<kI8, QFragI8<D, NT>, QFrag<D, NT>>::type qc, qB;
    if constexpr (kI8) {
      load_queries_i8<D, NT>(p, uA, true, col, grp, qc);
      if constexpr (kPair) load_queries_i8<D, NT>(p, uB, hasB, col, grp, qB);
    } else {
      load_queries<D, NT>(p, uA, true, col, grp, qc);
      if constexpr (kPair) load_queries<D, NT>(p, uB, hasB, col, grp, qB);
    }
    RowState<D, NT> st, parked;
    clear_state<D, NT>(st);
    CombineJob ja = job_of(sa), jb = ja;  // who else contributes to our units
    if (hasB) jb = job_of(sb);
    int cur_L = uA.L, cur_valid = uA.L + uA.nq, cur_blk = firstA;  // block index = cur_blk + s

    // fused append: the units whose new tokens lie in our blocks get their rows staged in LDS
    const bool fused = p.Knew != nullptr;
    // one unit's slice: K rows, V rows (bf16, or INT8 codes), then for INT8 the rows' K and V scales
    const unsigned lds_rows = (unsigned)p.kmax * D * (kI8 ? 1 : 2);
    const unsigned lds_unit = 2 * lds_rows + (kI8 ? 8 * (unsigned)p.kmax : 0);
    const unsigned lds_base = (threadIdx.x >> 6) * 2 * lds_unit;
    const NewRows newA{lds_base, lds_base + lds_rows, lds_base + 2 * lds_rows, lds_base + 2 * lds_rows + 4 * (unsigned)p.kmax,
                       uA.L, uA.nq};
    const NewRows newB{newA.k_off + lds_unit, newA.v_off + lds_unit, newA.ks_off + lds_unit, newA.vs_off + lds_unit,
                       uB.L, uB.nq};
    NewRows cur_new = newA;
    const bool stageA = fused && uA.nq > 0 && (firstA + nA) * kBlockTokens > uA.L;
    const bool stageB = fused && hasB && uB.nq > 0 && (firstB + nB) * kBlockTokens > uB.L;
    // one set of staging registers: a share that holds the new tokens of both its units is rare (the
    // second unit then lies wholly inside the share) and stages the second unit's rows afterwards
    const bool stage1 = stageA || stageB;
    const Unit& u1 = stageA ? uA : uB;
    const NewRows new1 = stageA ? newA : newB;  // a copy: a reference would put both structs in memory
    StageRegs sr;
    if (stage1) stage_issue<D>(p, u1, 0, lane, sr);
    auto commit = [&](const Unit& u, int c0, const StageRegs& regs, const NewRows nr) {
      if constexpr (kI8) stage_commit_i8<D>(u, c0, lane, regs, nr);
      else stage_commit<D>(u, c0, lane, regs, nr);
    };
    // what is left after the overlapped pass (drafts of more than 8 rows, a second unit): rare
    auto stage_rest = [&]() {
      for (int c0 = kStagePass; c0 < u1.nq * (D / 8); c0 += kStagePass) {
        StageRegs sr2;
        stage_issue<D>(p, u1, c0, lane, sr2);
        commit(u1, c0, sr2, new1);
      }
      if (stageA && stageB)
        for (int c0 = 0; c0 < uB.nq * (D / 8); c0 += kStagePass) {
          StageRegs sr2;
          stage_issue<D>(p, uB, c0, lane, sr2);
          commit(uB, c0, sr2, newB);
        }
    };

    // element offsets (in uint4) of step s inside the K and V caches
    const ptrdiff_t vecB = (((ptrdiff_t)uB.b * p.Hkv + uB.kvh) * p.nblk_cap + firstB - nA) * kBlkVec;

    // Every fetch is issued unconditionally so that the wait counts before each compute step are
    // exact (a fetch under a branch would force a wait for ALL outstanding loads at the join and
    // serialise load and compute).  A fetch past the end of the share reads 16 bytes of the
    // share's first block with every lane instead: valid memory, one cache line, never used.
    auto fetch = [&](Regs& r, int s) {
      if constexpr (kI8) {
        const bool real = s < n;
        const ptrdiff_t off = real ? (s < nA ? vecA : vecB) + (ptrdiff_t)s * kBlkVec : vecA;
        load_block_i8<D>(r, kc + off, vc + off, real ? lane : 0, real ? grp : 0);
      } else {
        ptrdiff_t off = vecA;
        if (s < n) off = (s < nA ? vecA : vecB) + (ptrdiff_t)s * kBlkVec + lane;
        load_block<D>(r, kc + off, vc + off);
      }
    };
    auto step = [&](Regs& r, int s) {
      if constexpr (kPair) {
        if (s == nA) {  // first block of unit B: park A's state (register moves only)
          parked = st;
          clear_state<D, NT>(st);
          qc = qB;
          cur_L = uB.L;
          cur_valid = uB.L + uB.nq;
          cur_blk = firstB - nA;
          cur_new = newB;
        }
      }
      const ptrdiff_t own = (s < nA ? vecA : vecB) + (ptrdiff_t)s * kBlkVec + lane;  // this lane's chunks of block s
      uint4* kdst = (uint4*)const_cast<void*>(p.Kc) + own;
      uint4* vdst = (uint4*)const_cast<void*>(p.Vc) + own;
      if constexpr (kI8) {
        if (fused && (cur_blk + s) * kBlockTokens + kBlockTokens - 1 >= cur_L) {  // the block holds new tokens
          const ptrdiff_t blk_vec = (s < nA ? vecA : vecB) + (ptrdiff_t)s * kBlkVec;
          patch_block_i8<D>(r, (cur_blk + s) * kBlockTokens, cur_new, lane,
                            (uint8_t*)const_cast<void*>(p.Kc) + blk_vec * 16, (uint8_t*)const_cast<void*>(p.Vc) + blk_vec * 16);
        }
        KvRegs<D> t;
        TokenScales sc;
        dequant_block<D>(r, t, sc);
        const I8Operands<D, NT> i8{r.k, qc.q, qc.q_scale_log2, &sc};
        const bf16x8 no_q[NT][D / 32] = {};
        block_dispatch<D, NT, true>(t, no_q, st, cur_blk + s, cur_L, cur_valid, qc.lim, p.scale_log2, lane, false,
                                    cur_new, nullptr, nullptr, &i8);  // the codes are patched already: no fused work inside
      } else {
        block_dispatch<D, NT>(r, qc.q, st, cur_blk + s, cur_L, cur_valid, qc.lim, p.scale_log2, lane, fused, cur_new, kdst, vdst);
      }
    };
    // Unused query rows of a unit are cleared by the wavefront that holds the unit's last block (it is handed
    // fewer real blocks), while its first fetches are under way: the stores are acknowledged long before the
    // wavefront waits for its partial stores at the end, and nothing waits for them here.
    auto clear_unused = [&]() {
      if (lastA) zero_rows<D>(p, uA.b, uA.kvh, uA.nq * p.g, lane);
      if (lastB) zero_rows<D>(p, uB.b, uB.kvh, uB.nq * p.g, lane);
    };
    // The next segments were requested right behind the first block and are here with it; kept as scalars
    // from here on, they do not take vector registers away from the ring.
    Segment next_sa, next_sb;
    auto next_arrived = [&]() {
      next_sa = arrived_segment(nextA);
      next_sb = arrived_segment(nextB);
    };
    if constexpr (NT <= 2) {
      // three-deep register ring: two blocks (32 KiB per wavefront) in flight while one is computed
      Regs r1, r2;  // r0 is on its way already
      fetch(r1, 1);
      if (stage1) {
        commit(u1, 0, sr, new1);  // these loads were issued before the fetches
        stage_rest();
      }
      clear_unused();
      next_arrived();
      for (int s = 0; s < n; s += 3) {
        fetch(r2, s + 2);
        step(r0, s);
        fetch(r0, s + 3);
        if (s + 1 < n) step(r1, s + 1);
        fetch(r1, s + 4);
        if (s + 2 < n) step(r2, s + 2);
      }
    } else {
      // many query rows need the registers for accumulators: two-deep ring
      Regs r1;
      if (stage1) {
        commit(u1, 0, sr, new1);
        stage_rest();
      }
      clear_unused();
      next_arrived();
      for (int s = 0; s < n; s += 2) {
        fetch(r1, s + 1);
        step(r0, s);
        fetch(r0, s + 2);
        if (s + 1 < n) step(r1, s + 1);
      }
    }
    // A unit that lies wholly inside this share (common with many short sequences) is finished from the
    // registers; the others leave a partial, and the wavefront that delivers a unit's last partial merges.
    // (With a merge launch of its own -- more than one query tile -- every unit leaves a partial.)
    const bool soloA = p.fused_reduce && ja.w_lo == ja.w_hi;
    const bool soloB = p.fused_reduce && hasB && jb.w_lo == jb.w_hi;
    if (hasB) {
      if (soloA) finalize_single<D, NT>(p, uA, parked, col, grp);
      else store_partial<D, NT>(p, uA, w, parked, col, grp);
      if (soloB) finalize_single<D, NT>(p, uB, st, col, grp);
      else store_partial<D, NT>(p, uB, w, st, col, grp);
    } else {
      if (soloA) finalize_single<D, NT>(p, uA, st, col, grp);
      else store_partial<D, NT>(p, uA, w, st, col, grp);
    }
    const bool exchA = !soloA, exchB = hasB && !soloB;
    if (p.fused_reduce && (exchA || exchB)) {
      partial_stores_done();
      bool mergeA = false, mergeB = false, unused;
      if (exchA) arrive(p, lane, ja, mergeA, exchB, jb, mergeB);
      else arrive(p, lane, jb, mergeB, false, jb, unused);
      if (mergeA || mergeB) combine_jobs<D>(p, ja, mergeA, jb, mergeB, lane);
    }
    si = si_next;
    sa = next_sa;
    sb = next_sb;
  } while (si < nseg);
  if (!ok) {
    report_mismatch(p, w == 0 && lane == 0);
    return;
  }
  // Unused query rows of inactive sequences (those of an active one: clear_unused above)
  if (rec_flags & kRecAnyInactive) zero_unused_rows<D, true>(p, w, p.nwaves, lane);
}

// ---------------------------------------------------------------------------------------
// Workgroup-level kernel for kv heads with more than 16 query rows (grouped-query attention), bf16.
// The accumulators of two to four 16-row tiles in ONE wavefront leave registers for a single block in
// flight, and re-reading blocks by several wavefronts crosses the fabric twice.  Here a workgroup of
// four wavefronts takes a stretch of the block list together: every K/V block is fetched from memory
// once (each wavefront a quarter of it, three blocks ahead), put into a two-slot ring in LDS, and
// read from there by the wavefronts that own a query tile (wavefront t: rows 16 t .. 16 t + 15), each
// running the one-tile block step.  A wavefront needs < 256 registers, so two workgroups share a
// compute unit.  One barrier per block: a slot is rewritten only after the barrier that follows the
// last step that read it.  Every barrier sits in workgroup-uniform control flow (the stretch, the
// units and the block counts depend on the workgroup index and the lengths only).
// ---------------------------------------------------------------------------------------
constexpr int kTileAhead = 3;  // blocks a workgroup has in flight from memory (measured best: 3)

template <int D, bool kFused>
__global__ __launch_bounds__(256, 2) void verify_attn_tiles_bf16(AttnParams p) {
  constexpr int kBlkVec = kBlockTokens * D * 2 / 16;  // uint4 per block and tensor
  constexpr int kQuarter = kBlkVec / 4;                // uint4 a wavefront moves per block and tensor
  constexpr int kLoads = kQuarter / 64;                // 16-byte loads per lane, block and tensor
  __shared__ uint4 ring_k[2][kBlkVec];
  __shared__ uint4 ring_v[2][kBlkVec];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int col = lane & 15, grp = lane >> 4;
  const int wg = blockIdx.x;  // the stretch of this workgroup
  const int row0 = 16 * wv;

  const ShareRecord* rec = p.records + wg;
  const int nseg = uniform(rec->nseg), overflow = uniform(rec->overflow);
  if (!record_matches(p, rec)) {
    report_mismatch(p, wg == 0 && threadIdx.x == 0);
    return;
  }
  // (the unused query rows are cleared by the merge launch, which visits every row of every unit anyway)

  const uint4* kc = (const uint4*)p.Kc;
  const uint4* vc = (const uint4*)p.Vc;
  struct Stage {
    uint4 k[kLoads], v[kLoads];
  };

  for (int si = 0; si < nseg; ++si) {
    const Segment seg = si == 0 ? load_segment(&rec->seg[0]) : later_segment(p, rec, overflow, si);
    const Unit u = unit_of(seg);
    const int n = seg.n;  // real blocks seg.first .. seg.first + n - 1 of the unit
    const bool active = row0 < u.nq * p.g;  // this wavefront owns a query tile of the unit
    QFrag<D, 1> q;
    load_queries<D, 1>(p, u, active, col, grp, q, row0);
    RowState<D, 1> st;
    clear_state<D, 1>(st);
    const int blk0 = seg.first;
    const ptrdiff_t vec0 = (((ptrdiff_t)u.b * p.Hkv + u.kvh) * p.nblk_cap + blk0) * kBlkVec;
    const int mine = wv * kQuarter + lane;  // first uint4 this lane moves

    // all fetches unconditional (exact wait counts); one past the end re-reads the stretch's first block
    auto fetch = [&](Stage& g, int s) {
      const ptrdiff_t off = vec0 + (s < n ? (ptrdiff_t)s * kBlkVec : 0) + mine;
#pragma unroll
      for (int i = 0; i < kLoads; ++i) g.k[i] = __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4*)(kc + off + i * 64)));
#pragma unroll
      for (int i = 0; i < kLoads; ++i) g.v[i] = __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4*)(vc + off + i * 64)));
    };
    // block s: own quarter into LDS, next fetch, barrier -- for every s, also past the end (the loads and
    // the barrier stay outside all branches: a load under a branch costs a full wait at the join) --
    // then, for real blocks, the one-tile step from LDS
    auto step = [&](Stage& g, int s) {
      const int slot = s & 1;
#pragma unroll
      for (int i = 0; i < kLoads; ++i) {
        ring_k[slot][mine + i * 64] = g.k[i];
        ring_v[slot][mine + i * 64] = g.v[i];
      }
      fetch(g, s + kTileAhead);
      // Fused append: a block that holds new tokens is patched in LDS once it is complete there (K: the
      // 16-byte chunks of the new rows; V: their elements, 2 bytes each), and the patched chunks go into the
      // cache from LDS as whole 16-byte chunks.  The test is workgroup-uniform; the loads of the new rows
      // sit under this branch and cost a full wait, in these one or two blocks per unit only.
      const int tok0 = (blk0 + s) * kBlockTokens;
      if (kFused && s < n && u.nq > 0 && tok0 < u.L + u.nq && tok0 + kBlockTokens > u.L) {
        __syncthreads();  // the block is complete in LDS
        const int i_hi = min(u.nq, tok0 + kBlockTokens - u.L);
        for (int i = max(0, tok0 - u.L) + wv; i < i_hi; i += 4) {  // new rows of this block, one per wavefront and turn
          const int tw = u.L + i - tok0;                              // its token slot in the block
          if (lane < D / 8) {                                         // one 16-byte chunk of the row per lane
            const size_t src = (((size_t)u.b * p.kmax + i) * p.Hkv + u.kvh) * D + 8 * lane;
            const uint4 kv = *(const uint4*)((const uint16_t*)p.Knew + src);
            const uint4 vv = *(const uint4*)((const uint16_t*)p.Vnew + src);
            const size_t ko = k_elem_offset(D, tw, 8 * lane) / 8;  // in 16-byte chunks
            ring_k[slot][ko] = kv;
            ((uint4*)const_cast<void*>(p.Kc))[vec0 + (ptrdiff_t)s * kBlkVec + (ptrdiff_t)ko] = kv;
            const uint32_t vw[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
            for (int e = 0; e < 8; ++e)
              ((uint16_t*)&ring_v[slot][0])[v_elem_offset(D, tw, 8 * lane + e)] = (uint16_t)(vw[e >> 1] >> (16 * (e & 1)));
          }
        }
        __syncthreads();  // the patches are visible
        for (int c = threadIdx.x; c < (D / 16) * 64; c += 256) {  // V chunks that hold a new token: back into the cache
          const int cg = (c & 63) >> 4;
          bool any = false;
#pragma unroll
          for (int jj = 0; jj < 8; ++jj) {
            const int t = tok0 + (jj < 4 ? 4 * cg + jj : 16 + 4 * cg + (jj - 4));
            any |= t >= u.L && t < u.L + u.nq;
          }
          if (any) ((uint4*)const_cast<void*>(p.Vc))[vec0 + (ptrdiff_t)s * kBlkVec + c] = ring_v[slot][c];
        }
      } else {
        __syncthreads();
      }
      if (active && s < n) {
        KvRegs<D> r;
#pragma unroll
        for (int i = 0; i < 2 * (D / 32); ++i) r.k[i] = ring_k[slot][i * 64 + lane];
#pragma unroll
        for (int i = 0; i < D / 16; ++i) r.v[i] = ring_v[slot][i * 64 + lane];
        block_dispatch<D, 1>(r, q.q, st, blk0 + s, u.L, u.L + u.nq, q.lim, p.scale_log2, lane, false, NewRows{}, nullptr, nullptr);
      }
    };
    __syncthreads();  // the previous unit's last step has left the ring
    Stage g[kTileAhead];
#pragma unroll
    for (int j = 0; j < kTileAhead; ++j) fetch(g[j], j);
    for (int s = 0; s < n; s += kTileAhead) {  // workgroup-uniform trip count
#pragma unroll
      for (int j = 0; j < kTileAhead; ++j) step(g[j], s + j);
    }
    if (active) store_partial<D, 1>(p, u, wg, st, col, grp, row0);
  }
}

// ---------------------------------------------------------------------------------------
// Split-context reduction as a launch of its own, used when a kv head has many query rows
// (grouped-query attention): a unit's partials are then tens of KiB per contributor, too much
// for the one wavefront that happens to arrive last, so the rows are spread over the whole chip:
// one wavefront per (unit, sweep of 4 rows).
// ---------------------------------------------------------------------------------------
template <int KC, int DC>
__global__ __launch_bounds__(256) void reduce_partials(AttnParams p) {
  const int lane = threadIdx.x & 63;
  const int sweeps = (p.rows_max + 3) / 4;
  const long item = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= (long)p.B * p.Hkv * sweeps) return;
  const int sweep = (int)(item % sweeps);
  const int unit = (int)(item / sweeps);
  const int b = unit / p.Hkv, kvh = unit % p.Hkv;
  if (!record_matches(p, p.records)) return;  // reported by the attention launch
  const int nq = uniform(p.seq_nq[b]);
  // query slots beyond draft_len (all of them for an inactive sequence) are zero in O and lse
  if (4 * sweep + 4 > nq * p.g) zero_rows<DC>(p, b, kvh, max(nq * p.g, 4 * sweep), lane, 4 * sweep + 4);
  if (nq == 0 || 4 * sweep >= nq * p.g) return;
  const int owners = uniform(p.unit_owners[unit]);
  CombineJob job{Unit{b, kvh, uniform(p.seq_L[b]), nq}, owners & 0xFFFF, (owners >> 16) & 0xFFFF};
  CombineRegs<KC> regs;
  combine_issue<KC, DC>(p, job, 4 * sweep, lane, regs);
  combine_finish<KC, DC>(p, job, lane, regs);
}

// ---------------------------------------------------------------------------------------
// fp32 kernel: same schedule and partial format, plain fp32 FMA arithmetic (no matrix cores;
// probabilities stay fp32).  Cache is token-major [B][Hkv][Lcap][D].  A wavefront handles up
// to 8 query rows at a time: lanes own tokens for the scores and head elements for P*V.
// ---------------------------------------------------------------------------------------
constexpr int kRowChunk = 8;

__global__ __launch_bounds__(256) void verify_attn_fp32(AttnParams p) {
  const int lane = threadIdx.x & 63;
  const int w = uniform(blockIdx.x * p.wpw + (threadIdx.x >> 6));
  const int D = p.D;
  const int nd = (D + 63) / 64;  // head elements per lane (<= 4)

  const ShareRecord* rec = p.records + w;
  const int nseg = uniform(rec->nseg), overflow = uniform(rec->overflow);
  if (!record_matches(p, rec)) {
    report_mismatch(p, w == 0 && lane == 0);
    return;
  }
  zero_unused_rows<0>(p, w, p.nwaves, lane);

  for (int si = 0; si < nseg; ++si) {
    const Segment seg = si == 0 ? load_segment(&rec->seg[0]) : later_segment(p, rec, overflow, si);
    const Unit u = unit_of(seg);
    const int blk0 = seg.first, nseg_blocks = seg.n;
    const int rows = u.nq * p.g;
    const int n_valid = u.L + u.nq;
    const int tok_lo = blk0 * kBlockTokens;
    const int tok_hi = min(n_valid, (blk0 + nseg_blocks) * kBlockTokens);
    if (p.Knew && append_own_rows_fp32(p, u, blk0, nseg_blocks, lane)) partial_stores_done();
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
            const int rrow = r0 + r, i = row_token(p, rrow), hg = rrow - i * p.g;
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
            if (k < nd && lane + 64 * k < D) store_dev1(dst + lane + 64 * k, acc[r][k]);
          if (lane == 0) store_dev(p.part_ml + (slot * p.rows_max + rrow) * 2, m[r], l[r]);
        }
      }
    }
    partial_stores_done();
    CombineJob job = job_of(seg);
    bool last, unused;
    arrive(p, lane, job, last, false, job, unused);
    if (last) combine_jobs<0>(p, job, true, job, false, lane);
  }
}

// Workspace = [unit counters, padded to 256 B][the plan of calls that bring none][partial outputs]
// [partial (max, sum) pairs], laid out for `shares` stretches.
struct Workspace {
  size_t plan, part_acc, part_ml, bytes;
};

static Workspace workspace_layout(const bass_attn_desc* d, int shares) {
  Workspace w;
  const size_t slots = (size_t)shares + (size_t)d->B * d->Hkv;
  const size_t rows = (size_t)d->kmax * (d->Hq / d->Hkv);
  w.plan = (((size_t)d->B * d->Hkv * sizeof(int32_t)) + 255) & ~(size_t)255;
  w.part_acc = w.plan + plan_layout(d->B, d->Hkv, shares).bytes;
  w.part_ml = w.part_acc + slots * rows * (size_t)d->D * sizeof(float);
  w.bytes = w.part_ml + slots * rows * 2 * sizeof(float);
  return w;
}

PlanShape plan_shape(const bass_attn_desc* d, const LaunchShape& ls, int span);
int launch_plan(const bass_attn_desc* d, const LaunchShape& ls, int span, const int32_t* ctx_len, const int32_t* draft_len,
                void* plan, int32_t* dev_status, void* stream, int32_t* clear_counters);

}  // namespace bass

extern "C" int bass_set_attention_waves(int waves) {
  bass::g_attention_waves.store(waves > 0 ? waves : 0, std::memory_order_relaxed);
  return bass::attention_waves(bass::attention_waves_setting(), false, false);
}

extern "C" size_t bass_verify_attention_workspace_bytes(const bass_attn_desc* d) {
  if (bass::check_desc(d) != BASS_OK) return 0;
  return bass::workspace_layout(d, bass::kMaxWaves).bytes;
}

namespace bass {

static int check_attention_args(const bass_attn_desc* d, const LaunchShape& ls, const void* Q, const void* K_new,
                                const void* V_new, const void* Kcache, const void* Vcache, const float* O,
                                const void* workspace) {
  if (!Q || !Kcache || !Vcache || !O || !workspace) return BASS_ERR_INVALID_ARG;
  if ((K_new == nullptr) != (V_new == nullptr)) return BASS_ERR_INVALID_ARG;
  if (((uintptr_t)workspace & 15) != 0) return BASS_ERR_INVALID_ARG;
  if (ls.mfma && ls.rows_max > 64) return BASS_ERR_UNSUPPORTED;
  // partials of one unit are addressed with 32-bit byte offsets
  if ((int64_t)ls.rows_max * d->D * 4 * kMaxWaves >= (1ll << 31)) return BASS_ERR_UNSUPPORTED;
  return BASS_OK;
}

// The attention launch (and, with many query rows per kv head, the merge launch) for a plan that lies at
// `plan`, made for the shape `ls`; K_new / V_new: the rows a fused append puts into the caches, or null.
static int launch_attention(const bass_attn_desc* d, const LaunchShape& ls, const void* Q, const void* K_new,
                            const void* V_new, const void* Kcache, const void* Vcache, const void* plan, float* O,
                            float* lse, const Workspace& wl, void* workspace, int32_t* dev_status, void* stream) {
  const int g = d->Hq / d->Hkv;
  const int rows_max = ls.rows_max;
  AttnParams p;
  p.B = d->B; p.kmax = d->kmax; p.Hq = d->Hq; p.Hkv = d->Hkv; p.D = d->D; p.Lcap = d->Lcap;
  p.nblk_cap = num_blocks(d->Lcap); p.g = g; p.rows_max = rows_max;
  p.g_magic = (g <= 64 && rows_max <= 2048) ? ((1u << 20) + (unsigned)g - 1u) / (unsigned)g : 0u;  // exact there: checked exhaustively
  p.nwaves = ls.nwaves;
  p.nshares = ls.nshares;
  p.fused_reduce = ls.fused_reduce;
  p.scale_log2 = d->scale * 1.4426950408889634f;
  p.Q = Q; p.Kc = Kcache; p.Vc = Vcache; p.Knew = K_new; p.Vnew = V_new;
  const PlanLayout pl = plan_layout(d->B, d->Hkv, ls.nshares);
  const char* pb = (const char*)plan;
  p.plan = (const PlanHeader*)pb;
  p.signature = plan_signature(d->B, d->kmax, d->Hkv, d->Lcap, ls.nshares, K_new ? kPlanAppend : 0);
  p.records = (const ShareRecord*)(pb + pl.records);
  p.overflow = (const Segment*)(pb + pl.overflow);
  p.seq_L = (const int32_t*)(pb + pl.seq_L);
  p.seq_nq = (const int32_t*)(pb + pl.seq_nq);
  p.unit_owners = (const int32_t*)(pb + pl.unit_owners);
  p.O = O; p.lse = lse; p.status = dev_status;
  p.counters = (int32_t*)workspace;
  p.part_acc = (float*)((char*)workspace + wl.part_acc);
  p.part_ml = (float*)((char*)workspace + wl.part_ml);

  hipStream_t s = (hipStream_t)stream;
  p.wpw = waves_per_workgroup(p.nwaves);
  const dim3 grid(p.nwaves / p.wpw), block(64 * p.wpw);
  if (d->dtype == BASS_DTYPE_FP32) {
    hipLaunchKernelGGL(verify_attn_fp32, grid, block, 0, s, p);
  } else if (ls.tiles) {
    const dim3 tgrid((unsigned)p.nshares), tblock(256);
    if (d->D == 128) {
      if (K_new) hipLaunchKernelGGL((verify_attn_tiles_bf16<128, true>), tgrid, tblock, 0, s, p);
      else hipLaunchKernelGGL((verify_attn_tiles_bf16<128, false>), tgrid, tblock, 0, s, p);
    } else {
      if (K_new) hipLaunchKernelGGL((verify_attn_tiles_bf16<64, true>), tgrid, tblock, 0, s, p);
      else hipLaunchKernelGGL((verify_attn_tiles_bf16<64, false>), tgrid, tblock, 0, s, p);
    }
  } else {
    const int nt = (rows_max + 15) / 16;
    // LDS slice per wavefront of a fused append: K and V rows of two units (bf16, or INT8 codes + scales)
    const size_t unit_lds = d->dtype == BASS_DTYPE_INT8KV ? (size_t)2 * d->kmax * d->D + 8 * d->kmax
                                                          : (size_t)2 * d->kmax * d->D * 2;
    const size_t lds = K_new ? (size_t)p.wpw * 2 * unit_lds : 0;
#define BASS_LAUNCH(DD, NN) hipLaunchKernelGGL((verify_attn_bf16<DD, NN>), grid, block, lds, s, p)
#define BASS_LAUNCH_I8(DD, NN) hipLaunchKernelGGL((verify_attn_bf16<DD, NN, true>), grid, block, lds, s, p)
    if (d->dtype == BASS_DTYPE_INT8KV) {
      if (d->D == 128) {
        if (nt == 1) BASS_LAUNCH_I8(128, 1); else if (nt == 2) BASS_LAUNCH_I8(128, 2);
        else if (nt == 3) BASS_LAUNCH_I8(128, 3); else BASS_LAUNCH_I8(128, 4);
      } else {
        if (nt == 1) BASS_LAUNCH_I8(64, 1); else if (nt == 2) BASS_LAUNCH_I8(64, 2);
        else if (nt == 3) BASS_LAUNCH_I8(64, 3); else BASS_LAUNCH_I8(64, 4);
      }
    } else if (d->D == 128) {  // bf16, one query tile (more tiles: the workgroup-level kernel above)
      BASS_LAUNCH(128, 1);
    } else {
      BASS_LAUNCH(64, 1);
    }
#undef BASS_LAUNCH_I8
#undef BASS_LAUNCH
  }
  if (launch_status() != BASS_OK) return BASS_ERR_HIP;
  if (!p.fused_reduce) {
    const long items = (long)d->B * d->Hkv * ((rows_max + 3) / 4);
    const dim3 rgrid((unsigned)((items + 3) / 4));
    if (d->D == 128) hipLaunchKernelGGL((reduce_partials<2, 128>), rgrid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL((reduce_partials<1, 64>), rgrid, dim3(256), 0, s, p);
  }
  return launch_status();
}

// Plan (into the workspace) and attention in one call.
static int plan_and_launch(const bass_attn_desc* d, const void* Q, const void* K_new, const void* V_new,
                           const void* Kcache, const void* Vcache, const int32_t* ctx_len, const int32_t* draft_len,
                           float* O, float* lse, void* workspace, size_t workspace_bytes, int32_t* dev_status,
                           void* stream, int span = 0) {
  int rc = check_desc(d);
  if (rc != BASS_OK) return rc;
  if (!ctx_len || !draft_len) return BASS_ERR_INVALID_ARG;
  const LaunchShape ls = launch_shape(d, K_new != nullptr);
  rc = check_attention_args(d, ls, Q, K_new, V_new, Kcache, Vcache, O, workspace);
  if (rc != BASS_OK) return rc;
  const Workspace wl = workspace_layout(d, kMaxWaves);
  if (workspace_bytes < wl.bytes) return BASS_ERR_WORKSPACE_TOO_SMALL;
  void* plan = (char*)workspace + wl.plan;
  rc = launch_plan(d, ls, span, ctx_len, draft_len, plan, dev_status, stream, nullptr);
  if (rc != BASS_OK) return rc;
  return launch_attention(d, ls, Q, K_new, V_new, Kcache, Vcache, plan, O, lse, wl, workspace, dev_status, stream);
}

}  // namespace bass

extern "C" int bass_verify_attention(const bass_attn_desc* d, const void* Q, const void* Kcache, const void* Vcache,
                                     const int32_t* ctx_len, const int32_t* draft_len, float* O, float* lse,
                                     void* workspace, size_t workspace_bytes, int32_t* dev_status, void* stream) {
  return bass::plan_and_launch(d, Q, nullptr, nullptr, Kcache, Vcache, ctx_len, draft_len, O, lse, workspace,
                               workspace_bytes, dev_status, stream);
}

extern "C" int bass_verify_attention_pad(const bass_attn_desc* d, const void* Q, const void* Kcache,
                                         const void* Vcache, const int32_t* ctx_len, const int32_t* draft_len,
                                         int32_t padded_len, float* O, float* lse, void* workspace,
                                         size_t workspace_bytes, int32_t* dev_status, void* stream) {
  if (padded_len < 0) return BASS_ERR_INVALID_ARG;
  return bass::plan_and_launch(d, Q, nullptr, nullptr, Kcache, Vcache, ctx_len, draft_len, O, lse, workspace,
                               workspace_bytes, dev_status, stream, padded_len);
}

extern "C" int bass_verify_attention_split(const bass_attn_desc* d, const void* Q, const void* Kcache,
                                           const void* Vcache, const int32_t* ctx_len, const int32_t* draft_len,
                                           float* O, float* lse, void* workspace, size_t workspace_bytes,
                                           int32_t* dev_status, void* stream) {
  const int rc = bass::check_desc(d);
  if (rc != BASS_OK) return rc;
  if (!Q || !Kcache || !Vcache || !ctx_len || !draft_len || !O || !workspace) return BASS_ERR_INVALID_ARG;
  if (workspace_bytes < bass::workspace_layout(d, bass::kMaxWaves).bytes) return BASS_ERR_WORKSPACE_TOO_SMALL;
  bass_attn_desc one = *d;
  one.B = 1;
  const size_t elt = d->dtype == BASS_DTYPE_FP32 ? 4 : 2;  // Q is bf16 with bf16 and with INT8 caches
  const size_t q_seq = (size_t)d->kmax * d->Hq * d->D;  // elements of Q (and O) per sequence
  const size_t cache_seq = bass_kv_cache_bytes(&one);
  for (int b = 0; b < d->B; ++b) {  // one plan and one launch per sequence; they share the workspace in stream order
    const int r = bass::plan_and_launch(&one, (const char*)Q + b * q_seq * elt, nullptr, nullptr,
                                        (const char*)Kcache + b * cache_seq, (const char*)Vcache + b * cache_seq,
                                        ctx_len + b, draft_len + b, O + b * q_seq,
                                        lse ? lse + (size_t)b * d->kmax * d->Hq : nullptr, workspace, workspace_bytes,
                                        dev_status, stream);
    if (r != BASS_OK) return r;
  }
  return BASS_OK;
}

extern "C" int bass_append_verify_attention(const bass_attn_desc* d, const void* Q, const void* K_new,
                                            const void* V_new, void* Kcache, void* Vcache, const int32_t* ctx_len,
                                            const int32_t* draft_len, float* O, float* lse, void* workspace,
                                            size_t workspace_bytes, int32_t* dev_status, void* stream) {
  if (!K_new || !V_new) return BASS_ERR_INVALID_ARG;
  if (d && d->dtype != BASS_DTYPE_FP32 && (int64_t)d->kmax * d->D > bass::kMaxStagedElems) {
    // more new rows than a wavefront stages in LDS: append with a launch of its own
    const int rc = bass_kv_append(d, Kcache, Vcache, K_new, V_new, ctx_len, draft_len, dev_status, stream);
    if (rc != BASS_OK) return rc;
    return bass::plan_and_launch(d, Q, nullptr, nullptr, Kcache, Vcache, ctx_len, draft_len, O, lse, workspace,
                                 workspace_bytes, dev_status, stream);
  }
  return bass::plan_and_launch(d, Q, K_new, V_new, Kcache, Vcache, ctx_len, draft_len, O, lse, workspace,
                               workspace_bytes, dev_status, stream);
}

// A verification step's attention with a plan made once for all of its layers (bass_attention_plan).
extern "C" int bass_verify_attention_planned(const bass_attn_desc* d, const void* Q, const void* K_new, const void* V_new,
                                             void* Kcache, void* Vcache, const void* plan, float* O, float* lse,
                                             void* workspace, size_t workspace_bytes, int32_t* dev_status,
                                             void* stream) {
  int rc = bass::check_desc(d);
  if (rc != BASS_OK) return rc;
  if (!plan || ((uintptr_t)plan & 15) != 0) return BASS_ERR_INVALID_ARG;
  const bass::LaunchShape ls = bass::launch_shape(d, K_new != nullptr);
  rc = bass::check_attention_args(d, ls, Q, K_new, V_new, Kcache, Vcache, O, workspace);
  if (rc != BASS_OK) return rc;
  const bass::Workspace wl = bass::workspace_layout(d, bass::kMaxWaves);
  if (workspace_bytes < wl.bytes) return BASS_ERR_WORKSPACE_TOO_SMALL;
  if (K_new && !ls.fused_append) {
    // more new rows than a wavefront stages in LDS: append with a launch of its own, at the (clamped)
    // lengths the plan holds
    const bass::PlanLayout pl = bass::plan_layout(d->B, d->Hkv, ls.nshares);
    const int32_t* L = (const int32_t*)((const char*)plan + pl.seq_L);
    const int32_t* nq = (const int32_t*)((const char*)plan + pl.seq_nq);
    rc = bass_kv_append(d, Kcache, Vcache, K_new, V_new, L, nq, dev_status, stream);
    if (rc != BASS_OK) return rc;
    return bass::launch_attention(d, ls, Q, nullptr, nullptr, Kcache, Vcache, plan, O, lse, wl, workspace, dev_status,
                                  stream);
  }
  return bass::launch_attention(d, ls, Q, K_new, V_new, Kcache, Vcache, plan, O, lse, wl, workspace, dev_status, stream);
}

// ---------------------------------------------------------------------------------------
// bass_verify_attention_noalloc: for callers that cannot allocate or own a workspace.  The arrival
// counters, the plan and the partial results live in a file-scope device array.  In host code the array's
// name is only a stand-in: its device address is asked for once per device (hipGetSymbolAddress, with that
// device current) and that pointer, never the name, is what launches receive.
// ---------------------------------------------------------------------------------------
constexpr size_t kScratchBytes = BASS_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace bass {

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];  // per device: each GPU holds its own copy of the array
static std::mutex g_scratch_mutex;

static int scratch_address(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return BASS_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return BASS_ERR_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return BASS_OK;
}

}  // namespace bass

extern "C" int bass_verify_attention_noalloc(const bass_attn_desc* d, const void* Q, const void* Kcache,
                                             const void* Vcache, const int32_t* ctx_len, const int32_t* draft_len,
                                             float* O, float* lse, int32_t* dev_status, void* stream) {
  int rc = bass::check_desc(d);
  if (rc != BASS_OK) return rc;
  if (!ctx_len || !draft_len) return BASS_ERR_INVALID_ARG;
  const bass::LaunchShape ls = bass::launch_shape(d, false);
  // laid out for the shares this launch really uses, not for the largest spread the tuning knob allows
  const bass::Workspace wl = bass::workspace_layout(d, ls.nshares);
  if (wl.bytes > kScratchBytes) return BASS_ERR_WORKSPACE_TOO_SMALL;
  void* ptr = nullptr;
  rc = bass::scratch_address(&ptr);
  if (rc != BASS_OK) return rc;
  rc = bass::check_attention_args(d, ls, Q, nullptr, nullptr, Kcache, Vcache, O, ptr);
  if (rc != BASS_OK) return rc;
  void* plan = (char*)ptr + wl.plan;
  // the array keeps the last call's contents: the planning launch also clears the arrival counters
  rc = bass::launch_plan(d, ls, 0, ctx_len, draft_len, plan, dev_status, stream, (int32_t*)ptr);
  if (rc != BASS_OK) return rc;
  return bass::launch_attention(d, ls, Q, nullptr, nullptr, Kcache, Vcache, plan, O, lse, wl, ptr, dev_status, stream);
}
