// Planning of a verification step's attention launches: bass_attention_plan (one small launch),
// bass_attention_plan_host (the same arithmetic on the host), bass_attention_plan_bytes.
//
// BASS paper, Section 3.2: every sequence of the batch has its own length and proceeds at its own pace;
// the lengths are the same for all attention layers of a verification step.  The division of the ragged
// work over the wavefronts of the attention launch (attn_plan.h) is therefore computed once per step, here,
// and each layer's launch reads its share from a record instead of recomputing it.
#include <cstring>

#include "bass_common.h"

namespace bass {

// Planning kernel.  Phase 1: clamp the lengths, count blocks, inclusive prefix over the sequences.  Phase 2: one
// thread per share walks its stretch of the block list and writes the record.  Phase 3: the contributors of
// every unit, for the merge launch.  Batches of up to kPlanSeqs sequences keep phase 1's results in LDS, every
// workgroup computes them for itself (a few hundred instructions) and the shares are spread over several
// workgroups, i.e. compute units: the walk is serial integer arithmetic with divisions, and one compute unit
// needs 10 us for 768 shares.  Larger batches are planned by a single workgroup through global memory.
constexpr int kPlanThreads = 256;
constexpr int kPlanSeqs = 1024;

// Inclusive prefix sum over the workgroup's kPlanThreads values and their total; all threads call.
__device__ inline int block_incl_scan(int v, int* lds, int tid, int& total) {
  const int lane = tid & 63, wv = tid >> 6;
  int x = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int t = __shfl_up(x, o);
    if (lane >= o) x += t;
  }
  if (lane == 63) lds[wv] = x;
  __syncthreads();
  int base = 0;
  total = 0;
  for (int i = 0; i < kPlanThreads / 64; ++i) {
    const int t = lds[i];
    if (i < wv) base += t;
    total += t;
  }
  __syncthreads();  // lds may be written again
  return x + base;
}

// Writes the segments of share w: the first two into its record, the others into the overflow list from entry
// w + (unit of the third segment) on.  These runs cannot overlap: the units of a share are distinct and
// increasing, and the next share starts at a unit that is not smaller than this share's last one.
struct RecordWriter {
  ShareRecord* rec;
  Segment* overflow;
  int w, Hkv, n, base;
  BASS_HD void operator()(const Segment& g) {
    if (n < 2) {
      rec->seg[n] = g;
    } else {
      if (n == 2) base = w + g.b * Hkv + g.kvh;
      overflow[base + n - 2] = g;
    }
    ++n;
  }
};

BASS_HD inline void clear_record(ShareRecord* r) {
  int32_t* w = (int32_t*)r;
  for (size_t i = 0; i < sizeof(ShareRecord) / 4; ++i) w[i] = 0;
}

BASS_HD inline void write_record(const PlanShape& s, const int32_t* seq_L, const int32_t* seq_nq, const int32_t* inc, int total,
                                 int w, int32_t signature, bool any_inactive, ShareRecord* records, Segment* overflow) {
  clear_record(&records[w]);
  RecordWriter wr{&records[w], overflow, w, s.Hkv, 0, 0};
  if (total > 0) plan_share(s, seq_L, seq_nq, inc, w, wr);
  records[w].nseg = wr.n;
  records[w].overflow = wr.base;
  records[w].signature = signature;
  records[w].flags = any_inactive ? kRecAnyInactive : 0;
}

BASS_HD inline int32_t owners_of_unit(const PlanShape& s, const Split& sp, int pb, const int32_t* inc, int unit) {
  const int b = unit / s.Hkv, kvh = unit - b * s.Hkv;
  const int npad = inc[b] - (b > 0 ? inc[b - 1] : 0);
  return npad > 0 ? unit_owners(sp, (inc[b] - npad) * s.Hkv + kvh * npad, npad - s.pad, pb) : 0;
}

BASS_HD inline PlanHeader make_header(const PlanShape& s, int flags, int total, bool any_inactive, bool any_clamped) {
  PlanHeader h;
  h.magic = kPlanMagic;
  h.B = s.B; h.kmax = s.kmax; h.Hkv = s.Hkv; h.Lcap = s.Lcap;
  h.nshares = s.nshares; h.pad = s.pad; h.pad_before = s.pad_before; h.span = s.span;
  h.flags = flags;
  h.total = total;
  h.any_inactive = any_inactive ? 1 : 0;
  h.any_clamped = any_clamped ? 1 : 0;
  h.reserved[0] = h.reserved[1] = h.reserved[2] = 0;
  return h;
}

// clear_counters (optional): the arrival counters of the attention launch that follows, B * Hkv words,
// cleared here for callers whose workspace is not known to be clean.
__global__ __launch_bounds__(kPlanThreads) void attention_plan_kernel(PlanShape s, int flags, const int32_t* ctx_len,
                                                                      const int32_t* draft_len, char* plan, int32_t* status,
                                                                      int32_t* clear_counters) {
  __shared__ int lds[kPlanThreads / 64];
  __shared__ int32_t lds_L[kPlanSeqs], lds_nq[kPlanSeqs], lds_inc[kPlanSeqs];
  const int tid = threadIdx.x;
  const int gtid = blockIdx.x * kPlanThreads + tid, gthreads = gridDim.x * kPlanThreads;
  const bool first = blockIdx.x == 0;
  const bool in_lds = s.B <= kPlanSeqs;  // else: one workgroup (the host launches it so), results through global memory
  const PlanLayout lay = plan_layout(s.B, s.Hkv, s.nshares);
  int32_t* seq_L = (int32_t*)(plan + lay.seq_L);
  int32_t* seq_nq = (int32_t*)(plan + lay.seq_nq);
  int32_t* inc = (int32_t*)(plan + lay.seq_inc);
  ShareRecord* records = (ShareRecord*)(plan + lay.records);
  Segment* overflow = (Segment*)(plan + lay.overflow);
  int32_t* owners = (int32_t*)(plan + lay.unit_owners);

  if (clear_counters)
    for (int i = gtid; i < s.B * s.Hkv; i += gthreads) clear_counters[i] = 0;

  // phase 1 (every workgroup for itself; the first one also writes the plan's copy)
  int carry = 0;
  bool bad = false, inactive = false;
  for (int c0 = 0; c0 < s.B; c0 += kPlanThreads) {
    const int b = c0 + tid;
    int nb = 0, L = 0, nq = 0;
    if (b < s.B) {
      L = ctx_len[b];
      nq = draft_len[b];
      bad |= clamp_lengths(L, nq, s.kmax, s.Lcap);
      inactive |= nq == 0;
      nb = padded_blocks(s.pad, seq_blocks(s, L, nq));
    }
    int chunk_total;
    const int incl = carry + block_incl_scan(nb, lds, tid, chunk_total);
    if (b < s.B) {
      if (first) {
        seq_L[b] = L;
        seq_nq[b] = nq;
        inc[b] = incl;
      }
      if (in_lds) {
        lds_L[b] = L;
        lds_nq[b] = nq;
        lds_inc[b] = incl;
      }
    }
    carry += chunk_total;
  }
  const int any_bad = __syncthreads_or(bad ? 1 : 0);
  const int any_inactive = __syncthreads_or(inactive ? 1 : 0);  // also orders the writes above before the reads below
  const int total = carry * s.Hkv;
  if (first && tid == 0) {
    *(PlanHeader*)plan = make_header(s, flags, total, any_inactive != 0, any_bad != 0);
    if (any_bad && status) atomicOr(status, BASS_STATUS_LEN_CLAMPED);
  }
  const int32_t* rd_L = in_lds ? lds_L : seq_L;
  const int32_t* rd_nq = in_lds ? lds_nq : seq_nq;
  const int32_t* rd_inc = in_lds ? lds_inc : inc;

  // phase 2
  const int32_t signature = plan_signature(s.B, s.kmax, s.Hkv, s.Lcap, s.nshares, flags);
  for (int w = gtid; w < s.nshares; w += gthreads)
    write_record(s, rd_L, rd_nq, rd_inc, total, w, signature, any_inactive != 0, records, overflow);

  // phase 3
  const Split sp = plan_split(s, total);
  const int pb = pad_before_in_effect(s, sp);
  for (int unit = gtid; unit < s.B * s.Hkv; unit += gthreads) owners[unit] = total > 0 ? owners_of_unit(s, sp, pb, rd_inc, unit) : 0;
}

// The same plan, byte for byte, written by the host into host memory.
static bool plan_on_host(const PlanShape& s, int flags, const int32_t* ctx_len, const int32_t* draft_len, char* plan) {
  const PlanLayout lay = plan_layout(s.B, s.Hkv, s.nshares);
  int32_t* seq_L = (int32_t*)(plan + lay.seq_L);
  int32_t* seq_nq = (int32_t*)(plan + lay.seq_nq);
  int32_t* inc = (int32_t*)(plan + lay.seq_inc);
  ShareRecord* records = (ShareRecord*)(plan + lay.records);
  Segment* overflow = (Segment*)(plan + lay.overflow);
  int32_t* owners = (int32_t*)(plan + lay.unit_owners);
  bool bad = false, any_inactive = false;
  int carry = 0;
  for (int b = 0; b < s.B; ++b) {
    int L = ctx_len[b], nq = draft_len[b];
    bad |= clamp_lengths(L, nq, s.kmax, s.Lcap);
    any_inactive |= nq == 0;
    carry += padded_blocks(s.pad, seq_blocks(s, L, nq));
    seq_L[b] = L;
    seq_nq[b] = nq;
    inc[b] = carry;
  }
  const int total = carry * s.Hkv;
  *(PlanHeader*)plan = make_header(s, flags, total, any_inactive, bad);
  const int32_t signature = plan_signature(s.B, s.kmax, s.Hkv, s.Lcap, s.nshares, flags);
  for (int w = 0; w < s.nshares; ++w) write_record(s, seq_L, seq_nq, inc, total, w, signature, any_inactive, records, overflow);
  const Split sp = plan_split(s, total);
  const int pb = pad_before_in_effect(s, sp);
  for (int unit = 0; unit < s.B * s.Hkv; ++unit) owners[unit] = total > 0 ? owners_of_unit(s, sp, pb, inc, unit) : 0;
  return bad;
}

PlanShape plan_shape(const bass_attn_desc* d, const LaunchShape& ls, int span) {
  PlanShape s;
  s.B = d->B; s.kmax = d->kmax; s.Hkv = d->Hkv; s.Lcap = d->Lcap;
  s.nshares = ls.nshares; s.target = ls.target; s.pad = ls.pad; s.pad_before = ls.pad_before; s.span = span;
  return s;
}

size_t plan_bytes_max(const bass_attn_desc* d) { return plan_layout(d->B, d->Hkv, kMaxWaves).bytes; }

int launch_plan(const bass_attn_desc* d, const LaunchShape& ls, int span, const int32_t* ctx_len, const int32_t* draft_len,
                void* plan, int32_t* dev_status, void* stream, int32_t* clear_counters) {
  const PlanShape s = plan_shape(d, ls, span);
  const unsigned groups = s.B <= kPlanSeqs ? (unsigned)((s.nshares + kPlanThreads - 1) / kPlanThreads) : 1u;
  hipLaunchKernelGGL(attention_plan_kernel, dim3(groups), dim3(kPlanThreads), 0, (hipStream_t)stream, s,
                     ls.fused_append ? kPlanAppend : 0, ctx_len, draft_len, (char*)plan, dev_status, clear_counters);
  return launch_status();
}

}  // namespace bass

extern "C" size_t bass_attention_plan_bytes(const bass_attn_desc* d) {
  if (bass::check_desc(d) != BASS_OK) return 0;
  return bass::plan_bytes_max(d);
}

static int check_plan_args(const bass_attn_desc* d, const void* ctx_len, const void* draft_len, int32_t flags,
                           int32_t padded_len, const void* plan, size_t plan_bytes) {
  const int rc = bass::check_desc(d);
  if (rc != BASS_OK) return rc;
  if (!ctx_len || !draft_len || !plan || padded_len < 0 || (flags & ~BASS_PLAN_APPEND) != 0) return BASS_ERR_INVALID_ARG;
  if (((uintptr_t)plan & 15) != 0) return BASS_ERR_INVALID_ARG;
  if ((flags & BASS_PLAN_APPEND) && padded_len > 0) return BASS_ERR_INVALID_ARG;
  if (plan_bytes < bass::plan_bytes_max(d)) return BASS_ERR_WORKSPACE_TOO_SMALL;
  return BASS_OK;
}

extern "C" int bass_attention_plan(const bass_attn_desc* d, const int32_t* ctx_len, const int32_t* draft_len, int32_t flags,
                                   int32_t padded_len, void* plan, size_t plan_bytes, int32_t* dev_status, void* stream) {
  const int rc = check_plan_args(d, ctx_len, draft_len, flags, padded_len, plan, plan_bytes);
  if (rc != BASS_OK) return rc;
  const bass::LaunchShape ls = bass::launch_shape(d, (flags & BASS_PLAN_APPEND) != 0);
  return bass::launch_plan(d, ls, padded_len, ctx_len, draft_len, plan, dev_status, stream, nullptr);
}

extern "C" int bass_attention_plan_host(const bass_attn_desc* d, const int32_t* ctx_len, const int32_t* draft_len,
                                        int32_t flags, int32_t padded_len, void* plan, size_t plan_bytes,
                                        int32_t* host_status) {
  const int rc = check_plan_args(d, ctx_len, draft_len, flags, padded_len, plan, plan_bytes);
  if (rc != BASS_OK) return rc;
  const bass::LaunchShape ls = bass::launch_shape(d, (flags & BASS_PLAN_APPEND) != 0);
  const bass::PlanShape s = bass::plan_shape(d, ls, padded_len);
  memset(plan, 0, bass::plan_layout(s.B, s.Hkv, s.nshares).bytes);
  const bool bad = bass::plan_on_host(s, ls.fused_append ? bass::kPlanAppend : 0, ctx_len, draft_len, (char*)plan);
  if (bad && host_status) *host_status |= BASS_STATUS_LEN_CLAMPED;
  return BASS_OK;
}
