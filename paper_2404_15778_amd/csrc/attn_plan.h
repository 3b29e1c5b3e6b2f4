// Work plan of the ragged verify attention: which cache blocks every wavefront (or workgroup) of the
// attention launch streams, and who merges what.  Host- and device-callable; no HIP header is needed,
// so the same arithmetic is compiled into the planning kernel, into the host-side planner
// (bass_attention_plan_host) and into the CPU tests.
//
// BASS paper, Section 3.2: attention shares no reads between sequences, every sequence has its own
// length, and padding wastes work.  All (sequence, kv head) units are therefore cut into 32-token cache
// blocks and laid end to end; that flattened list is divided evenly over a fixed number of shares (one
// per wavefront, or per workgroup in the grouped-query kernel).  All attention layers of a verification
// step see the same lengths, so the division is computed once per step and every layer's launch reads
// its share from a record.
#pragma once
#include <stddef.h>
#include <stdint.h>

#if defined(__HIPCC__)
#define BASS_HD __host__ __device__
#else
#define BASS_HD
#endif

namespace bass {

constexpr int kBlockTokens = 32;  // tokens per cache block (one PV contraction step of the bf16 MFMA)
constexpr int kMaxWaves = 8192;   // upper bound of the attention work spread (sizes plans and workspaces)
constexpr int kMaxPad = 8;        // upper bound of the virtual blocks per unit

BASS_HD inline int imin(int a, int b) { return a < b ? a : b; }
BASS_HD inline int imax(int a, int b) { return a > b ? a : b; }

BASS_HD inline int num_blocks(int tokens) { return (tokens + kBlockTokens - 1) / kBlockTokens; }

// Per-sequence lengths with the clamping the header promises.  L = cached tokens before the step,
// nq = query tokens; on return 0 <= nq <= kmax, 0 <= L, L + nq <= Lcap.
BASS_HD inline bool clamp_lengths(int& L, int& nq, int kmax, int Lcap) {
  bool bad = false;
  if (nq < 0) { nq = 0; bad = true; }
  if (nq > kmax) { nq = kmax; bad = true; }
  if (nq > Lcap) { nq = Lcap; bad = true; }
  if (L < 0) { L = 0; bad = true; }
  if (L + nq > Lcap) { L = Lcap - nq; bad = true; }
  return bad;
}

// What the division depends on besides the lengths.
struct PlanShape {
  int32_t B, kmax, Hkv, Lcap;
  int32_t nshares;     // stretches the launch has room for (one record each)
  int32_t target;      // stretches aimed at (<= nshares); see plan_split
  int32_t pad;         // virtual blocks of every unit in the flattened list
  int32_t pad_before;  // how many of them sit in front of the unit's last real block
  int32_t span;        // BASS-PAD variant: every active sequence is processed over at least this many cache
                       // positions (0: over its own length); the positions beyond its length are masked
};

// Real blocks of a sequence (per kv head) after clamping; 0 for an inactive sequence.
BASS_HD inline int seq_blocks(const PlanShape& s, int L, int nq) {
  if (nq <= 0) return 0;
  return num_blocks(imax(L + nq, imin(s.span, s.Lcap)));
}

// Length of a unit in the flattened list = its real blocks plus `pad` virtual ones.  A virtual block is
// no work; it stands for the fixed cost of the wavefront that handles the unit's last blocks (the masked
// block steps, the rows of a fused append), so that this wavefront is handed correspondingly fewer real
// blocks and finishes with the others.
BASS_HD inline int padded_blocks(int pad, int nblk) { return nblk > 0 ? nblk + pad : 0; }

// Where a unit's virtual blocks sit.  With all of them behind the last real block, the wavefront that
// holds that block gets between none and all of the credit, depending on where the even cut falls.  With
// pb of them in front of the last real block and the others behind it, it gets at least min(pb, pad - pb).
// A unit's entries are then: real blocks 0 .. nblk-2, pb virtual ones, the last real block, pad - pb
// virtual ones.
BASS_HD inline int real_below(int t, int nblk, int pb) {  // real blocks at entries below t, 0 <= t <= nblk + pad
  return imin(t, nblk - 1) + (t > nblk - 1 + pb ? 1 : 0);
}
BASS_HD inline int entry_of(int j, int nblk, int pb) { return j < nblk - 1 ? j : j + pb; }  // entry of real block j

// Division of the flattened list into consecutive stretches: shares 0 .. rem-1 take per + 1 entries, the
// following ones per, until the list ends (shares beyond that are empty).
struct Split {
  int per, rem, total;
  BASS_HD int first(int w) const { return imin(w * per + imin(w, rem), total); }  // first entry of share w
  BASS_HD int owner(int x) const {                                                // share that holds entry x
    const int big = rem * (per + 1);
    return x < big ? x / (per + 1) : rem + (x - big) / imax(per, 1);
  }
};
// Even division over exactly n shares: they differ by at most one entry.
BASS_HD inline Split make_split(int total, int n) { return Split{total / n, total % n, total}; }

// The division a plan uses.  A launch lasts as long as its longest share, and with an even division over
// `target` shares most of them are one entry longer than total / target.  If the launch has room for more
// shares than it aims at (nshares > target), all shares get floor(total / target) entries instead and there
// are correspondingly more of them (at most nshares: the share length grows until they fit); the last one
// takes what is left, the launch's remaining wavefronts stay idle.
BASS_HD inline Split plan_split(const PlanShape& s, int total) {
  if (s.target >= s.nshares || total <= 0) return make_split(total, s.nshares);
  int per = imax(1, total / s.target);
  while ((total + per - 1) / per > s.nshares) ++per;
  return Split{per, 0, total};
}

// pb in effect: the split placement is switched off when shares are not longer than a unit's pad, so that
// no share can lie between two real blocks of a unit without holding one (every share between a unit's
// first and last contributor then contributes).
BASS_HD inline int pad_before_in_effect(const PlanShape& s, const Split& sp) { return sp.per > s.pad ? s.pad_before : 0; }

// One stretch of one unit inside one share: real blocks first .. first + n - 1 of (sequence b, kv head kvh).
struct Segment {
  int32_t b, kvh;
  int32_t L, nq;     // the sequence's clamped lengths
  int32_t first, n;  // real blocks of the unit this share streams
  int32_t owners;    // w_lo | w_hi << 16: the shares that contribute to the unit (all of w_lo .. w_hi do)
  int32_t flags;     // kSegLast: the stretch holds the unit's last real block
};
constexpr int32_t kSegLast = 1;

BASS_HD inline int seg_w_lo(const Segment& s) { return s.owners & 0xFFFF; }
BASS_HD inline int seg_w_hi(const Segment& s) { return (s.owners >> 16) & 0xFFFF; }

// What a share's wavefront reads first: its first two segments, how many it has, and where the others are.
struct ShareRecord {
  Segment seg[2];
  int32_t nseg;       // segments of this share
  int32_t overflow;   // index of segment 2 in the overflow list (segments 2 .. nseg-1 are consecutive there); it is
                      // share + unit index of that segment, which keeps the runs of different shares apart
  int32_t signature;  // plan_signature() of the plan: what a launch checks before it trusts the record
  int32_t flags;      // kRecAnyInactive (the same in every record)
};
constexpr int32_t kRecAnyInactive = 1;  // some sequence has no query token: its output rows still have to be cleared

// What a launch and its plan must agree on, folded into one word that every record carries (a launch then
// needs no second read to know that the record was made for it).  Never 0: cleared memory does not match.
BASS_HD inline int32_t plan_signature(int B, int kmax, int Hkv, int Lcap, int nshares, int flags) {
  const int32_t v[6] = {B, kmax, Hkv, Lcap, nshares, flags};
  uint32_t h = 2166136261u;
  for (int i = 0; i < 6; ++i) h = (h ^ (uint32_t)v[i]) * 16777619u;
  return (int32_t)(h | 1u);
}

constexpr int32_t kPlanMagic = 0x42415331;  // "BAS1"
constexpr int32_t kPlanAppend = 1;          // PlanHeader::flags: made for a launch that appends the step's rows

struct PlanHeader {
  int32_t magic;
  int32_t B, kmax, Hkv, Lcap;
  int32_t nshares, pad, pad_before, span;
  int32_t flags;
  int32_t total;         // entries of the flattened list (all kv heads)
  int32_t any_inactive;  // some sequence has no query token (its output rows still have to be cleared)
  int32_t any_clamped;   // some length was out of range
  int32_t reserved[3];
};

// Layout of a plan in memory (byte offsets; every part 16-byte aligned):
//   header | records [nshares] | overflow segments [nshares + B*Hkv] | seq L [B] | seq nq [B] |
//   inclusive prefix of padded blocks per sequence [B] | owners of every unit [B*Hkv]
struct PlanLayout {
  size_t records, overflow, seq_L, seq_nq, seq_inc, unit_owners, bytes;
};

BASS_HD inline size_t align16(size_t v) { return (v + 15) & ~(size_t)15; }

BASS_HD inline PlanLayout plan_layout(int B, int Hkv, int nshares) {
  PlanLayout l;
  l.records = align16(sizeof(PlanHeader));
  l.overflow = l.records + (size_t)nshares * sizeof(ShareRecord);
  l.seq_L = l.overflow + ((size_t)nshares + (size_t)B * Hkv) * sizeof(Segment);
  l.seq_nq = align16(l.seq_L + (size_t)B * 4);
  l.seq_inc = align16(l.seq_nq + (size_t)B * 4);
  l.unit_owners = align16(l.seq_inc + (size_t)B * 4);
  l.bytes = align16(l.unit_owners + (size_t)B * Hkv * 4);
  return l;
}

// Sequence that holds flattened entry x: the first b with inc[b] * Hkv > x (inc: inclusive prefix of the
// padded block counts; 0 <= x < inc[B-1] * Hkv).
BASS_HD inline int seq_of_entry(const int32_t* inc, int B, int Hkv, int x) {
  int lo = 0, hi = B - 1;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if ((int64_t)inc[mid] * Hkv > (int64_t)x) hi = mid; else lo = mid + 1;
  }
  return lo;
}

BASS_HD inline int32_t unit_owners(const Split& sp, int begin, int nblk, int pb) {
  const int lo = sp.owner(begin + entry_of(0, nblk, pb));
  const int hi = sp.owner(begin + entry_of(nblk - 1, nblk, pb));
  return (int32_t)(lo | (hi << 16));
}

// The segments of share w, in list order; emit(segment) is called for each and their number returned.
// Stretches that hold virtual blocks only produce no segment.
template <class Emit>
BASS_HD inline int plan_share(const PlanShape& s, const int32_t* seq_L, const int32_t* seq_nq, const int32_t* inc, int w,
                              Emit&& emit) {
  const int total = inc[s.B - 1] * s.Hkv;
  const Split sp = plan_split(s, total);
  const int pb = pad_before_in_effect(s, sp);
  int x = sp.first(w);
  const int x_end = sp.first(w + 1);
  int count = 0;
  while (x < x_end) {
    const int b = seq_of_entry(inc, s.B, s.Hkv, x);
    const int npad = inc[b] - (b > 0 ? inc[b - 1] : 0);  // > 0: the entry exists
    const int pre = inc[b] - npad;
    const int kvh = (x - pre * s.Hkv) / npad;
    const int begin = pre * s.Hkv + kvh * npad;
    const int nblk = npad - s.pad;
    const int span = imin(x_end, begin + npad) - x;  // our stretch of the unit, virtual blocks included
    const int first = real_below(x - begin, nblk, pb);
    const int n = real_below(x - begin + span, nblk, pb) - first;
    if (n > 0) {
      Segment g;
      g.b = b;
      g.kvh = kvh;
      g.L = seq_L[b];
      g.nq = seq_nq[b];
      g.first = first;
      g.n = n;
      g.owners = unit_owners(sp, begin, nblk, pb);
      g.flags = first + n == nblk ? kSegLast : 0;
      emit(g);
      ++count;
    }
    x += span;
  }
  return count;
}

}  // namespace bass
