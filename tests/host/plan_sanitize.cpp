// Host build (g++ -fsanitize=address,undefined) of the work-division arithmetic that the planning kernel,
// the host planner and the attention kernels share (paper_2404_15778_amd/csrc/attn_plan.h, bass_common.h's
// layout maps): sweeps shapes, lengths and spreads and checks, with every array access under the
// sanitizers, that
//   - every real block of every (sequence, kv head) unit lies in exactly one share's segments,
//   - the share that Split::owner names for a share's first entry is that share,
//   - every share between a unit's first and last contributor holds at least one real block of it,
//   - partial slots (share + unit) never collide,
//   - the cache layout maps are bijections onto a block.
// Prints "ok <cases>" and exits 0, or reports the first violation and exits 1.
#include <cstdio>
#include <cstdlib>
#include <map>
#include <random>
#include <set>
#include <vector>

#include "attn_plan.h"

#include "bass_layout.h"

using namespace bass;

static int fail(const char* what, int a = 0, int b = 0, int c = 0) {
  printf("FAIL: %s (%d, %d, %d)\n", what, a, b, c);
  return 1;
}

static int check_case(const PlanShape& s, const std::vector<int32_t>& ctx, const std::vector<int32_t>& dl) {
  std::vector<int32_t> L(s.B), nq(s.B), inc(s.B);
  int carry = 0;
  for (int b = 0; b < s.B; ++b) {
    int l = ctx[b], n = dl[b];
    clamp_lengths(l, n, s.kmax, s.Lcap);
    if (n < 0 || n > s.kmax || l < 0 || l + n > s.Lcap) return fail("clamp", b, l, n);
    L[b] = l;
    nq[b] = n;
    carry += padded_blocks(s.pad, seq_blocks(s, l, n));
    inc[b] = carry;
  }
  const int total = carry * s.Hkv;
  const Split sp = plan_split(s, total);
  if (sp.first(s.nshares) != total) return fail("split does not cover the list", total);
  int longest = 0, shortest = 1 << 30, nonempty = 0;
  for (int w = 0; w < s.nshares && total > 0; ++w) {
    const int len = sp.first(w + 1) - sp.first(w);
    if (len < 0) return fail("shares not monotonic", w);
    if (len == 0) continue;
    ++nonempty;
    if (sp.owner(sp.first(w)) != w) return fail("owner(first(w)) != w", w);
    if (sp.owner(sp.first(w + 1) - 1) != w) return fail("owner(last(w)) != w", w);
    longest = len > longest ? len : longest;
    if (sp.first(w + 1) < total) shortest = len < shortest ? len : shortest;  // all but the last non-empty share
  }
  if (total > 0) {
    if (nonempty > 1 && longest - shortest > 1) return fail("uneven shares", longest, shortest);
    // no share is longer than an even division over the aimed-at number of shares would make it
    if (longest > (total + s.target - 1) / s.target) return fail("a share is longer than total / target", longest, total, s.target);
    if (s.target < s.nshares && nonempty > 1 && total >= 2 * s.nshares && longest != shortest)
      return fail("room for more shares, but they are not equally long", longest, shortest);
  }
  // coverage[unit][block] = number of segments that hold it; holders[unit] = shares with a segment of it
  std::vector<std::vector<int>> coverage((size_t)s.B * s.Hkv);
  std::vector<std::set<int>> holders((size_t)s.B * s.Hkv);
  std::vector<int32_t> owners((size_t)s.B * s.Hkv, -1);
  for (int b = 0; b < s.B; ++b)
    for (int h = 0; h < s.Hkv; ++h) coverage[(size_t)b * s.Hkv + h].assign(seq_blocks(s, L[b], nq[b]), 0);
  std::set<long> slots;
  int err = 0;
  for (int w = 0; w < s.nshares && total > 0; ++w) {
    int prev_unit = -1;
    plan_share(s, L.data(), nq.data(), inc.data(), w, [&](const Segment& g) {
      if (err) return;
      if (g.b < 0 || g.b >= s.B || g.kvh < 0 || g.kvh >= s.Hkv) { err = fail("unit out of range", w, g.b, g.kvh); return; }
      const int unit = g.b * s.Hkv + g.kvh;
      std::vector<int>& cov = coverage[unit];
      if (g.n < 1 || g.first < 0 || g.first + g.n > (int)cov.size()) { err = fail("blocks out of range", w, g.first, g.n); return; }
      if (g.first + g.n > num_blocks(s.Lcap)) { err = fail("beyond the cache", w, g.first, g.n); return; }
      if (g.L != L[g.b] || g.nq != nq[g.b]) { err = fail("lengths", w, g.L, g.nq); return; }
      if (((g.flags & kSegLast) != 0) != (g.first + g.n == (int)cov.size())) { err = fail("last flag", w, g.first, g.n); return; }
      if (unit <= prev_unit) { err = fail("units of a share not increasing", w, unit, prev_unit); return; }
      prev_unit = unit;
      for (int j = g.first; j < g.first + g.n; ++j) cov[j]++;
      holders[unit].insert(w);
      if (owners[unit] >= 0 && owners[unit] != g.owners) { err = fail("owners differ between segments", w, unit); return; }
      owners[unit] = g.owners;
      if (!slots.insert((long)w + unit).second) { err = fail("partial slot used twice", w, unit); return; }
    });
    if (err) return err;
  }
  for (size_t unit = 0; unit < coverage.size(); ++unit) {
    for (size_t j = 0; j < coverage[unit].size(); ++j)
      if (coverage[unit][j] != 1) return fail("block not covered exactly once", (int)unit, (int)j, coverage[unit][j]);
    if (coverage[unit].empty()) {
      if (!holders[unit].empty()) return fail("inactive unit has segments", (int)unit);
      continue;
    }
    const int lo = owners[unit] & 0xFFFF, hi = (owners[unit] >> 16) & 0xFFFF;
    if (lo > hi || hi >= s.nshares) return fail("owner range", (int)unit, lo, hi);
    if ((int)holders[unit].size() != hi - lo + 1) return fail("contributors are not all of w_lo..w_hi", (int)unit, lo, hi);
    if (*holders[unit].begin() != lo || *holders[unit].rbegin() != hi) return fail("contributors do not span w_lo..w_hi", (int)unit, lo, hi);
  }
  return 0;
}

static int check_layout(int D) {
  std::set<size_t> k, v, k8, v8;
  for (int t = 0; t < kBlockTokens; ++t)
    for (int d = 0; d < D; ++d) {
      k.insert(k_elem_offset(D, t, d));
      v.insert(v_elem_offset(D, t, d));
      k8.insert(i8_k_offset(D, t, d));
      v8.insert(i8_v_offset(D, t, d));
    }
  const size_t n = (size_t)kBlockTokens * D;
  if (k.size() != n || *k.rbegin() != n - 1) return fail("k_elem_offset is not a bijection", D);
  if (v.size() != n || *v.rbegin() != n - 1) return fail("v_elem_offset is not a bijection", D);
  if (k8.size() != n || *k8.rbegin() != n - 1) return fail("i8_k_offset is not a bijection", D);
  if (v8.size() != n || *v8.rbegin() != n - 1) return fail("i8_v_offset is not a bijection", D);
  if (i8_block_bytes(D) != n + 4 * kBlockTokens) return fail("i8 block size", D);
  // a K chunk of 8 (bf16) / 16 (int8) head elements of one token is contiguous; a V fragment of one
  // head element holds 8 tokens
  for (int t = 0; t < kBlockTokens; ++t)
    for (int d = 0; d < D; d += 8)
      for (int j = 1; j < 8; ++j)
        if (k_elem_offset(D, t, d + j) != k_elem_offset(D, t, d) + j) return fail("K chunk not contiguous", D, t, d);
  return 0;
}

int main(int argc, char** argv) {
  const int cases = argc > 1 ? atoi(argv[1]) : 3000;
  std::mt19937 rng(12345);
  auto uni = [&](int lo, int hi) { return (int)(lo + rng() % (unsigned)(hi - lo + 1)); };
  if (check_layout(64) || check_layout(128)) return 1;
  int done = 0;
  for (int it = 0; it < cases; ++it) {
    PlanShape s;
    s.B = it % 7 == 0 ? uni(60, 140) : uni(1, 12);
    s.Hkv = uni(1, it % 5 == 0 ? 32 : 6);
    s.kmax = uni(1, 16);
    s.Lcap = it % 3 == 0 ? uni(1, 200) : uni(200, 9000);
    const int nshares_choices[] = {16, 64, 100, 256, 448, 768, 1020, 1024, 2048, 8192};
    s.nshares = nshares_choices[uni(0, 9)];
    s.target = it % 2 == 0 ? s.nshares : imax(1, s.nshares * 3 / 4);
    s.pad = uni(0, kMaxPad);
    s.pad_before = uni(0, s.pad);
    s.span = it % 4 == 0 ? uni(0, s.Lcap + 50) : 0;
    std::vector<int32_t> ctx(s.B), dl(s.B);
    for (int b = 0; b < s.B; ++b) {
      const int mode = uni(0, 9);
      ctx[b] = mode == 0 ? 0 : mode == 1 ? s.Lcap : mode == 2 ? uni(-5, s.Lcap + 40) : uni(0, s.Lcap);
      dl[b] = mode == 3 ? 0 : mode == 4 ? uni(-2, s.kmax + 3) : uni(1, s.kmax);
      if (it % 11 == 0) ctx[b] = uni(0, imin(s.Lcap, 40));  // many tiny units
    }
    if (check_case(s, ctx, dl)) {
      printf("case %d: B=%d Hkv=%d kmax=%d Lcap=%d nshares=%d target=%d pad=%d pad_before=%d span=%d\n", it, s.B, s.Hkv, s.kmax,
             s.Lcap, s.nshares, s.target, s.pad, s.pad_before, s.span);
      return 1;
    }
    ++done;
  }
  printf("ok %d\n", done);
  return 0;
}
